"""Helpers that compare a replay through the C-ABI library with the oracle."""

import numpy as np

import paper_2511_14124_amd as T
import workloads as W
from oracle import tc_oracle as o


def oracle_log_array(r):
    a = np.zeros(len(r.log), dtype=T.OP)
    if len(r.log):
        cols = list(zip(*r.log))
        for name, col in zip(("iteration", "step", "phase", "op", "tensor", "src_tier", "src_slot",
                              "dst_tier", "dst_slot", "bytes"), cols):
            a[name] = col
    return a


def compare_logs(got, want):
    assert len(got) == len(want), (len(got), len(want))
    for name in T.OP.names:
        if not np.array_equal(got[name], want[name]):
            i = int(np.nonzero(got[name] != want[name])[0][0])
            raise AssertionError(f"op log differs at record {i} field {name}: got {got[i]} want {want[i]}")


def run_library(wl, *, payload=True, null_mover=False, file_path=None, staging_bytes=0, mover=None,
                busy=False, window=None, merge_bytes=None, dma_threshold=None, fill=False, direct=False,
                io_writers=None, stripes=1, io_chunk=None, ahead=None, tune=False, host_tier=False, dma_when_behind=False,
                stripe_paths=None, one_stream=False, gpu_deps=False):
    """Replays every iteration of wl through the library; returns the context.

    window None: one tc_migrate_step call per hook (the hook-driven interface);
    otherwise tc_replay_iteration with that many steps per decision launch.
    fill: the library's fill kernel writes the payload pattern instead of
    tc_load_tensor (for footprints too large to generate on the host).
    host_tier: the two-tier mode (the fast tier is pinned host memory).
    one_stream: the stand-in modules run on the migration stream itself."""
    import torch
    tc = T.TensorCache.from_workload(wl)
    tc.bind_torch(null_mover=null_mover, file_path=file_path, staging_bytes=staging_bytes, direct=direct,
                  stripes=stripes, host_tier=host_tier, stripe_paths=stripe_paths)
    if tune and not null_mover:
        tc.tune_mover()                            # as bench.py does: the workgroup count is measured
    if ahead is not None:
        tc.set_decide_ahead(ahead)
    if io_chunk is not None:
        tc.set_io_chunk(io_chunk)
    if io_writers is not None:                     # (writers, readers)
        tc.set_io_threads(*io_writers)
    if mover:
        tc.set_mover(*mover)
    if gpu_deps and not null_mover:            # True, or the bound of the waits in ms
        tc.set_gpu_dependencies(True, 0 if gpu_deps is True else int(gpu_deps))
    if merge_bytes is not None:
        tc.set_merge_bytes(merge_bytes)
    if dma_threshold is not None:
        tc.set_dma_threshold(dma_threshold)
        tc.set_dma_policy(dma_when_behind)
    if window is not None:
        tc.set_replay_window(window)
    if fill and not null_mover:
        tc.fill_payload(W.PAYLOAD_SEED)
    elif payload and not null_mover:
        for t in range(wl.n_tensors):
            tc.load_tensor(t, W.workload_payload(wl, t))
    cs = tc.mstream if one_stream else torch.cuda.Stream()
    for steps in wl.iterations:
        ns = wl.compute_ns if busy else None
        if window is None:
            tc.replay_iteration(steps, cs.cuda_stream, busy_ns=ns)
        else:
            tc.replay_iteration_c(steps, cs.cuda_stream, busy_ns=ns)
    tc.synchronize()
    torch.cuda.synchronize()
    return tc


def check_against_oracle(wl, tc, *, check_bytes=True, tensors=None):
    r = o.replay_workload(wl, pattern=W.payload_bytes)
    compare_logs(tc.dump_oplog(), oracle_log_array(r))
    st = tc.cache_stats()
    assert (st["hits"], st["misses"], st["fails"]) == (r.hits, r.misses, r.fails)
    assert (st["bytes_h2d"], st["bytes_d2h"], st["bytes_file_read"], st["bytes_file_write"]) == \
        (r.bytes_h2d, r.bytes_d2h, r.bytes_file_read, r.bytes_file_write)
    tier, gs, cs = tc.dump_state()
    assert tier.tolist() == r.cur and gs.tolist() == r.gslot and cs.tolist() == r.cslot
    assert st["cursor"] == r.cursor and st["iteration"] == r.iteration
    allocs = [e for e in r.log if e[3] == o.ALLOC]
    assert (st["n_alloc"], st["undefined_reads"]) == (len(allocs), r.undefined_reads)
    assert st["bytes_not_fetched"] == sum(r.bytes_of[e[4]] for e in allocs)
    if check_bytes:
        pay = lambda t: W.workload_payload(wl, t)
        for t in (range(wl.n_tensors) if tensors is None else tensors):
            want = r.expected_bytes(t, pay)
            if want is None:
                continue                # allocated without fetch and never written: its bytes are unspecified
            got = tc.read_tensor(t)
            assert np.array_equal(got, want), f"tensor {t} bytes differ"
    return r
