"""The optimizer step on the CPU over the two-tier cache: Adam states in a pinned
host cache and on the file tier, fetched and written back behind the update.

Run as `python -m paper_2511_14124_amd.opt_demo` on the GPU machine.  Per parameter
tensor of a Llama-shaped model there are three fp32 state tensors (master copy,
momentum, variance); step j of the sweep updates the three of parameter j with
PyTorch CPU ops, between the PRE and POST calls of `tc_migrate_step` (the paper's
optimizer states scheduling policy, Sec. 3.4.2: a share of the states lives in
CPU memory, the rest on NVMe; an updated state is evicted and the next absent
one prefetched while the CPU computes).  Three runs of the same sweep:

  resident   the cache holds every state (what the update alone costs),
  prefetch   the cache holds `--cache` of the states, Alg. 3-4 as they are,
  demand     the same cache without prefetching (the paper's base variant):
             every absent state is read when its step asks for it.

Prints one JSON line: time per sweep, the share of it the PRE calls spent
blocked, the miss rate (accesses that had to be fetched on demand), bytes read
and written, and whether sampled states equal a plain Adam on resident tensors
bit for bit.
"""

from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import tempfile
import time

import numpy as np

from .opt_states import RW, adam_


def parameter_elems(layers: int, hidden: int, ffn: int, vocab: int, shard_rows: int = 4096):
    h, f = hidden, ffn
    shards = [min(shard_rows, vocab - r) * h for r in range(0, vocab, shard_rows)]
    elems = list(shards)
    for _ in range(layers):
        elems += [h, h * h, h * h, h * h, h * h, h, h * f, h * f, f * h]
    return elems + [h] + shards


def plain_io_rate(T, path, stripes, bytes_each_way, chunk=8 << 20):
    """What this box's file system gives plain threads for the same job: one
    reader and one writer thread per stripe file, 8 MiB preadv / pwrite calls
    between the file and a pinned region, bytes_each_way read and as many
    written at the same time (buffered; the extents read were written by the
    runs before).  Returns GB/s, both directions together."""
    import threading
    n = max(1, stripes)
    per_file = min(bytes_each_way // n, os.path.getsize(path) // 2) // chunk * chunk
    if per_file == 0:
        return None
    region = T._PinnedRegion(2 * n * chunk)
    mem = (C.c_uint8 * region.nbytes).from_address(region.ptr)
    fds = [os.open(path if k == 0 else f"{path}.{k}", os.O_RDWR) for k in range(n)]
    errors = []

    def work(k, write):
        try:
            buf = memoryview(mem)[(2 * k + write) * chunk:(2 * k + write + 1) * chunk]
            base = per_file if write else 0
            for off in range(0, per_file, chunk):
                if write:
                    os.pwrite(fds[k], buf, base + off)
                else:
                    os.preadv(fds[k], [buf], base + off)
        except OSError as e:
            errors.append(e)

    threads = [threading.Thread(target=work, args=(k, w)) for k in range(n) for w in (0, 1)]
    t0 = time.perf_counter()
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    dt = time.perf_counter() - t0
    for fd in fds:
        os.close(fd)
    del mem
    region.free()
    return None if errors else 2 * n * per_file / dt / 1e9


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--layers", type=int, default=4)
    ap.add_argument("--hidden", type=int, default=2048)
    ap.add_argument("--ffn", type=int, default=5504)
    ap.add_argument("--vocab", type=int, default=32000)
    ap.add_argument("--cache", type=float, default=0.5, help="host cache as a fraction of the state bytes")
    ap.add_argument("--sweeps", type=int, default=3)
    ap.add_argument("--file", default=None, help="file of the slow tier (default: a temporary file)")
    ap.add_argument("--stripes", type=int, default=4)
    ap.add_argument("--direct", action="store_true", help="open the file tier with O_DIRECT (no page cache)")
    ap.add_argument("--threads", type=int, default=8,
                    help="PyTorch CPU threads (0: leave the default); the I/O workers need cores of their own")
    args = ap.parse_args(argv)

    import torch
    from . import binding as T
    T.load_library()
    if args.threads:
        torch.set_num_threads(args.threads)

    elems = parameter_elems(args.layers, args.hidden, args.ffn, args.vocab)
    n_p = len(elems)
    tensor_bytes = np.repeat(np.asarray(elems, dtype=np.uint64) * 4, 3)
    group = np.ones(3 * n_p, dtype=np.uint8)
    ev_step = np.repeat(np.arange(n_p, dtype=np.uint32), 3)
    ev_tensor = np.arange(3 * n_p, dtype=np.uint32)
    ev_rw = np.full(3 * n_p, RW, dtype=np.uint8)
    state_bytes = int(tensor_bytes.sum())
    rng = np.random.default_rng(0)
    grad = torch.from_numpy(rng.standard_normal(max(elems), dtype=np.float32) * 1e-2)
    tmp = torch.empty(max(elems), dtype=torch.float32)
    sampled = sorted({0, 1, n_p // 2, n_p - 2, n_p - 1})

    def initial(t):
        j, k = divmod(t, 3)
        if k:
            return np.zeros(elems[j], dtype=np.float32)
        return np.random.default_rng(1000 + j).standard_normal(elems[j], dtype=np.float32) * 0.02

    def view(ptr, n):
        buf = (C.c_float * n).from_address(ptr)
        return torch.from_numpy(np.ctypeslib.as_array(buf))

    def run(cache_frac, prefetch, path):
        tc = T.TensorCache()
        tc.profile_order(tensor_bytes, group, ev_step, ev_tensor, ev_rw)
        tc.plan_pools(int(state_bytes * cache_frac), (0, 0), 256, 0 if prefetch else T.NO_PREFETCH)
        tc.plan_schedule()
        tc.bind_torch(file_path=path, host_tier=True, stripes=args.stripes, direct=args.direct)
        tc.set_oplog(False, True)
        for t in range(3 * n_p):
            tc.load_tensor(t, initial(t).view(np.uint8))
        tc.synchronize()
        views = {}
        sweep_s, tail_s = [], []
        in_pre = in_update = in_post = 0.0
        for it in range(args.sweeps + 1):           # the first sweep warms up (kernel load, page faults): not counted
            if it == 1:
                s0 = tc.cache_stats()
                sweep_s, tail_s = [], []
                in_pre = in_update = in_post = 0.0
            t0 = time.perf_counter()
            for j in range(n_p):
                ids = (3 * j, 3 * j + 1, 3 * j + 2)
                ta = time.perf_counter()
                ptrs = tc.migrate_step(j, T.PRE, ids, (RW,) * 3, 0, want_ptrs=True)
                tb = time.perf_counter()
                pmv = []
                for a in ptrs:
                    if (a, elems[j]) not in views:
                        views[(a, elems[j])] = view(a, elems[j])
                    pmv.append(views[(a, elems[j])])
                p, m, v = pmv
                adam_(torch, p, m, v, grad[: elems[j]], tmp[: elems[j]], it + 1)
                tc_ = time.perf_counter()
                tc.migrate_step(j, T.POST, ids, (RW,) * 3, 0)
                td = time.perf_counter()
                in_pre += tb - ta
                in_update += tc_ - tb
                in_post += td - tc_
            t1 = time.perf_counter()
            tc.end_iteration(0)                     # restore: queued behind the sweep's writes, not waited for
            t2 = time.perf_counter()
            sweep_s.append(t1 - t0)
            tail_s.append(t2 - t1)
        t3 = time.perf_counter()
        tc.synchronize()
        drain_s = time.perf_counter() - t3
        s1 = tc.cache_stats()
        got = {j: [tc.read_tensor(3 * j + k).view(np.float32).copy() for k in range(3)] for j in sampled}
        plan = tc.plan
        d = {k: s1[k] - s0[k] for k in ("hits", "misses", "stall_ns", "waits_total", "waits_under_30us",
                                       "bytes_file_read", "bytes_file_write", "file_read_ns", "file_write_ns")}
        n = args.sweeps
        out = {
            "cache_GiB": float(plan.hbm_total) / 2**30,
            "ms_per_sweep": 1e3 * sum(sweep_s) / n,
            "ms_in_pre_calls": 1e3 * in_pre / n, "ms_in_update": 1e3 * in_update / n, "ms_in_post_calls": 1e3 * in_post / n,
            "ms_blocked_in_pre_per_sweep": d["stall_ns"] / n / 1e6,
            "waits_under_0.03ms": d["waits_under_30us"] / max(1, d["waits_total"]),
            "miss_rate": d["misses"] / max(1, d["hits"] + d["misses"]),
            "file_read_GiB_per_sweep": d["bytes_file_read"] / n / 2**30,
            "file_write_GiB_per_sweep": d["bytes_file_write"] / n / 2**30,
            "ms_end_iteration_call": 1e3 * sum(tail_s) / n,
            "ms_drain_after_last_sweep": 1e3 * drain_s,
        }
        tc.close()
        return out, got

    # what a plain Adam on resident tensors gives for the sampled parameters
    want = {}
    for j in sampled:
        p, m, v = [torch.from_numpy(initial(3 * j + k).copy()) for k in range(3)]
        for it in range(args.sweeps + 1):
            adam_(torch, p, m, v, grad[: elems[j]], tmp[: elems[j]], it + 1)
        want[j] = [p.numpy(), m.numpy(), v.numpy()]

    tmpdir = None
    path = args.file
    if path is None:
        tmpdir = tempfile.TemporaryDirectory(prefix="tc_opt_")
        path = os.path.join(tmpdir.name, "states.bin")
    def migration_only(path):
        """The prefetch variant's schedule with nothing between the hooks: what the scheduler
        and the I/O workers move per second when no update competes for the cores."""
        tc = T.TensorCache()
        tc.profile_order(tensor_bytes, group, ev_step, ev_tensor, ev_rw)
        tc.plan_pools(int(state_bytes * args.cache), (0, 0), 256, 0)
        tc.plan_schedule()
        tc.bind_torch(file_path=path, host_tier=True, stripes=args.stripes, direct=args.direct, staging_bytes=int(tensor_bytes.max()))
        tc.set_oplog(False, True)
        tc.fill_payload(1)
        steps = [[(3 * j, RW), (3 * j + 1, RW), (3 * j + 2, RW)] for j in range(n_p)]
        tc.replay_iteration_c(steps, 0)             # warm-up
        tc.synchronize()
        s0 = tc.cache_stats()
        t0 = time.perf_counter()
        for _ in range(args.sweeps):
            tc.replay_iteration_c(steps, 0)
        tc.synchronize()
        dt = time.perf_counter() - t0
        s1 = tc.cache_stats()
        moved = (s1["bytes_file_read"] - s0["bytes_file_read"]) + (s1["bytes_file_write"] - s0["bytes_file_write"])
        tc.close()
        return {"ms_per_sweep": 1e3 * dt / args.sweeps, "GBps_read_plus_written": moved / dt / 1e9,
                "GiB_per_sweep": moved / args.sweeps / 2**30}

    res = {}
    ok = True
    for name, frac, prefetch in (("resident", 1.0, True), ("prefetch", args.cache, True), ("demand", args.cache, False)):
        res[name], got = run(frac, prefetch, path)
        ok = ok and all(np.array_equal(got[j][k], want[j][k]) for j in sampled for k in range(3))
    res["migration_only"] = migration_only(path)
    ceiling = None if args.direct else plain_io_rate(
        T, path, args.stripes, int(res["migration_only"]["GiB_per_sweep"] * 2**30 / 2))
    res["plain_threads_GBps_read_plus_written"] = ceiling
    if ceiling:
        res["migration_only"]["share_of_plain_threads"] = res["migration_only"]["GBps_read_plus_written"] / ceiling
    out = {
        "states": {"parameters": int(sum(elems)), "tensors": 3 * n_p, "GiB": state_bytes / 2**30,
                   "layers": args.layers, "hidden": args.hidden, "ffn": args.ffn, "vocab": args.vocab},
        "cpu_threads": torch.get_num_threads(), "o_direct": bool(args.direct), "stripes": args.stripes,
        "sweeps_timed": args.sweeps, **res,
        "speedup_prefetch_over_demand": res["demand"]["ms_per_sweep"] / res["prefetch"]["ms_per_sweep"],
        "sampled_states_equal_plain_adam": bool(ok),
    }
    print(json.dumps(out))
    if tmpdir is not None:
        tmpdir.cleanup()
    return out


if __name__ == "__main__":
    main()
