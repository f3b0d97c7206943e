"""Parity of the HIP path with the oracle, through the C-ABI library, on a real
MI355X: schedule (op log), slot assignment, hit/miss counts, byte counters,
final maps and every byte of every tensor."""

import os

import numpy as np
import pytest

import paper_2511_14124_amd as T
import workloads as W
from tests.parity import run_library, check_against_oracle, compare_logs, oracle_log_array

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")    # imported at collection: a fresh box pages it in slowly


def _tmpfile(tmp_path, name="tier.bin"):
    return os.path.join(str(tmp_path), name)


def test_worked_example_cpu_gpu():
    wl = W.example_cpu_gpu()
    tc = run_library(wl)
    r = check_against_oracle(wl, tc)
    assert r.misses == 0 and len(r.log) == 12
    tc.close()


def test_worked_example_cpu_gpu_nvme(tmp_path):
    wl = W.example_cpu_gpu_nvme()
    tc = run_library(wl, file_path=_tmpfile(tmp_path), staging_bytes=1 << 16)
    check_against_oracle(wl, tc)
    tc.close()
    # the same example with the two sizes its text implies (tensor 2 is the one spilled)
    wl = W.example_cpu_gpu_nvme_two_sizes()
    tc = run_library(wl, file_path=_tmpfile(tmp_path), staging_bytes=1 << 16)
    r = check_against_oracle(wl, tc)
    from oracle import tc_oracle as o
    assert [e[4] for e in r.log if e[3] == o.SPILL] == [1]
    tc.close()


@pytest.mark.parametrize("n,k", [(8, 3), (8, 1), (5, 5), (70, 9), (200, 130)])
def test_single_class(n, k, tmp_path):
    # sizes off the 256-byte stride leave fewer buffers than tensors: some land on the file tier
    wl = W.single_class_fwd_bwd(n, k, n - k, size=4096 + 16 * (n % 3), n_iterations=2, rw_bwd=W.RW)
    tc = run_library(wl, file_path=_tmpfile(tmp_path), staging_bytes=1 << 16)
    check_against_oracle(wl, tc)
    tc.close()


def _random(seed):
    # 120 tensors in ten (size, group) classes, odd sizes (100 B, 33000 B), write accesses,
    # several iterations; by seed: order drift, scarce host buffers (spills, write-backs,
    # restores) and, for the literal-Alg.-2 seeds, classes without any GPU buffer (failed
    # accesses).  Every seed migrates (150-450 ops in the oracle's log).
    return W.random_workload(seed, n_tensors=120, n_steps=80, max_per_step=3,
                             hbm_frac=(0.08 if seed % 2 else 0.2), perturb_one_in=(0 if seed % 2 else 7),
                             host_frac=(0.3 if seed % 3 else 1.2), literal=(seed % 4 == 3))


@pytest.mark.parametrize("seed", range(12))
def test_random_multi_class_traces_with_file_tier(seed, tmp_path):
    wl = _random(seed)
    tc = run_library(wl, file_path=_tmpfile(tmp_path), staging_bytes=1 << 20)
    r = check_against_oracle(wl, tc)
    assert len(r.log) > 100
    tc.close()


def test_many_tensors_per_step_and_tiny_staging(tmp_path):
    # 12 tensors per step and a bounce buffer of only two tensors: the dispatch
    # must split a hook call into several launches
    wl = W.random_workload(101, n_tensors=80, n_steps=40, max_per_step=12, sizes=(4096, 8192, 100),
                           host_frac=0.2, perturb_one_in=5)
    tc = run_library(wl, file_path=_tmpfile(tmp_path), staging_bytes=2 * 8192)
    check_against_oracle(wl, tc)
    tc.close()


@pytest.mark.parametrize("window", [None, 8])
def test_a_step_may_name_as_many_tensors_as_a_wavefront_has_lanes(window, tmp_path):
    # up to 64 tensors per hook call (an optimizer step over a whole layer's tensors at once),
    # hook by hook and in windows, with misses and the file tier; 65 are refused
    wl = W.random_workload(211, n_tensors=1200, n_steps=30, max_per_step=64, sizes=(4096, 8192, 100, 20000),
                           hbm_frac=0.0, host_frac=0.3, perturb_one_in=7)
    assert max(len(st) for it in wl.iterations for st in it) > 48
    tc = run_library(wl, file_path=_tmpfile(tmp_path), staging_bytes=1 << 20, window=window)
    r = check_against_oracle(wl, tc)
    assert r.misses > 0
    tc.close()


def test_gpt2_small_config_full_bytes():
    # configuration 1 at full size: 800 tensors, 1.85 GiB, fp16 N(0, 0.02) parameters
    wl = W.config(0)
    tc = run_library(wl, mover=(512, 65536))
    r = check_against_oracle(wl, tc)
    assert r.misses == 0
    tc.close()


def test_ragged_tiles_and_launch_shapes():
    # sizes that are not multiples of the chunk or of 16 bytes, several grid shapes
    wl = W.random_workload(7, n_tensors=30, n_steps=50, sizes=(70001, 262144 + 48, 1 << 20, 17), host_frac=1.5)
    for mover in ((1, 4096), (7, 8192), (512, 65536), (2048, 1 << 20)):
        tc = run_library(wl, mover=mover)
        check_against_oracle(wl, tc)
        tc.close()


@pytest.mark.parametrize("index", [2, 3, 4])
def test_large_configs_schedule_parity_without_moving_bytes(index):
    # configurations 3-5 at full size (100-485 GiB): decisions, slots and counters
    # are exact; bytes are not moved (the footprint exceeds what a test may pin)
    wl = W.config(index)
    tc = run_library(wl, null_mover=True)
    check_against_oracle(wl, tc, check_bytes=False)
    tc.close()


def test_modelled_compute_does_not_change_the_schedule():
    wl = W.config(0, layers=8)
    tc = run_library(wl, busy=True)
    check_against_oracle(wl, tc)
    tc.close()


def test_wait_time_measurement_does_not_change_the_schedule():
    # with the host timing every pre-hook's waits (and no stream-side waits) the log, the
    # state and the bytes stay those of the oracle; every listed tensor is measured once
    import torch as _torch
    wl = W.config(0, layers=8)
    tc = T.TensorCache.from_workload(wl)
    tc.bind_torch()
    for t in range(wl.n_tensors):
        tc.load_tensor(t, W.workload_payload(wl, t))
    cs = _torch.cuda.Stream()
    tc.replay_iteration_c(wl.iterations[0], cs.cuda_stream, busy_ns=wl.compute_ns, measure_stall=True)
    tc.synchronize()
    r = check_against_oracle(wl, tc)
    st = tc.cache_stats()
    assert st["waits_total"] == r.hits + r.misses - r.fails
    assert st["waits_under_30us"] <= st["waits_total"]
    tc.close()


# ---- the same schedule whatever the launch shape -----------------------------

@pytest.mark.parametrize("window", [1, 3, 64, 256])
def test_windowed_replay_equals_hook_by_hook(window, tmp_path):
    # tc_replay_iteration decides a window of steps per launch; log, state, counters
    # and bytes must be those of one tc_migrate_step call per hook
    for seed in (2, 7, 9):
        wl = _random(seed)
        tc = run_library(wl, file_path=_tmpfile(tmp_path, f"w{seed}.bin"), staging_bytes=1 << 20, window=window)
        check_against_oracle(wl, tc)
        tc.close()
    wl = W.config(0, layers=8)
    tc = run_library(wl, window=window)
    check_against_oracle(wl, tc)
    tc.close()


@pytest.mark.parametrize("merge_bytes", [0, 1 << 20, 1 << 30])
def test_merging_hook_calls_into_launches_keeps_every_byte(merge_bytes, tmp_path):
    wl = W.random_workload(11, n_tensors=120, n_steps=90, max_per_step=3, sizes=(70001, 262144 + 48, 1 << 20, 17, 4096),
                           hbm_frac=0.1, host_frac=0.5, perturb_one_in=9)
    tc = run_library(wl, file_path=_tmpfile(tmp_path), staging_bytes=4 << 20, merge_bytes=merge_bytes, window=16)
    check_against_oracle(wl, tc)
    tc.close()
    wl = W.config(0, layers=6)
    tc = run_library(wl, merge_bytes=merge_bytes)
    check_against_oracle(wl, tc)
    tc.close()


@pytest.mark.parametrize("window", [None, 16])
def test_modules_on_the_migration_stream_itself_keep_every_byte(window, tmp_path):
    # a caller may compute on the stream the copies run on (one queue, in order): no event is waited for
    # across streams then, and schedule and bytes are what they are with two streams
    wl = W.random_workload(23, n_tensors=120, n_steps=90, max_per_step=3, sizes=(70001, 262144 + 48, 1 << 20, 17, 4096),
                           hbm_frac=0.1, host_frac=0.5, perturb_one_in=9)
    tc = run_library(wl, file_path=_tmpfile(tmp_path), staging_bytes=4 << 20, window=window, one_stream=True, busy=True)
    check_against_oracle(wl, tc)
    tc.close()
    wl = W.config(0, layers=6)
    tc = run_library(wl, window=window, one_stream=True)
    check_against_oracle(wl, tc)
    tc.close()


@pytest.mark.parametrize("window", [None, 16])
def test_dependencies_resolved_on_the_gpu_keep_every_byte(window, tmp_path):
    # tc_set_gpu_dependencies: launches wait for their modules' signal themselves and modules wait for a launch's
    # done word through a small kernel, no event between the streams; schedule and bytes are the oracle's, with
    # modelled compute running beside the copies, with the file tier and misses, hook by hook and in windows
    wl = W.random_workload(29, n_tensors=120, n_steps=90, max_per_step=3, sizes=(70001, 262144 + 48, 1 << 20, 17, 4096),
                           hbm_frac=0.1, host_frac=0.5, perturb_one_in=9, n_iterations=3)
    tc = run_library(wl, file_path=_tmpfile(tmp_path), staging_bytes=4 << 20, window=window, gpu_deps=True, busy=True)
    check_against_oracle(wl, tc)
    tc.close()
    wl = W.config(0, layers=8)
    for merge in (0, 1 << 30):
        tc = run_library(wl, window=window, gpu_deps=True, merge_bytes=merge)
        check_against_oracle(wl, tc)
        tc.close()
    # with allocate-without-fetch (units that only take a tensor out of a buffer the module then fills)
    wl = W.config(0, layers=6)
    wl.alloc_write_only = True
    tc = run_library(wl, window=window, gpu_deps=True, busy=True)
    check_against_oracle(wl, tc)
    tc.close()


def test_a_wait_on_the_gpu_that_runs_out_is_reported_and_every_kernel_still_ends():
    # the waits on the GPU are bounded: with a bound of 1 ms and modules that run for 20 ms a launch gives up
    # waiting for the modules before it; it moves nothing, every later waiter gives up at once, every kernel
    # ends, and the library reports it at the next call (the bytes are then not to be trusted)
    wl = W.config(0, layers=6)
    tc = T.TensorCache.from_workload(wl)
    tc.bind_torch()
    tc.set_gpu_dependencies(True, 1)
    tc.fill_payload(W.PAYLOAD_SEED)
    cs = torch.cuda.Stream()
    busy = np.full(wl.n_steps, 20_000_000, dtype=np.uint64)
    with pytest.raises(T.TcError) as e:
        for _ in range(3):
            tc.replay_iteration(wl.iterations[0], cs.cuda_stream, busy_ns=busy)
        tc.synchronize()
    assert e.value.code == -5 and "gave up" in str(e.value)            # TC_E_HIP
    torch.cuda.synchronize()                                          # everything queued has ended
    tc.close()


@pytest.mark.parametrize("busy", [False, True], ids=["idle_compute", "busy_compute"])
def test_dma_copies_only_behind_a_compute_backlog_keep_every_byte(busy, tmp_path):
    # with the policy "when behind" the path a large tensor takes (DMA engines or the kernel)
    # changes from launch to launch with the state of the compute stream; schedule and bytes do not
    wl = _random(4)
    if busy:
        wl.compute_ns = np.full_like(wl.compute_ns, 200000)
    for window in (None, 16):
        tc = run_library(wl, file_path=_tmpfile(tmp_path, f"p{window}.bin"), staging_bytes=2 << 20, window=window,
                         dma_threshold=1 << 10, dma_when_behind=True, busy=busy)
        check_against_oracle(wl, tc)
        st = tc.cache_stats()
        assert busy or st["dma_copies"] == 0 or st["mover_launches"] > 0
        tc.close()


@pytest.mark.parametrize("threshold", [1 << 16, 1 << 20])
def test_dma_engine_path_keeps_every_byte(threshold, tmp_path):
    # tensors at or above the threshold leave through an HBM bounce block and two
    # hipMemcpyAsync side streams; smaller ones stay in the migration kernel
    wl = W.random_workload(13, n_tensors=120, n_steps=90, max_per_step=2, sizes=(70001, 262144 + 48, 1 << 20, 17, 4096),
                           hbm_frac=0.1, host_frac=0.6, perturb_one_in=8)
    tc = run_library(wl, file_path=_tmpfile(tmp_path), staging_bytes=4 << 20, dma_threshold=threshold)
    check_against_oracle(wl, tc)
    assert tc.cache_stats()["dma_copies"] > 0
    tc.close()
    wl = W.config(0, layers=6)
    tc = run_library(wl, dma_threshold=threshold, window=32)
    check_against_oracle(wl, tc)
    tc.close()


def test_gpt_1p3b_config_full_size_sampled_bytes():
    # configuration 2 at full size in the launch configuration bench.py times: 1544
    # tensors, 19.95 GiB (17 GiB pinned, 3 GiB HBM), windows of 64 steps, launches merged up
    # to 1 GiB, the measured number of workgroups on one XCD taking 16 KiB chunks.
    # Schedule, counters and final maps are compared in full; bytes on a sample of
    # tensors the oracle rebuilds one by one (smallest, largest, every kind, stamped ones).
    wl = W.config(1)
    tc = run_library(wl, fill=True, window=64, merge_bytes=1 << 30, tune=True)
    kinds = wl.tensor_kind
    order = np.argsort(wl.tensor_bytes, kind="stable")
    sample = set(order[:6].tolist()) | set(order[-6:].tolist())
    for k in range(6):
        ids = np.nonzero(kinds == k)[0]
        sample |= set(ids[:: max(1, len(ids) // 5)].tolist())
    r = check_against_oracle(wl, tc, tensors=sorted(sample))
    assert r.misses == 0 and any(r.stamps[t] for t in sample)
    tc.close()


@pytest.mark.parametrize("window", [None, 64], ids=["hook_by_hook", "windows"])
def test_gpt_1p3b_config_full_size_with_compute_beside_the_copies(window):
    # the same configuration with the modelled compute stretched to about the migration time
    # (both streams busy throughout, launches merged up to 64 MiB as in the bench's stall run):
    # the copies overlap the stand-in kernels that stamp the buffers, so a copy that started
    # before its buffer was done with, or a module that started before its copy had landed,
    # shows in the sampled bytes
    wl = W.config(1)
    wl.compute_ns = (wl.compute_ns.astype(np.float64) * (0.6e9 / float(wl.compute_ns.sum()))).astype(np.uint64)
    tc = run_library(wl, fill=True, window=window, merge_bytes=64 << 20, tune=True, busy=True)
    kinds = wl.tensor_kind
    order = np.argsort(wl.tensor_bytes, kind="stable")
    sample = set(order[:6].tolist()) | set(order[-6:].tolist())
    for k in range(6):
        ids = np.nonzero(kinds == k)[0]
        sample |= set(ids[:: max(1, len(ids) // 8)].tolist())
    r = check_against_oracle(wl, tc, tensors=sorted(sample))
    assert r.misses == 0 and any(r.stamps[t] for t in sample)
    tc.close()


def _sample(wl, r, per_kind=4, extremes=4):
    kinds = wl.tensor_kind
    order = np.argsort(wl.tensor_bytes, kind="stable")
    sample = set(order[:extremes].tolist()) | set(order[-extremes:].tolist())
    for k in range(6):
        ids = np.nonzero(kinds == k)[0]
        if len(ids):
            sample |= set(ids[:: max(1, len(ids) // per_kind)].tolist())
    # tensors that ended on every tier, and some that were written
    for tier in (0, 1, 2):
        on = [t for t in range(wl.n_tensors) if r.cur[t] == tier]
        sample |= set(on[:: max(1, len(on) // per_kind)])
    return sorted(sample)


def test_llama_7b_config_full_size_sampled_bytes():
    # configuration 3 at full size: 1525 tensors, 100.4 GiB (40 GiB HBM cache, 60.6 GiB pinned),
    # three iterations replayed from the profile of the first, 363 GiB moved each way
    wl = W.config(2)
    tc = run_library(wl, fill=True, window=64, merge_bytes=1 << 30, tune=True)
    from oracle import tc_oracle as o
    r0 = o.replay_workload(wl)
    r = check_against_oracle(wl, tc, tensors=_sample(wl, r0, per_kind=3, extremes=3))
    assert r.misses == 0 and r.iteration == 3
    tc.close()


@pytest.mark.parametrize("index", [3, 4])
def test_file_tier_configs_at_two_layers_full_bytes(index, tmp_path):
    # configurations 4 and 5 at their real tensor sizes (10 KiB norms to 270 / 455 MiB fp32
    # matrices) but two layers deep, so that pinned pools and the file tier fit the box:
    # optimizer states on the file tier (4), scarce host pools with spills and 1 % of the
    # accesses perturbed (5).  Schedule, counters and maps in full; bytes of every tensor
    # under 1 MiB and of a sample of the large ones over all kinds and final tiers.  Launch
    # configuration as bench.py times it: file tier striped over eight files, staging ring
    # sixteen largest tensors deep, 8 + 8 I/O threads, launches merged up to 1 GiB.
    wl = W.config(index, layers=2)
    big = int(wl.tensor_bytes.max())
    tc = run_library(wl, fill=True, window=64, merge_bytes=1 << 30, file_path=_tmpfile(tmp_path),
                     staging_bytes=16 * ((big + 4095) // 4096 * 4096), stripes=8, io_writers=(8, 8), tune=True)
    from oracle import tc_oracle as o
    r0 = o.replay_workload(wl)
    small = [t for t in range(wl.n_tensors) if wl.tensor_bytes[t] < (1 << 20)]
    r = check_against_oracle(wl, tc, tensors=sorted(set(small) | set(_sample(wl, r0, per_kind=3, extremes=2))))
    st = tc.cache_stats()
    assert st["bytes_file_read"] > 0 and st["bytes_file_write"] > 0
    if index == 4:
        assert r.misses > 0
    tc.close()


def test_pre_hook_returns_the_buffers_the_oracle_names():
    # dev_ptrs_out of every PRE call = HBM region + class offset + buffer * stride of the
    # oracle's (class, buffer) for that access; and the bytes found there are the tensor's
    from oracle import tc_oracle as o
    wl = W.random_workload(21, n_tensors=60, n_steps=50, max_per_step=3, hbm_frac=0.15, host_frac=1.5,
                           two_groups=True, perturb_one_in=6, n_iterations=1)
    st, te, rw, _ = wl.events()
    r = o.build(wl.tensor_bytes.tolist(), wl.tensor_group.tolist(), st, te, rw, wl.hbm_bytes, wl.host_bytes,
                wl.align, wl.literal_alg2)
    tc = T.TensorCache.from_workload(wl)
    tc.bind_torch()
    for t in range(wl.n_tensors):
        tc.load_tensor(t, W.workload_payload(wl, t))
    cs = torch.cuda.Stream()
    base = tc.hbm.data_ptr()
    for k, access in enumerate(wl.iterations[0]):
        ids = [t for (t, _a) in access]
        flags = [a for (_t, a) in access]
        ptrs = tc.migrate_step(k, T.PRE, ids, flags, cs.cuda_stream, want_ptrs=True)
        want = r.pre(k, access)
        for (t, _a), p, w in zip(access, ptrs, want):
            if w is None:
                assert p == 0
                continue
            s, slot = w
            assert p == base + int(tc.classes["hbm_off"][s]) + slot * int(tc.classes["stride"][s])
        # what a module would read through the pointer (after the stream wait the call queued)
        cs.synchronize()
        tc.synchronize()
        t0, p0 = ids[0], ptrs[0]
        if p0:
            n = int(wl.tensor_bytes[t0])
            off = p0 - base
            got = tc.hbm[off:off + n].cpu().numpy()
            stamps = [x for x in r.stamps[t0] if x != (r.iteration, k)]     # this step's stamp comes after PRE
            want_bytes = np.array(W.workload_payload(wl, t0), dtype=np.uint8, copy=True)
            for (it, step) in stamps:
                o.apply_stamp(want_bytes, o.stamp16(it, step, t0))
            assert np.array_equal(got, want_bytes), (k, t0)
        tc.emulate_compute(cs.cuda_stream)
        tc.migrate_step(k, T.POST, ids, flags, cs.cuda_stream)
        r.post(k, ids)
    tc.end_iteration(cs.cuda_stream)
    r.end_iteration()
    tc.synchronize()
    tier, gs, cslot = tc.dump_state()
    assert tier.tolist() == r.cur and gs.tolist() == r.gslot and cslot.tolist() == r.cslot
    tc.close()


@pytest.mark.parametrize("ahead", [0, 1, 3, 16, 256])
def test_deciding_ahead_of_the_hooks_changes_nothing(ahead, tmp_path):
    # tc_migrate_step decides windows of profiled steps ahead of the calls.  Calls that leave
    # the profile (one access in six perturbed), state dumps in the middle of an iteration
    # (after an odd number of calls, inside a window) and an iteration cut short all have to
    # put the tables back in step: state after every few calls, op log, counters and bytes
    # are the oracle's whatever the window.
    from oracle import tc_oracle as o
    wl = W.random_workload(33, n_tensors=90, n_steps=70, max_per_step=3, hbm_frac=0.12, host_frac=0.5,
                           perturb_one_in=6, n_iterations=3)
    st, te, rw, _ = wl.events()
    r = o.build(wl.tensor_bytes.tolist(), wl.tensor_group.tolist(), st, te, rw, wl.hbm_bytes, wl.host_bytes,
                wl.align, wl.literal_alg2, payload=lambda t: W.workload_payload(wl, t))
    tc = T.TensorCache.from_workload(wl)
    tc.bind_torch(file_path=_tmpfile(tmp_path), staging_bytes=1 << 20)
    tc.set_decide_ahead(ahead)
    for t in range(wl.n_tensors):
        tc.load_tensor(t, W.workload_payload(wl, t))
    cs = torch.cuda.Stream()

    def same_state():
        tier, gs, cslot = tc.dump_state()
        assert tier.tolist() == r.cur and gs.tolist() == r.gslot and cslot.tolist() == r.cslot

    for it, steps in enumerate(wl.iterations):
        last = len(steps) if it != 1 else len(steps) // 2          # the second iteration stops half way
        for k, access in enumerate(steps[:last]):
            ids = [t for (t, _a) in access]
            flags = [a for (_t, a) in access]
            tc.migrate_step(k, T.PRE, ids, flags, cs.cuda_stream)
            r.pre(k, access)
            if k % 7 == 3:
                same_state()                                       # between a step's two calls
            tc.emulate_compute(cs.cuda_stream)
            tc.migrate_step(k, T.POST, ids, flags, cs.cuda_stream)
            r.post(k, ids)
            if k % 11 == 5:
                same_state()
        tc.end_iteration(cs.cuda_stream)
        r.end_iteration()
        same_state()
    tc.synchronize()
    compare_logs(tc.dump_oplog(), oracle_log_array(r))
    stt = tc.cache_stats()
    assert (stt["hits"], stt["misses"], stt["fails"]) == (r.hits, r.misses, r.fails)
    assert r.misses > 0
    for t in range(wl.n_tensors):
        assert np.array_equal(tc.read_tensor(t), r.read_tensor(t)), t
    tc.close()


def test_tuning_the_mover_measures_on_empty_regions_only():
    # tc_tune_mover times exchanges between the bound regions: allowed while they hold nothing,
    # refused afterwards; whatever it picks, the replay that follows equals the oracle
    wl = W.config(0, layers=8)
    tc = T.TensorCache.from_workload(wl)
    tc.bind_torch()
    wg = tc.tune_mover()
    assert wg in (8, 10, 12, 14, 16, 20, 24)
    for t in range(wl.n_tensors):
        tc.load_tensor(t, W.workload_payload(wl, t))
    with pytest.raises(T.TcError) as e:
        tc.tune_mover()
    assert e.value.code == -2                       # TC_E_STATE
    cs = torch.cuda.Stream()
    for steps in wl.iterations:
        tc.replay_iteration_c(steps, cs.cuda_stream)
    tc.synchronize()
    check_against_oracle(wl, tc)
    tc.close()
    # regions too small to tell anything: the setting stays
    small = W.example_cpu_gpu()
    tc = T.TensorCache.from_workload(small)
    tc.bind_torch()
    assert tc.tune_mover() == 12
    tc.close()


@pytest.mark.parametrize("window", [None, 8])
def test_long_replay_wraps_the_operation_ring(window, tmp_path):
    # thirty iterations with one launch per hook call: well over a thousand copy operations, so the
    # ring of 1024 operation events is reused, the ticket counters alternate over a
    # thousand times and the file tier queues hundreds of requests; everything still equals the
    # oracle, byte for byte
    wl = W.random_workload(8, n_tensors=120, n_steps=80, max_per_step=3, hbm_frac=0.08, perturb_one_in=9,
                           host_frac=0.3, n_iterations=30)
    tc = run_library(wl, file_path=_tmpfile(tmp_path), staging_bytes=1 << 20, merge_bytes=0, window=window)
    r = check_against_oracle(wl, tc)
    st = tc.cache_stats()
    assert st["mover_launches"] > 1024 and r.bytes_file_write > 0          # more operations than the ring has events
    tc.close()


def _direct_ok(tmp_path):
    try:
        fd = os.open(os.path.join(str(tmp_path), "probe.bin"), os.O_RDWR | os.O_CREAT | os.O_DIRECT, 0o600)
    except OSError:
        return False
    os.close(fd)
    return True


@pytest.mark.parametrize("seed", [1, 4, 11])
def test_file_tier_through_o_direct(seed, tmp_path):
    # the same traces with a file opened O_DIRECT: odd sizes (100 B, 33000 B) force every
    # request through 4 KiB rounding, staging blocks and the bounce block
    if not _direct_ok(tmp_path):
        pytest.skip("the temporary directory's file system does not take O_DIRECT")
    wl = _random(seed)
    tc = run_library(wl, file_path=_tmpfile(tmp_path), staging_bytes=1 << 20, direct=True, window=(8 if seed == 4 else None))
    r = check_against_oracle(wl, tc)
    st = tc.cache_stats()
    assert st["bytes_file_read"] + st["bytes_file_write"] > 0
    assert (st["file_read_ns"] > 0) == (st["bytes_file_read"] > 0)
    tc.close()


@pytest.mark.parametrize("seed", [1, 2, 11])
def test_base_variant_without_prefetching(seed, tmp_path):
    # TC_NO_PREFETCH: post-hook calls move nothing, every non-resident access is a demand miss
    wl = _random(seed)
    wl.no_prefetch = True
    tc = run_library(wl, file_path=_tmpfile(tmp_path), staging_bytes=1 << 20, window=(None if seed == 1 else 16))
    r = check_against_oracle(wl, tc)
    assert r.misses > 0 and not any(e[2] == 1 for e in r.log)
    tc.close()
    wl = W.config(0, layers=6)
    wl.no_prefetch = True
    tc = run_library(wl, window=64)
    r = check_against_oracle(wl, tc)
    assert r.misses > 0
    st = tc.cache_stats()
    assert st["hbm_pool_bytes"] <= st["hbm_budget"] and st["host_pool_bytes"] <= st["host_budget"]
    tc.close()


@pytest.mark.parametrize("prefetch", [False, True], ids=["demand_fetch_only", "with_alg3"])
def test_smallest_first_placement_ablation(prefetch, tmp_path):
    # TC_SMALLEST_FIRST: GPU buffers to the smallest tensors first (the baseline placement of
    # Sec. 3.1 / 3.3.2); the same kernels replay whatever plan they are given
    wl = W.config(0, layers=6)
    wl.smallest_first, wl.no_prefetch = True, not prefetch
    tc = run_library(wl, window=64)
    r = check_against_oracle(wl, tc)
    assert (r.misses > 0) == (not prefetch)
    tc.close()
    wl = _random(3)
    wl.smallest_first, wl.no_prefetch = True, not prefetch
    tc = run_library(wl, file_path=_tmpfile(tmp_path), staging_bytes=1 << 20)
    check_against_oracle(wl, tc)
    tc.close()
    # the nine tensors of the hand-written pin, through the library
    sizes = [4096, 4096] + [1024] * 7
    steps = [[(t, W.R)] for t in range(9)] + [[(t, W.R)] for t in reversed(range(9))]
    wl = W.traces._simple("nine_two_large", sizes, [0] * 9, steps, hbm_bytes=2 * 4096 + 2 * 1024,
                          host_bytes=(1 << 20, 0), literal=False)
    wl.smallest_first, wl.no_prefetch = True, not prefetch
    tc = run_library(wl)
    r = check_against_oracle(wl, tc)
    if not prefetch:
        assert (r.hits, r.misses) == (14, 4)
    tc.close()


def test_allocate_without_fetch_hand_example_and_small_config():
    # TC_ALLOC_WRITE_ONLY: a tensor whose coming access only writes gets its buffer without a copy
    steps = [[(0, W.R)], [(1, W.R)], [(2, W.W)], [(3, W.R)]]
    wl = W.traces._simple("awf4", [512] * 4, [0] * 4, steps, hbm_bytes=1024, host_bytes=(1024, 0), literal=True)
    wl.alloc_write_only = True
    tc = run_library(wl)
    r = check_against_oracle(wl, tc)
    assert [o_[3] for o_ in r.log[:4]] == [2, 8, 2, 1] and tc.cache_stats()["bytes_h2d"] == 3 * 512
    assert np.array_equal(tc.read_tensor(2), W.payload_bytes(2, 512, 0x10000000 + 2))
    tc.close()
    for window in (None, 16):
        wl = W.config(0, layers=6)
        wl.alloc_write_only = True
        tc = run_library(wl, window=window)
        r = check_against_oracle(wl, tc)
        st = tc.cache_stats()
        assert st["n_alloc"] > 50 and st["undefined_reads"] == 0 and r.misses == 0
        tc.close()


@pytest.mark.parametrize("seed", range(8))
def test_allocate_without_fetch_on_random_traces_with_file_tier(seed, tmp_path):
    # order drift included (even seeds): a tensor allocated for a write that never comes stays
    # unspecified and is left out of the byte comparison; everything else must be exact
    wl = _random(seed)
    wl.alloc_write_only = True
    tc = run_library(wl, file_path=_tmpfile(tmp_path), staging_bytes=1 << 20, window=(None if seed % 4 else 8),
                     stripes=(2 if seed % 3 == 0 else 1))
    r = check_against_oracle(wl, tc)
    assert any(e[3] == 8 for e in r.log)
    tc.close()


def test_allocate_without_fetch_on_the_gpt_1p3b_config_sampled_bytes():
    # configuration 2 at full size in the launch configuration bench.py times: 18 % of the fetches
    # become allocations, the schedule is otherwise the plain one
    wl = W.config(1)
    wl.alloc_write_only = True
    tc = run_library(wl, fill=True, window=64, merge_bytes=1 << 30, tune=True)
    from oracle import tc_oracle as o
    r0 = o.replay_workload(wl, pattern=W.payload_bytes)
    r = check_against_oracle(wl, tc, tensors=_sample(wl, r0, per_kind=6, extremes=4))
    st = tc.cache_stats()
    assert r.misses == 0 and 0.17 < st["bytes_not_fetched"] / (st["bytes_not_fetched"] + st["bytes_h2d"]) < 0.21
    tc.close()


def test_allocate_without_fetch_in_the_two_tier_mode(tmp_path):
    # the optimizer-state sweep with its master copies only written (a variant of the sweep where the
    # update reads momentum and variance and rewrites the master copy whole)
    n = 12
    steps = [[(3 * j, W.W), (3 * j + 1, W.RW), (3 * j + 2, W.RW)] for j in range(n)]
    wl = W.traces._simple("sweep_w", [4096] * (3 * n), [1] * (3 * n), steps, hbm_bytes=5 * 3 * 4096, host_bytes=(0, 0),
                          literal=False, n_iterations=3)
    wl.alloc_write_only = True
    tc = run_library(wl, file_path=_tmpfile(tmp_path), staging_bytes=1 << 16, host_tier=True)
    r = check_against_oracle(wl, tc)
    assert any(e[3] == 8 for e in r.log) and r.misses == 0
    tc.close()


def test_op_log_can_be_cleared_and_switched_off():
    wl = W.single_class_fwd_bwd(8, 3, 5, n_iterations=3)
    tc = T.TensorCache.from_workload(wl)
    tc.bind_torch()
    cs = torch.cuda.Stream()
    tc.replay_iteration(wl.iterations[0], cs.cuda_stream)
    n1 = len(tc.dump_oplog())
    assert n1 == 20
    tc.set_oplog(enable=True, clear=True)
    tc.replay_iteration(wl.iterations[1], cs.cuda_stream)
    log = tc.dump_oplog()
    assert len(log) == n1 and set(log["iteration"].tolist()) == {1}
    tc.set_oplog(enable=False, clear=True)
    tc.replay_iteration_c(wl.iterations[2], cs.cuda_stream)
    assert len(tc.dump_oplog()) == 0 and sum(tc.cache_stats()["n_ops"]) == 3 * n1
    tc.close()


@pytest.mark.parametrize("writers", [(0, 0), (1, 0), (0, 1), (1, 1), (2, 3), (5, 2)])
@pytest.mark.parametrize("staging", ["tight", "deep"])
def test_write_behind_keeps_every_byte(writers, staging, tmp_path):
    # file reads and writes run behind the hook thread: whatever the number of writer and
    # reader threads and however shallow the staging ring (twice the largest tensor = one
    # block at a time), the schedule and every byte are those of the oracle
    for seed in (4, 7):
        wl = _random(seed)
        big = int(wl.tensor_bytes.max())
        half = (big + 255) // 256 * 256
        tc = run_library(wl, file_path=_tmpfile(tmp_path, f"wb{seed}.bin"),
                         staging_bytes=2 * half if staging == "tight" else 16 * half,
                         window=(None if seed == 4 else 32), io_writers=writers)
        r = check_against_oracle(wl, tc)
        assert r.bytes_file_write > 0 and r.bytes_file_read > 0
        tc.close()


@pytest.mark.parametrize("stripes,threads,direct,chunk", [(1, (2, 4), False, None), (3, (3, 2), False, 1 << 16),
                                                          (4, (1, 5), True, None), (2, (0, 0), True, 1 << 20),
                                                          (8, (8, 8), False, 12 << 20), (2, (4, 4), True, 1 << 30)])
def test_multi_chunk_extents_over_stripes(stripes, threads, direct, chunk, tmp_path):
    # tensors of several 8 MiB chunks (odd tails), so that one request spreads over the
    # workers and, with stripes, over the files; the bytes must come back whole from
    # whatever file, in whatever order the workers finished
    if direct and not _direct_ok(tmp_path):
        pytest.skip("the temporary directory's file system does not take O_DIRECT")
    wl = W.random_workload(21, n_tensors=36, n_steps=50, max_per_step=2,
                           sizes=((8 << 20) + 100, (20 << 20) + 4096 + 48, 1 << 19, 33000), hbm_frac=0.1,
                           host_frac=0.25, n_iterations=2)
    big = (int(wl.tensor_bytes.max()) + 4095) // 4096 * 4096
    tc = run_library(wl, file_path=_tmpfile(tmp_path), staging_bytes=6 * big, window=16, io_writers=threads,
                     stripes=stripes, direct=direct, io_chunk=chunk)
    r = check_against_oracle(wl, tc)
    assert r.bytes_file_write > (64 << 20) and r.bytes_file_read > (64 << 20)
    tc.close()


def test_stripes_are_fixed_once_the_file_tier_is_in_use(tmp_path):
    wl = _random(4)
    tc = T.TensorCache.from_workload(wl)
    tc.bind_torch(file_path=_tmpfile(tmp_path), staging_bytes=1 << 20, stripes=2)
    for t in range(wl.n_tensors):
        tc.load_tensor(t, W.workload_payload(wl, t))
    fd = os.open(_tmpfile(tmp_path, "late.bin"), os.O_RDWR | os.O_CREAT, 0o600)
    with pytest.raises(T.TcError) as e:
        tc.add_stripe(fd)
    assert e.value.code == -2                       # TC_E_STATE
    with pytest.raises(T.TcError) as e:
        tc.set_io_chunk(1 << 20)
    assert e.value.code == -2
    os.close(fd)
    tc.close()


def test_write_behind_with_dma_copies_and_o_direct(tmp_path):
    wl = _random(5)
    direct = _direct_ok(tmp_path)
    tc = run_library(wl, file_path=_tmpfile(tmp_path), staging_bytes=4 << 20, dma_threshold=1 << 15, direct=direct,
                     window=16, io_writers=(3, 2))
    r = check_against_oracle(wl, tc)
    assert r.bytes_file_write > 0
    st = tc.cache_stats()
    assert st["dma_copies"] > 0 and st["file_write_ns"] > 0
    tc.close()


@pytest.mark.parametrize("seed", range(6))
def test_random_settings_keep_the_schedule_and_every_byte(seed, tmp_path):
    # the launch shape must never matter: random combinations of window, merge size, DMA
    # threshold, mover grid and chunk, modelled compute, buffered or direct file I/O
    rng = np.random.default_rng(500 + seed)
    wl = W.random_workload(40 + seed, n_tensors=140, n_steps=90, max_per_step=3,
                           sizes=(512, 4096, 100, 33000, 70001, 262144 + 48), hbm_frac=0.1,
                           host_frac=float(rng.choice([0.3, 0.6, 1.3])), perturb_one_in=int(rng.choice([0, 6, 11])),
                           n_iterations=3)
    window = [None, 1, 5, 64, 256][int(rng.integers(0, 5))]
    direct = bool(rng.integers(0, 2)) and _direct_ok(tmp_path)
    tc = run_library(wl, file_path=_tmpfile(tmp_path), staging_bytes=2 << 20, window=window,
                     merge_bytes=int(rng.choice([0, 1 << 16, 1 << 22, 1 << 30])),
                     dma_threshold=int(rng.choice([0, 0, 1 << 16, 1 << 18])) or None,
                     mover=(int(rng.choice([1, 8, 64, 300])), int(rng.choice([4096, 16384, 65536, 1 << 20]))),
                     busy=bool(rng.integers(0, 2)), direct=direct,
                     io_writers=(int(rng.integers(0, 4)), int(rng.integers(0, 4))))
    r = check_against_oracle(wl, tc)
    assert len(r.log) > 100
    tc.close()


# ----------------------------------------------------------------------------
# two tiers: host cache over the file (optimizer states, Sec. 3.4.2)
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("window", [None, 16])
@pytest.mark.parametrize("n,k", [(8, 5), (8, 3), (40, 1), (6, 6)])
def test_two_tier_sweep_of_equal_tensors(n, k, window, tmp_path):
    wl = W.single_class_sweep(n, k, size=5120, n_iterations=3)
    tc = run_library(wl, file_path=_tmpfile(tmp_path), host_tier=True, window=window)
    r = check_against_oracle(wl, tc)
    assert r.bytes_d2h == 0 and r.misses == 0
    assert r.bytes_file_write == 3 * ((n - k) + min(k, n - k)) * 5120
    tc.close()


@pytest.mark.parametrize("threads,stripes,chunk", [((4, 4), 1, None), ((0, 0), 1, None), ((1, 3), 3, 1 << 16),
                                                   ((3, 0), 2, 1 << 16), ((0, 2), 1, 1 << 17)])
def test_two_tier_optimizer_sweep(threads, stripes, chunk, tmp_path):
    # state tensors of several chunks, a fast tier of 40 % of the states: every updated
    # tensor goes straight from its host buffer to the file and the next one straight in,
    # whatever the worker threads; the reader of a buffer waits for the writer that drains it
    wl = W.optimizer_sweep("opt_small", layers=3, hidden=128, ffn=344, vocab=3000, cache_frac=0.4, n_iterations=3)
    tc = run_library(wl, file_path=_tmpfile(tmp_path), host_tier=True, io_writers=threads, stripes=stripes,
                     io_chunk=chunk, window=(None if stripes == 1 else 8))
    r = check_against_oracle(wl, tc)
    assert r.misses == 0 and r.bytes_file_write > wl.total_bytes() and r.bytes_d2h == 0
    st = tc.cache_stats()
    assert st["waits_total"] == 3 * 3 * len(wl.profile)        # every fetch of a PRE call is waited for on the host
    tc.close()


@pytest.mark.parametrize("seed", range(6))
def test_two_tier_random_traces(seed, tmp_path):
    # irregular traces (tensors dropped unused, re-fetched, several per step, read-only
    # accesses that release without a write-back), with and without prefetching
    wl = W.random_workload(seed + 40, n_tensors=60, n_steps=90, hbm_frac=0.1, host_frac=0.0, n_iterations=3,
                           perturb_one_in=(7 if seed % 2 else 0),
                           sizes=(512, 4096, 100, 33000, (1 << 17) + 24))
    wl.no_prefetch = seed == 5
    assert wl.host_bytes == (0, 0)
    tc = run_library(wl, file_path=_tmpfile(tmp_path), host_tier=True, window=(None if seed < 3 else 4),
                     io_chunk=1 << 16, ahead=(None if seed != 2 else 0))
    r = check_against_oracle(wl, tc)
    assert r.bytes_file_read > 0 and r.bytes_d2h == 0
    tc.close()


def test_two_tier_mode_wants_a_plan_without_host_buffers_and_host_memory(tmp_path):
    import torch
    wl = _random(3)                                     # has host budgets
    tc = T.TensorCache.from_workload(wl)
    with pytest.raises(T.TcError, match="host budgets 0"):
        tc.bind_torch(file_path=_tmpfile(tmp_path), host_tier=True)
    tc.close()
    wl = W.single_class_sweep(8, 5)
    tc = T.TensorCache.from_workload(wl)
    dev = torch.empty(1 << 16, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(T.TcError, match="pinned host memory"):
        tc.bind_memory(dev.data_ptr(), dev.numel(), 0, 0, 0, 0, -1, 0, T.BIND_HOST_TIER)
    tc.close()


# ----------------------------------------------------------------------------
# degenerate traces
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("window", [None, 4])
def test_degenerate_traces(window, tmp_path):
    # an iteration without steps, modules without tensors, tensors no module uses (they never
    # get a GPU buffer), tensors barely larger than a stamp, one tensor per class
    from workloads import traces as Tr
    cases = [
        ("no_steps", [512, 1024], [0, 1], [], 4096, (4096, 4096)),
        ("empty_steps", [512, 1024, 512], [0, 1, 0], [[], [(0, 1)], [], [(2, 3)], []], 1024, (4096, 4096)),
        ("unused_tensors", [512, 512, 512, 2048, 100], [0, 0, 0, 1, 1], [[(0, 1)], [(1, 3)], [(0, 3)]], 512, (512, 0)),
        ("tiny_tensors", [16, 16, 16, 20, 20, 20, 32, 32], [0] * 8,
         [[(0, 3)], [(3, 3), (6, 2)], [(1, 3)], [(4, 3), (7, 3)], [(2, 3), (5, 1)], [(0, 1), (6, 3)]], 1024, (1024, 0)),
        ("every_class_one_tensor", [256, 512, 768, 1024], [0, 0, 1, 1], [[(0, 3), (2, 3)], [(1, 3), (3, 3)]] * 2, 2560,
         (0, 0)),
    ]
    for name, sizes, groups, steps, hbm, host in cases:
        wl = Tr._simple(name, sizes, groups, steps, hbm, host, literal=False, n_iterations=3)
        tc = run_library(wl, file_path=_tmpfile(tmp_path, name + ".bin"), staging_bytes=1 << 16, window=window)
        check_against_oracle(wl, tc)
        tc.close()


# ----------------------------------------------------------------------------
# no host buffers under the GPU cache: every eviction is a write-back to the file
# ----------------------------------------------------------------------------

def test_a_tensor_written_back_a_moment_ago_is_read_back_whole(tmp_path):
    # four tensors, three GPU buffers, no host buffer: tensor 1 leaves for its file extent after
    # step 4 and is prefetched again after step 5, while the unit that writes it back still
    # waits for the read of its partner; the read of the extent has to come behind that write
    from workloads import traces as Tr
    R_, W_, RW_ = 1, 2, 3
    steps = [[(1, RW_)], [(1, R_), (3, W_), (0, RW_)], [(0, RW_), (3, RW_)], [(3, W_), (1, R_)], [(1, R_), (3, RW_)],
             [(2, R_), (3, RW_)], [(0, R_)], [(1, W_), (3, R_), (0, W_)], [(2, R_), (0, RW_)]]
    wl = Tr._simple("wb_then_fetch", [33000] * 4, [0] * 4, steps, hbm_bytes=112272, host_bytes=(13209, 0),
                    literal=False, n_iterations=2)
    for window in (None, 4):
        tc = run_library(wl, file_path=_tmpfile(tmp_path, f"w{window}.bin"), staging_bytes=8 * 36864, window=window)
        r = check_against_oracle(wl, tc)
        assert r.plan.cpu_count == [0] and sum(1 for e in r.log if e[3] == 4) >= 4      # write-backs
        tc.close()


@pytest.mark.parametrize("seed", [0, 1, 2, 3, 4, 5, 7, 8, 9, 11])
def test_single_group_traces_with_few_or_no_host_buffers(seed, tmp_path):
    # one group only and a host budget between nothing and a third: most evictions go to the
    # file and come back from it a few steps later, whatever the launch settings
    rng = np.random.default_rng(900 + seed)
    wl = W.random_workload(700 + seed, n_tensors=int(rng.integers(6, 90)), n_steps=int(rng.integers(10, 120)),
                           max_per_step=int(rng.integers(1, 5)),
                           sizes=[(33000,), (512, 1024), (16, 17, 31, 4096), (70001, 262144 + 48, 1024)][seed % 4],
                           hbm_frac=float(rng.choice([0.0, 0.1, 0.3])), host_frac=float(rng.choice([0.0, 0.1, 0.3])),
                           two_groups=False, n_iterations=int(rng.integers(1, 4)), perturb_one_in=int(rng.choice([0, 6])))
    big = (int(wl.tensor_bytes.max()) + 4095) // 4096 * 4096
    tc = run_library(wl, file_path=_tmpfile(tmp_path), staging_bytes=int(rng.choice([2, 8])) * big,
                     window=[None, 5, 64][seed % 3], io_writers=(int(rng.integers(0, 4)), int(rng.integers(0, 4))),
                     busy=bool(seed % 2))
    r = check_against_oracle(wl, tc)
    assert r.bytes_file_write > 0 and r.bytes_file_read > 0
    tc.close()


def test_dma_path_switched_on_and_off_between_iterations(tmp_path):
    # the side streams and the bounce ring come and go with tc_set_dma_threshold; whatever path
    # an iteration's copies took, schedule and bytes are the oracle's
    wl = _random(6)
    wl.iterations = [wl.iterations[0]] * 5
    tc = T.TensorCache.from_workload(wl)
    tc.bind_torch(file_path=_tmpfile(tmp_path), staging_bytes=2 << 20)
    for t in range(wl.n_tensors):
        tc.load_tensor(t, W.workload_payload(wl, t))
    cs = torch.cuda.Stream()
    for i, steps in enumerate(wl.iterations):
        tc.set_dma_threshold((0, 1 << 10, 0, 1 << 16, 1 << 10)[i])
        tc.set_dma_policy(i == 4)
        if i % 2:
            tc.replay_iteration_c(steps, cs.cuda_stream)
        else:
            tc.replay_iteration(steps, cs.cuda_stream)
    tc.synchronize()
    check_against_oracle(wl, tc)
    assert tc.cache_stats()["dma_copies"] > 0
    tc.close()
