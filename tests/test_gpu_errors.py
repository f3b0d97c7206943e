"""Error behaviour of the bound library on a real MI355X: every failure is a
return code (raised as TcError by the binding), forced from the host - a file
that is missing or too short, regions that are too small, arguments out of
range.  No kernel is made to fault; after a failed replay the context is only
destroyed."""

import os

import numpy as np
import pytest

import paper_2511_14124_amd as T
import workloads as W

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

E_ARG, E_STATE, E_CAPACITY, E_IO = -1, -2, -3, -4


def _planned(wl):
    return T.TensorCache.from_workload(wl)


def test_bind_rejects_small_or_misaligned_regions():
    wl = W.example_cpu_gpu()
    tc = _planned(wl)
    hbm = torch.empty(4096, dtype=torch.uint8, device="cuda:0")
    pinned = torch.empty(4096, dtype=torch.uint8, pin_memory=True)
    with pytest.raises(T.TcError) as e:
        tc.bind_memory(hbm.data_ptr(), 256, pinned.data_ptr(), 4096)           # HBM region smaller than the plan
    assert e.value.code == E_CAPACITY
    with pytest.raises(T.TcError) as e:
        tc.bind_memory(hbm.data_ptr(), 4096, pinned.data_ptr(), 256)           # pinned region smaller than the plan
    assert e.value.code == E_CAPACITY
    with pytest.raises(T.TcError) as e:
        tc.bind_memory(hbm.data_ptr() + 16, 4000, pinned.data_ptr(), 4096)     # not 256-byte aligned
    assert e.value.code == E_ARG
    tc.bind_memory(hbm.data_ptr(), 4096, pinned.data_ptr(), 4096)
    with pytest.raises(T.TcError) as e:
        tc.bind_memory(hbm.data_ptr(), 4096, pinned.data_ptr(), 4096)          # only once
    assert e.value.code == E_STATE
    tc.close()


def test_hook_arguments_are_checked_before_any_kernel_runs():
    wl = W.example_cpu_gpu()
    tc = _planned(wl)
    tc.bind_torch()
    n_ops = len(tc.dump_oplog())
    for args in ((99, T.PRE, [0], [1]),                 # step outside the profiled iteration
                 (0, T.PRE, [77], [1]),                 # unknown tensor
                 (0, 5, [0], [1]),                      # no such phase
                 (0, T.PRE, list(range(6)) * 11, [1] * 66)):  # more than TC_MAX_STEP_TENSORS
        with pytest.raises(T.TcError) as e:
            tc.migrate_step(*args)
        assert e.value.code == E_ARG
    with pytest.raises(T.TcError) as e:
        tc.set_replay_window(0)
    assert e.value.code == E_ARG
    with pytest.raises(T.TcError) as e:
        tc.set_replay_window(257)
    assert e.value.code == E_ARG
    with pytest.raises(T.TcError) as e:
        tc.set_mover(64, 1000)                          # chunk not a multiple of 4096
    assert e.value.code == E_ARG
    with pytest.raises(T.TcError) as e:
        tc.replay_iteration_c([[(0, 1)], [(123, 1)]])   # unknown tensor inside a replayed list
    assert e.value.code == E_ARG
    # nothing was decided or moved by the rejected calls
    assert len(tc.dump_oplog()) == n_ops and tc.cache_stats()["decide_launches"] == 0
    tc.close()


def test_file_tier_errors_are_return_codes(tmp_path):
    wl = W.example_cpu_gpu_nvme()                       # tensor 6 lives on the file tier
    # no file bound although the plan needs one
    tc = _planned(wl)
    tc.bind_torch(staging_bytes=1 << 16)
    with pytest.raises(T.TcError) as e:
        tc.load_tensor(6, W.workload_payload(wl, 6))
    assert e.value.code == E_IO
    tc.close()
    # a file that is too short: the fetch of tensor 6 reads past its end
    path = os.path.join(str(tmp_path), "short.bin")
    tc = _planned(wl)
    tc.bind_torch(file_path=path, staging_bytes=1 << 16)
    for t in range(wl.n_tensors):
        tc.load_tensor(t, W.workload_payload(wl, t))
    os.truncate(path, 0)
    cs = torch.cuda.Stream()
    with pytest.raises(T.TcError) as e:
        tc.replay_iteration(wl.iterations[0], cs.cuda_stream)
    assert e.value.code == E_IO
    tc.close()                                          # destroy after a failed replay must be clean
    # a staging region smaller than the tensor that needs it
    tc = _planned(wl)
    tc.bind_torch(file_path=os.path.join(str(tmp_path), "ok.bin"), staging_bytes=256)
    for t in range(wl.n_tensors):
        tc.load_tensor(t, W.workload_payload(wl, t))
    with pytest.raises(T.TcError) as e:
        tc.replay_iteration(wl.iterations[0], cs.cuda_stream)
    assert e.value.code == E_CAPACITY
    tc.close()


def test_failed_background_write_is_reported(tmp_path):
    # /dev/full takes no byte: every queued write fails in its writer thread, and the next
    # call that queues or waits for a write (at the latest tc_synchronize) returns TC_E_IO
    wl = W.random_workload(3, n_tensors=60, n_steps=40, max_per_step=2, sizes=(4096, 33000), hbm_frac=0.1,
                           host_frac=0.3, n_iterations=1)
    for writers in ((2, 1), (0, 0)):
        tc = _planned(wl)
        tc.bind_torch(file_fd=os.open("/dev/full", os.O_RDWR), staging_bytes=1 << 20)
        tc.set_io_threads(*writers)
        cs = torch.cuda.Stream()
        with pytest.raises(T.TcError) as e:
            tc.replay_iteration_c(wl.iterations[0], cs.cuda_stream)
            tc.synchronize()
        assert e.value.code == E_IO and "pwrite" in str(e.value)
        tc.close()


def test_two_tier_mode_reports_failed_writes_and_short_reads(tmp_path):
    # the host cache over the file: a write that fails in its writer thread (/dev/full) and a
    # read beyond the end of a file that was cut short both come back as TC_E_IO, the read from
    # the PRE call that waits for its bytes at the latest
    wl = W.single_class_sweep(12, 4, size=1 << 16, n_iterations=1)
    for threads in ((2, 2), (0, 0)):
        tc = _planned(wl)
        tc.bind_torch(file_fd=os.open("/dev/full", os.O_RDWR), host_tier=True)
        tc.set_io_threads(*threads)
        with pytest.raises(T.TcError) as e:
            tc.replay_iteration(wl.iterations[0], 0)
            tc.synchronize()
        assert e.value.code == E_IO and "pwrite" in str(e.value)
        tc.close()
        path = os.path.join(str(tmp_path), f"short{threads[0]}.bin")
        tc = _planned(wl)
        tc.bind_torch(file_path=path, host_tier=True)
        tc.set_io_threads(*threads)
        os.truncate(path, 4096)                          # the extents of the absent tensors are gone
        with pytest.raises(T.TcError) as e:
            tc.replay_iteration(wl.iterations[0], 0)
            tc.synchronize()
        assert e.value.code == E_IO and "short file" in str(e.value)
        tc.close()


def test_null_mover_context_refuses_payload_calls():
    wl = W.example_cpu_gpu()
    tc = _planned(wl)
    tc.bind_torch(null_mover=True)
    with pytest.raises(T.TcError) as e:
        tc.read_tensor(0)
    assert e.value.code == E_STATE
    with pytest.raises(T.TcError) as e:
        tc.set_dma_threshold(1 << 20)
    assert e.value.code == E_STATE
    tc.close()
