"""Many small seeded workloads through the C-ABI library against the oracle: random shapes
(tensor counts, sizes from 16 bytes to a MiB, one or two groups, budgets from the working-set
floor up, host buffers from none to ample, perturbed orders, the base variant, the two-tier
mode) under random launch settings, and the hook-level interface driven in lockstep with the
full-bytes oracle with state dumps, tensor read-backs and setting changes between the calls.
A few seconds each; the cases that once failed are pinned by name in test_gpu_parity.py."""

import os

import numpy as np
import pytest

import paper_2511_14124_amd as T
import workloads as W
from oracle import tc_oracle as o
from tests.parity import run_library, check_against_oracle, compare_logs, oracle_log_array

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

SIZE_SETS = [(512, 4096, 100, 33000), (16, 17, 31, 4096), (70001, 262144 + 48, 1024), ((1 << 20) + 24, 65536, 300, 5000),
             (256, 256, 512), (33000,)]


@pytest.mark.parametrize("block", range(4))
def test_random_workloads_under_random_settings(block, tmp_path):
    ran = 0
    for seed in range(30000 + 40 * block, 30000 + 40 * (block + 1)):
        rng = np.random.default_rng(seed)
        host_tier = bool(rng.integers(0, 4) == 0)
        wl = W.random_workload(seed, n_tensors=int(rng.integers(8, 160)), n_steps=int(rng.integers(5, 140)),
                               max_per_step=int(rng.integers(1, 6)), sizes=SIZE_SETS[int(rng.integers(0, len(SIZE_SETS)))],
                               hbm_frac=float(rng.choice([0.0, 0.05, 0.1, 0.3, 0.7, 1.5])),
                               host_frac=0.0 if host_tier else float(rng.choice([0.0, 0.1, 0.3, 0.6, 1.3])),
                               two_groups=bool(rng.integers(0, 2)), n_iterations=int(rng.integers(1, 5)),
                               literal=bool(rng.integers(0, 5) == 0), perturb_one_in=int(rng.choice([0, 0, 3, 6, 11])))
        wl.no_prefetch = bool(rng.integers(0, 6) == 0)
        settings = dict(window=[None, None, 1, 5, 64, 256][int(rng.integers(0, 6))],
                        merge_bytes=int(rng.choice([0, 1 << 16, 1 << 22, 1 << 30])),
                        dma_threshold=(None if host_tier else (int(rng.choice([0, 0, 1 << 16, 1 << 18])) or None)),
                        mover=(int(rng.choice([1, 8, 12, 64, 300])), int(rng.choice([4096, 16384, 65536, 1 << 20]))),
                        busy=bool(rng.integers(0, 2)), io_writers=(int(rng.integers(0, 5)), int(rng.integers(0, 5))),
                        stripes=int(rng.choice([1, 1, 2, 4])), io_chunk=int(rng.choice([1 << 16, 1 << 17, 8 << 20])),
                        ahead=[None, 0, 1, 3, 16, 256][int(rng.integers(0, 6))], host_tier=host_tier,
                        dma_when_behind=bool(seed % 2), one_stream=bool(seed % 5 == 0),
                        gpu_deps=bool(seed % 3 == 0) and not host_tier)
        wl.alloc_write_only = bool(seed % 7 == 0)
        try:
            o.replay_workload(wl)
        except o.CapacityError:                           # literal Alg. 2 below a step's working set
            continue
        big = (int(wl.tensor_bytes.max()) + 4095) // 4096 * 4096
        tc = run_library(wl, file_path=os.path.join(str(tmp_path), f"r{seed}.bin"),
                         staging_bytes=int(rng.choice([2, 3, 8])) * big, **settings)
        try:
            check_against_oracle(wl, tc)
        except AssertionError as e:
            raise AssertionError(f"seed {seed}, settings {settings}: {e}") from e
        tc.close()
        ran += 1
    assert ran >= 30


@pytest.mark.parametrize("block", range(3))
def test_hook_calls_in_lockstep_with_the_full_bytes_oracle(block, tmp_path):
    for seed in range(40000 + 60 * block, 40000 + 60 * (block + 1)):
        rng = np.random.default_rng(seed)
        host_tier = bool(rng.integers(0, 4) == 0)
        wl = W.random_workload(seed, n_tensors=int(rng.integers(6, 60)), n_steps=int(rng.integers(5, 60)),
                               max_per_step=int(rng.integers(1, 5)),
                               sizes=[(512, 4096, 100, 33000), (33000,), (70001, 1024)][int(rng.integers(0, 3))],
                               hbm_frac=float(rng.choice([0.0, 0.1, 0.3])),
                               host_frac=0.0 if host_tier else float(rng.choice([0.0, 0.1, 0.6])),
                               two_groups=bool(rng.integers(0, 2)), n_iterations=int(rng.integers(1, 4)),
                               perturb_one_in=int(rng.choice([0, 5])))
        pay = lambda t: W.workload_payload(wl, t)
        st, te, rw, _ns = wl.events()
        r = o.build(wl.tensor_bytes.tolist(), wl.tensor_group.tolist(), st, te, rw, wl.hbm_bytes, wl.host_bytes,
                    wl.align, wl.literal_alg2, pay)
        tc = T.TensorCache.from_workload(wl)
        big = (int(wl.tensor_bytes.max()) + 4095) // 4096 * 4096
        tc.bind_torch(file_path=os.path.join(str(tmp_path), f"a{seed}.bin"), staging_bytes=int(rng.choice([2, 8])) * big,
                      host_tier=host_tier, stripes=int(rng.choice([1, 2])))
        for t in range(wl.n_tensors):
            tc.load_tensor(t, pay(t))
        cs = torch.cuda.Stream()
        where = f"seed {seed}"
        for steps in wl.iterations:
            for k, access in enumerate(steps):
                ids = [t for (t, _a) in access]
                flags = [a for (_t, a) in access]
                tc.migrate_step(k, T.PRE, ids, flags, cs.cuda_stream)
                r.pre(k, access)
                tc.emulate_compute(cs.cuda_stream, 0)
                what = int(rng.integers(0, 12))
                if what == 0:
                    tier, gs, _ = tc.dump_state()
                    assert tier.tolist() == r.cur and gs.tolist() == r.gslot, where
                elif what == 1:
                    t = int(rng.integers(0, wl.n_tensors))
                    assert np.array_equal(tc.read_tensor(t), r.read_tensor(t)), (where, k, t)
                elif what == 2:
                    tc.synchronize()
                tc.migrate_step(k, T.POST, ids, flags, cs.cuda_stream)
                r.post(k, ids)
                what = int(rng.integers(0, 14))
                if what == 0:
                    t = int(rng.integers(0, wl.n_tensors))
                    assert np.array_equal(tc.read_tensor(t), r.read_tensor(t)), (where, k, t)
                elif what == 1:
                    tc.set_merge_bytes(int(rng.choice([0, 1 << 16, 1 << 28])))
                elif what == 2:
                    tc.set_decide_ahead(int(rng.choice([0, 1, 4, 16])))
                elif what == 3:
                    tc.set_io_threads(int(rng.integers(0, 4)), int(rng.integers(0, 4)))
                elif what == 4:
                    tier, gs, cslot = tc.dump_state()
                    assert tier.tolist() == r.cur and gs.tolist() == r.gslot and cslot.tolist() == r.cslot, where
                elif what == 5:
                    s_ = tc.cache_stats()
                    assert (s_["hits"], s_["misses"]) == (r.hits, r.misses), where
            tc.end_iteration(cs.cuda_stream)
            r.end_iteration()
        tc.synchronize()
        compare_logs(tc.dump_oplog(), oracle_log_array(r))
        for t in range(wl.n_tensors):
            assert np.array_equal(tc.read_tensor(t), r.read_tensor(t)), (where, "end", t)
        tc.close()
