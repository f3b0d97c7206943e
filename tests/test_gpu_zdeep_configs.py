"""Configurations 4 and 5 as deep as the box holds them, byte-checked against the oracle.

At full size the two need 200 and 485 GiB; a GPU machine has 288 GB of HBM, 295 GB of RAM and 80 GB of
free disk.  The layer count is derived from the box by the arithmetic bench.py uses
(paper_2511_14124_amd/box.py), once with the file tier on the box's disk and once with it in memory
(tmpfs), where configuration 4 fits whole.  Schedule, counters and maps are compared in full, bytes
on every tensor under 1 MiB and a sample of the large ones over all kinds and final tiers, in the
launch configuration bench.py times.  (Collected late on purpose: these are the longest tests.)"""

import os
import tempfile

import pytest

import paper_2511_14124_amd as T
import workloads as W
from paper_2511_14124_amd import box
from tests.parity import run_library, check_against_oracle
from tests.test_gpu_parity import _sample

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

STAGING_DEPTH, STRIPES = 16, 8


@pytest.mark.parametrize("tier_dir", ["/tmp", "/dev/shm"], ids=["tier_on_disk", "tier_in_memory"])
@pytest.mark.parametrize("index", [3, 4], ids=["llama_13b_ckpt_nvme", "llama_30b_perturbed"])
def test_file_tier_configs_at_the_depth_the_box_holds(index, tier_dir):
    if not os.path.isdir(tier_dir):
        pytest.skip(f"{tier_dir} does not exist here")
    limits = box.box_limits(torch, [tier_dir])
    layers, rows = box.depth_the_box_holds(T, W, index, limits, STAGING_DEPTH)
    print(f"configuration {index + 1}: {layers} of {box.FULL_LAYERS[index]} layers, file tier in {tier_dir}: {rows}",
          flush=True)
    assert layers >= 4, "the box holds less than the test is meant for"
    wl = W.config(index, layers=layers)
    big = (int(wl.tensor_bytes.max()) + 4095) // 4096 * 4096
    with tempfile.TemporaryDirectory(dir=tier_dir) as d:
        paths = [os.path.join(d, f"tier.{k}.bin") for k in range(STRIPES)]
        tc = run_library(wl, fill=True, window=64, merge_bytes=1 << 30, stripe_paths=paths,
                         staging_bytes=STAGING_DEPTH * big, io_writers=(8, 8), tune=True)
        from oracle import tc_oracle as o
        r0 = o.replay_workload(wl)
        small = [t for t in range(wl.n_tensors) if wl.tensor_bytes[t] < (1 << 20)]
        r = check_against_oracle(wl, tc, tensors=sorted(set(small) | set(_sample(wl, r0, per_kind=4, extremes=3))))
        st = tc.cache_stats()
        assert st["bytes_file_read"] > 0 and st["bytes_file_write"] > 0
        if index == 4:
            assert r.misses > 0
        tc.close()
