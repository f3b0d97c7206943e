"""The optimizer-state demo end to end on a small model: CPU Adam over the
two-tier cache gives the states a plain Adam gives, prefetching removes the
misses of the demand-only variant."""

import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.mark.parametrize("direct", [False, True])
def test_optimizer_demo_small(direct, tmp_path):
    from paper_2511_14124_amd import opt_demo
    import os
    path = os.path.join(str(tmp_path), "states.bin")
    if direct:
        try:
            os.close(os.open(path, os.O_RDWR | os.O_CREAT | os.O_DIRECT, 0o600))
        except OSError:
            pytest.skip("the temporary directory's file system does not take O_DIRECT")
    out = opt_demo.main(["--layers", "2", "--hidden", "256", "--ffn", "688", "--vocab", "6000", "--cache", "0.4",
                         "--sweeps", "2", "--file", path, "--stripes", "2"] + (["--direct"] if direct else []))
    assert out["sampled_states_equal_plain_adam"]
    assert out["resident"]["file_read_GiB_per_sweep"] == 0 and out["resident"]["miss_rate"] == 0
    assert out["prefetch"]["miss_rate"] == 0 and out["prefetch"]["file_read_GiB_per_sweep"] > 0
    assert out["demand"]["miss_rate"] > 0.3
