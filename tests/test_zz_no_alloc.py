"""tc_pack_static, the entry point for callers that cannot allocate, on a real
MI355X: its output against tc_pack / tc_unpack with a caller-provided index
(and against the plain definition in oracle/pack_oracle.py), byte for byte, on
two calls in a row, the second with a smaller input, so that what the first
call left in the library's device array is shown not to matter."""

import numpy as np
import pytest

import paper_2511_14124_amd as T
from oracle import pack_oracle as po

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def _case(seed, n, aligned):
    rng = np.random.default_rng(seed)
    kinds = rng.integers(0, 4, size=n)
    sizes = np.where(kinds == 0, rng.integers(1, 64, size=n),
             np.where(kinds == 1, 16 * rng.integers(1, 256, size=n),
              np.where(kinds == 2, 256 * rng.integers(1, 160, size=n), rng.integers(1, 40000, size=n))))
    if aligned:
        sizes = (sizes + 255) // 256 * 256
    src_gaps = [0, 256] if aligned else [0, 1, 2, 4, 7, 16, 100]
    slab_gaps = [0, 16] if aligned else [0, 0, 3, 16, 40]
    nb = sizes.astype(np.uint64)
    src_off = np.zeros(n, dtype=np.uint64)
    slab_off = np.zeros(n, dtype=np.uint64)
    a = b = 0
    for i in range(n):
        a += int(rng.choice(src_gaps))
        b += int(rng.choice(slab_gaps))
        src_off[i], slab_off[i] = a, b
        a += int(nb[i])
        b += int(nb[i])
    src = rng.integers(0, 256, size=a + 16, dtype=np.uint8)
    return nb, src_off, slab_off, b + 11, src


def _run_pair(seed, n, aligned):
    """pack + unpack through tc_pack_static and through tc_pack / tc_unpack; returns nothing, asserts equality"""
    nb, src_off, slab_off, slab_total, src = _case(seed, n, aligned)
    st = torch.cuda.current_stream().cuda_stream
    d_src = _dev(src)
    d_nb, d_off = _dev(nb.astype(np.int64)), _dev(slab_off.astype(np.int64))
    ptrs = _dev((src_off + np.uint64(d_src.data_ptr())).astype(np.int64))
    # the existing entry point, with an index the caller allocates
    d_index = torch.full((T.pack_tiles(slab_total),), -1, dtype=torch.int32, device="cuda:0")
    ref_slab = torch.full((slab_total,), 0xEE, dtype=torch.uint8, device="cuda:0")
    T.pack_index(d_off.data_ptr(), n, slab_total, d_index.data_ptr(), st)
    T.pack(ref_slab.data_ptr(), ptrs.data_ptr(), d_nb.data_ptr(), d_off.data_ptr(), n, slab_total, st, d_index.data_ptr())
    ref_back = torch.full((src.size,), 0x55, dtype=torch.uint8, device="cuda:0")
    ptrs_ref_back = _dev((src_off + np.uint64(ref_back.data_ptr())).astype(np.int64))
    T.unpack(ref_slab.data_ptr(), ptrs_ref_back.data_ptr(), d_nb.data_ptr(), d_off.data_ptr(), n, slab_total, st,
             d_index.data_ptr())
    # the entry point that allocates nothing; every buffer it touches exists before the first call
    new_slab = torch.full((slab_total,), 0xEE, dtype=torch.uint8, device="cuda:0")
    new_back = torch.full((src.size,), 0x55, dtype=torch.uint8, device="cuda:0")
    ptrs_new_back = _dev((src_off + np.uint64(new_back.data_ptr())).astype(np.int64))
    torch.cuda.synchronize()
    T.pack_static(new_slab.data_ptr(), ptrs.data_ptr(), d_nb.data_ptr(), d_off.data_ptr(), n, slab_total, False, st)
    T.pack_static(new_slab.data_ptr(), ptrs_new_back.data_ptr(), d_nb.data_ptr(), d_off.data_ptr(), n, slab_total, True, st)
    torch.cuda.synchronize()
    got_slab, want_slab = new_slab.cpu().numpy(), ref_slab.cpu().numpy()
    assert np.array_equal(got_slab, want_slab), (seed, n, "pack")
    assert np.array_equal(new_back.cpu().numpy(), ref_back.cpu().numpy()), (seed, n, "unpack")
    # and both against the plain definition
    tensors = [src[int(o):int(o) + int(k)] for o, k in zip(src_off, nb)]
    assert np.array_equal(got_slab, po.pack(tensors, slab_off, np.full(slab_total, 0xEE, dtype=np.uint8)))


@pytest.mark.parametrize("aligned", [True, False], ids=["pool_aligned", "any_address"])
def test_pack_static_equals_pack_on_two_calls_in_a_row_the_second_smaller(aligned):
    _run_pair(seed=31 + aligned, n=900, aligned=aligned)      # a few hundred tiles
    _run_pair(seed=77 + aligned, n=60, aligned=aligned)       # fewer tiles than the array still holds entries for
    _run_pair(seed=5 + aligned, n=1, aligned=aligned)         # one segment


def test_pack_static_refuses_a_slab_beyond_its_array_and_launches_nothing():
    st = torch.cuda.current_stream().cuda_stream
    d = torch.zeros(256, dtype=torch.uint8, device="cuda:0")
    one = _dev(np.asarray([d.data_ptr()], dtype=np.int64))
    nb = _dev(np.asarray([16], dtype=np.int64))
    off = _dev(np.asarray([0], dtype=np.int64))
    with pytest.raises(T.TcError) as e:
        T.pack_static(d.data_ptr(), one.data_ptr(), nb.data_ptr(), off.data_ptr(), 1, T.PACK_STATIC_MAX_BYTES + 1, False, st)
    assert e.value.code == -3                                  # TC_E_CAPACITY
    # the limit itself is accepted as a size (16 bytes of payload in a 4 GiB slab would need the slab;
    # only the argument check is exercised here): an empty batch of that size is a no-op
    T.pack_static(d.data_ptr(), one.data_ptr(), nb.data_ptr(), off.data_ptr(), 0, T.PACK_STATIC_MAX_BYTES, False, st)
    torch.cuda.synchronize()


def test_pack_static_inside_a_captured_graph_replays_like_the_eager_call():
    # the callers it is for: after one eager call (the library asks for its array's address once per
    # device) a pack and an unpack are captured into a graph; three replays, with eager work and
    # synchronisation between them and new bytes in the tensors each time, against the plain definition
    nb, src_off, slab_off, slab_total, src = _case(seed=19, n=300, aligned=False)
    n = len(nb)
    st = torch.cuda.Stream()
    d_src = _dev(src)
    d_nb, d_off = _dev(nb.astype(np.int64)), _dev(slab_off.astype(np.int64))
    ptrs = _dev((src_off + np.uint64(d_src.data_ptr())).astype(np.int64))
    slab = torch.zeros(slab_total, dtype=torch.uint8, device="cuda:0")
    back = torch.zeros(src.size, dtype=torch.uint8, device="cuda:0")
    ptrs_back = _dev((src_off + np.uint64(back.data_ptr())).astype(np.int64))
    torch.cuda.synchronize()
    T.pack_static(slab.data_ptr(), ptrs.data_ptr(), d_nb.data_ptr(), d_off.data_ptr(), n, slab_total, False, st.cuda_stream)
    st.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(st):
        with torch.cuda.graph(g, stream=st):
            T.pack_static(slab.data_ptr(), ptrs.data_ptr(), d_nb.data_ptr(), d_off.data_ptr(), n, slab_total, False,
                          st.cuda_stream)
            T.pack_static(slab.data_ptr(), ptrs_back.data_ptr(), d_nb.data_ptr(), d_off.data_ptr(), n, slab_total, True,
                          st.cuda_stream)
    for replay in range(3):
        d_src.random_(0, 255)                               # eager work between the replays
        slab.zero_()
        back.fill_(0x55)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        now = d_src.cpu().numpy()
        tensors = [now[int(o):int(o) + int(k)] for o, k in zip(src_off, nb)]
        assert np.array_equal(slab.cpu().numpy(), po.pack(tensors, slab_off, np.zeros(slab_total, dtype=np.uint8))), replay
        got = back.cpu().numpy()
        for o, k in zip(src_off, nb):
            assert np.array_equal(got[int(o):int(o) + int(k)], now[int(o):int(o) + int(k)]), replay
