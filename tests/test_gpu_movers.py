"""The stand-alone movers of the library on a real MI355X, byte for byte
against the plain definitions in oracle/pack_oracle.py: pack and unpack (the
register path at any alignment, the LDS-staged path for tiles of many tiny
pieces), the batched copy and the batched exchange of the migration kernel."""

import numpy as np
import pytest

import paper_2511_14124_amd as T
from oracle import pack_oracle as po

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def _layout(rng, sizes, gap_choices):
    off, at = [], 0
    for n in sizes:
        at += int(rng.choice(gap_choices))
        off.append(at)
        at += int(n)
    return np.asarray(off, dtype=np.uint64), at


PACK_CASES = [
    # (name, segment sizes, source gaps, slab gaps): sizes off 16 bytes, misaligned on both sides,
    # segments smaller than a vector, segments spanning several 16 KiB tiles, a ragged last tile
    ("aligned", [4096] * 37, [0], [0]),
    ("tiny", [1, 2, 3, 15, 16, 17, 31, 33, 1, 1, 64, 5], [0, 1, 3, 7], [0]),
    ("misaligned_both", [100, 33000, 4096, 17, 70001, 12288, 8192, 555], [1, 5, 9, 13], [0, 3, 16, 21]),
    ("multi_tile", [16384 * 3 + 48, 16384, 16383, 16385, 200000], [2], [0]),
    ("one_big", [5 << 20], [4], [0]),
    # 256-byte aligned buffers with padding between them (pool strides): the register path, gaps kept
    ("pool_strides", [1536, 4096, 12288, 3072, 24576, 512, 16384 * 2, 768] * 6, [0, 256, 1024], [0, 256]),
    # 33 to 256 pieces in a tile: the register path with the workgroup-wide piece table
    ("many_small_aligned", [256] * 200 + [4096] * 5, [0], [0]),
    ("wide_64B", [64] * 700 + [8192, 64, 64], [0, 192], [0]),
    ("wide_ragged", [100] * 500 + [33, 7, 4096] + [52] * 300, [0, 1, 3, 28], [0, 0, 5]),
    ("wide_exactly_256_pieces", [64] * 256 + [16384] + [64] * 257, [0], [0]),
    # more pieces than that: staged in LDS, piece after piece
    ("beyond_wide", [20] * 2000 + [16384] + [3] * 700, [0, 2], [0, 1]),
    # tensors at odd addresses holding two to a few whole vectors of the slab: where a piece's interior
    # vectors (moved as the aligned dwords around them) begin and end, for every address modulo 4
    ("odd_addresses_few_vectors", [1024, 48, 2048, 64, 4096, 80, 96, 3072, 112, 128, 1500, 33, 144, 160] * 5,
     [1, 2, 3, 5, 6, 7], [0, 0, 16]),
    ("mixed", [4096] * 9 + [100] + [4096] * 7 + [8192, 33, 16384, 16384], [0], [0]),
]


@pytest.mark.parametrize("indexed", [False, True], ids=["bisect", "indexed"])
@pytest.mark.parametrize("name,sizes,src_gaps,slab_gaps", PACK_CASES, ids=[c[0] for c in PACK_CASES])
def test_pack_and_unpack_match_the_definition(name, sizes, src_gaps, slab_gaps, indexed):
    rng = np.random.default_rng(len(sizes))
    nb = np.asarray(sizes, dtype=np.uint64)
    src_off, src_total = _layout(rng, sizes, src_gaps)
    slab_off, slab_total = _layout(rng, sizes, slab_gaps)
    slab_total += 11                                   # ragged tail no segment covers
    src = rng.integers(0, 256, size=src_total + 16, dtype=np.uint8)
    tensors = [src[int(o):int(o) + int(n)] for o, n in zip(src_off, nb)]
    want = po.pack(tensors, slab_off, np.full(slab_total, 0xEE, dtype=np.uint8))

    d_src = _dev(src)
    d_slab = torch.full((slab_total,), 0xEE, dtype=torch.uint8, device="cuda:0")
    ptrs = _dev((src_off + np.uint64(d_src.data_ptr())).astype(np.int64))
    d_nb, d_off = _dev(nb.astype(np.int64)), _dev(slab_off.astype(np.int64))
    st = torch.cuda.current_stream().cuda_stream
    index = 0
    if indexed:
        d_index = torch.full((T.pack_tiles(slab_total),), -1, dtype=torch.int32, device="cuda:0")
        T.pack_index(d_off.data_ptr(), len(sizes), slab_total, d_index.data_ptr(), st)
        index = d_index.data_ptr()
    T.pack(d_slab.data_ptr(), ptrs.data_ptr(), d_nb.data_ptr(), d_off.data_ptr(), len(sizes), slab_total, st, index)
    torch.cuda.synchronize()
    assert np.array_equal(d_slab.cpu().numpy(), want), name

    # unpack into a fresh, differently filled source image
    d_back = torch.full((src_total + 16,), 0x55, dtype=torch.uint8, device="cuda:0")
    ptrs2 = _dev((src_off + np.uint64(d_back.data_ptr())).astype(np.int64))
    T.unpack(d_slab.data_ptr(), ptrs2.data_ptr(), d_nb.data_ptr(), d_off.data_ptr(), len(sizes), slab_total, st, index)
    torch.cuda.synchronize()
    got = d_back.cpu().numpy()
    want_back = np.full(src_total + 16, 0x55, dtype=np.uint8)
    for t, o in zip(po.unpack(want, nb, slab_off), src_off):
        want_back[int(o):int(o) + t.size] = t
    assert np.array_equal(got, want_back), name


@pytest.mark.parametrize("seed", range(8))
def test_pack_and_unpack_on_random_layouts(seed):
    # random sizes (1 B .. 40 KiB, skewed to small ones), random gaps and phases on both
    # sides, several hundred segments over dozens of tiles: the register path with aligned and
    # with misaligned tensor-side accesses, ragged piece edges, and the LDS-staged many-piece
    # path (more than 32 pieces in a tile) all occur, tile by tile
    rng = np.random.default_rng(1000 + seed)
    n = int(rng.integers(150, 700))
    kinds = rng.integers(0, 4, size=n)
    sizes = np.where(kinds == 0, rng.integers(1, 64, size=n),
             np.where(kinds == 1, 16 * rng.integers(1, 256, size=n),
              np.where(kinds == 2, 256 * rng.integers(1, 160, size=n), rng.integers(1, 40000, size=n)))).tolist()
    aligned = seed % 2 == 0
    src_gaps = [0, 16, 256] if aligned else [0, 1, 2, 4, 7, 16, 100]
    slab_gaps = [0, 16] if aligned else [0, 0, 3, 16, 40]
    if aligned:
        sizes = [(x + 15) // 16 * 16 if i % 7 else x for i, x in enumerate(sizes)]   # mostly regular, some odd
    nb = np.asarray(sizes, dtype=np.uint64)
    src_off, src_total = _layout(rng, sizes, src_gaps)
    slab_off, slab_total = _layout(rng, sizes, slab_gaps)
    slab_total += int(rng.integers(0, 40))
    src = rng.integers(0, 256, size=src_total + 16, dtype=np.uint8)
    tensors = [src[int(o):int(o) + int(k)] for o, k in zip(src_off, nb)]
    want = po.pack(tensors, slab_off, np.full(slab_total, 0xEE, dtype=np.uint8))
    d_src = _dev(src)
    d_slab = torch.full((slab_total,), 0xEE, dtype=torch.uint8, device="cuda:0")
    ptrs = _dev((src_off + np.uint64(d_src.data_ptr())).astype(np.int64))
    d_nb, d_off = _dev(nb.astype(np.int64)), _dev(slab_off.astype(np.int64))
    st = torch.cuda.current_stream().cuda_stream
    d_index = torch.empty(T.pack_tiles(slab_total), dtype=torch.int32, device="cuda:0")
    T.pack_index(d_off.data_ptr(), n, slab_total, d_index.data_ptr(), st)
    T.pack(d_slab.data_ptr(), ptrs.data_ptr(), d_nb.data_ptr(), d_off.data_ptr(), n, slab_total, st, d_index.data_ptr())
    torch.cuda.synchronize()
    assert np.array_equal(d_slab.cpu().numpy(), want)
    d_back = torch.full((src_total + 16,), 0x55, dtype=torch.uint8, device="cuda:0")
    ptrs2 = _dev((src_off + np.uint64(d_back.data_ptr())).astype(np.int64))
    T.unpack(d_slab.data_ptr(), ptrs2.data_ptr(), d_nb.data_ptr(), d_off.data_ptr(), n, slab_total, st, d_index.data_ptr())
    torch.cuda.synchronize()
    want_back = np.full(src_total + 16, 0x55, dtype=np.uint8)
    for t, o in zip(po.unpack(want, nb, slab_off), src_off):
        want_back[int(o):int(o) + t.size] = t
    assert np.array_equal(d_back.cpu().numpy(), want_back)


def test_pack_of_nothing_is_a_no_op():
    d = torch.zeros(64, dtype=torch.uint8, device="cuda:0")
    assert T.pack_tiles(0) == 0 and T.pack_tiles(1) == 1 and T.pack_tiles(16384) == 1 and T.pack_tiles(16385) == 2
    T.pack(d.data_ptr(), 0, 0, 0, 0, 0, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert int(d.sum()) == 0


@pytest.mark.parametrize("wg,chunk", [(1, 4096), (7, 8192), (64, 65536), (512, 1 << 20)])
def test_copy_batch_moves_every_segment(wg, chunk):
    # sizes off the chunk and off 16 bytes; device->device, pinned->device and device->pinned
    rng = np.random.default_rng(wg)
    sizes = [16, 17, 4096, 70001, 262144 + 48, (1 << 20) + 3, 31] * 9      # 63 segments: two launches
    off, at = [], 0
    for n in sizes:
        off.append(at)
        at += (n + 15) // 16 * 16
    off = np.asarray(off, dtype=np.uint64)
    img = rng.integers(0, 256, size=at, dtype=np.uint8)
    pinned_src = torch.from_numpy(img.copy()).pin_memory()
    d_mid = torch.zeros(at, dtype=torch.uint8, device="cuda:0")
    d_mid2 = torch.zeros(at, dtype=torch.uint8, device="cuda:0")
    pinned_dst = torch.zeros(at, dtype=torch.uint8).pin_memory()
    st = torch.cuda.current_stream().cuda_stream
    nb = np.asarray(sizes, dtype=np.uint64)
    for a, b in ((pinned_src, d_mid), (d_mid, d_mid2), (d_mid2, pinned_dst)):
        T.copy_batch(off + np.uint64(a.data_ptr()), off + np.uint64(b.data_ptr()), nb, st, wg, chunk)
    torch.cuda.synchronize()
    want = np.zeros(at, dtype=np.uint8)
    for o, n in zip(off, sizes):
        want[int(o):int(o) + n] = img[int(o):int(o) + n]
    assert np.array_equal(pinned_dst.numpy(), want)


@pytest.mark.parametrize("wg,chunk", [(3, 4096), (64, 65536)])
def test_exchange_batch_swaps_in_place(wg, chunk):
    # unit i: a tensor leaves GPU buffer y_i for host buffer x_i while the tensor in x_i arrives in y_i
    rng = np.random.default_rng(5)
    sizes = [16, 48, 4096 + 16, 70000, 262144 + 48, 1 << 20]
    off, at = [], 0
    for n in sizes:
        off.append(at)
        at += n
    host = rng.integers(0, 256, size=at, dtype=np.uint8)
    gpu = rng.integers(0, 256, size=at, dtype=np.uint8)
    # the oracle works on one flat array: [gpu image | host image]
    mem = np.concatenate([gpu, host])
    units = [(o, at + o, at + o, o, n) for o, n in zip(off, sizes)]
    units[1] = (-1, 0, at + off[1], off[1], sizes[1])          # incoming half only
    units[2] = (off[2], at + off[2], -1, 0, sizes[2])          # outgoing half only
    want = po.exchange(mem.copy(), units)
    d = _dev(gpu)
    h = torch.from_numpy(host.copy()).pin_memory()
    D, H = d.data_ptr(), h.data_ptr()
    o64 = np.asarray(off, dtype=np.uint64)
    out_src, out_dst = o64 + np.uint64(D), o64 + np.uint64(H)
    in_src, in_dst = o64 + np.uint64(H), o64 + np.uint64(D)
    out_src[1] = 0
    in_src[2] = 0
    T.exchange_batch(out_src, out_dst, in_src, in_dst, np.asarray(sizes, dtype=np.uint64),
                     torch.cuda.current_stream().cuda_stream, wg, chunk)
    torch.cuda.synchronize()
    assert np.array_equal(d.cpu().numpy(), want[:at]) and np.array_equal(h.numpy(), want[at:])


def test_movers_reject_bad_arguments():
    with pytest.raises(T.TcError):
        T.copy_batch(np.asarray([8], dtype=np.uint64), np.asarray([16], dtype=np.uint64),
                     np.asarray([16], dtype=np.uint64))                     # misaligned pointer
    with pytest.raises(T.TcError):
        T.copy_batch(np.asarray([0], dtype=np.uint64), np.asarray([16], dtype=np.uint64),
                     np.asarray([16], dtype=np.uint64))                     # null source
    d = torch.zeros(64, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(T.TcError):
        T.copy_batch(np.asarray([d.data_ptr()], dtype=np.uint64), np.asarray([d.data_ptr() + 32], dtype=np.uint64),
                     np.asarray([16], dtype=np.uint64), 0, 64, 1000)        # chunk not a multiple of 4096


def _counter_bytes(n):
    # n bytes of a 64-bit counter pattern on the device (every aligned 8 bytes differ)
    words = torch.arange((n + 7) // 8, dtype=torch.int64, device="cuda:0") * 0x1E3779B97F4A7C15    # wraps
    return words.view(torch.uint8)[:n]


def test_copy_batch_segment_beyond_4_gib():
    # one segment whose byte offsets pass 2^32 (and whose chunk count passes 2^18), next to small
    # ones: offsets inside the kernel are 64-bit; the bytes behind each segment stay untouched
    big = (1 << 32) + (3 << 20) + 4096 + 5
    sizes = [4096, big, 70001]
    off, at = [], 0
    for n in sizes:
        off.append(at)
        at += (n + 255) // 256 * 256
    src = _counter_bytes(at)
    dst = torch.full((at,), 0xEE, dtype=torch.uint8, device="cuda:0")
    o64 = np.asarray(off, dtype=np.uint64)
    T.copy_batch(o64 + np.uint64(src.data_ptr()), o64 + np.uint64(dst.data_ptr()), np.asarray(sizes, dtype=np.uint64),
                 torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    for o, n in zip(off, sizes):
        assert torch.equal(dst[o:o + n], src[o:o + n])
        pad = (n + 255) // 256 * 256 - n
        assert bool((dst[o + n:o + n + pad] == 0xEE).all())


def test_pack_and_unpack_beyond_4_gib():
    # a slab of more than 2^32 bytes: tile starts, slab offsets and piece addresses are 64-bit
    rng = np.random.default_rng(9)
    sizes = ((1 << 20) + 16 * rng.integers(0, 4096, size=4200)).astype(np.uint64)
    sizes[7] += 5                                          # one ragged segment shifts the phase of all behind it
    src_off = np.concatenate([[0], np.cumsum((sizes + 255) // 256 * 256)[:-1]]).astype(np.uint64)
    slab_off = np.concatenate([[0], np.cumsum(sizes)[:-1]]).astype(np.uint64)
    total = int(sizes.sum())
    assert total > (1 << 32)
    src_total = int(src_off[-1] + sizes[-1])
    src = _counter_bytes(src_total)
    slab = torch.full((total,), 0xEE, dtype=torch.uint8, device="cuda:0")
    ptrs = _dev((src_off + np.uint64(src.data_ptr())).astype(np.int64))
    d_nb, d_off = _dev(sizes.astype(np.int64)), _dev(slab_off.astype(np.int64))
    st = torch.cuda.current_stream().cuda_stream
    d_index = torch.empty(T.pack_tiles(total), dtype=torch.int32, device="cuda:0")
    T.pack_index(d_off.data_ptr(), len(sizes), total, d_index.data_ptr(), st)
    T.pack(slab.data_ptr(), ptrs.data_ptr(), d_nb.data_ptr(), d_off.data_ptr(), len(sizes), total, st, d_index.data_ptr())
    torch.cuda.synchronize()
    for o, so, n in zip(src_off.tolist(), slab_off.tolist(), sizes.tolist()):
        assert torch.equal(slab[so:so + n], src[o:o + n])
    back = torch.full((src_total,), 0x55, dtype=torch.uint8, device="cuda:0")
    ptrs2 = _dev((src_off + np.uint64(back.data_ptr())).astype(np.int64))
    T.unpack(slab.data_ptr(), ptrs2.data_ptr(), d_nb.data_ptr(), d_off.data_ptr(), len(sizes), total, st, d_index.data_ptr())
    torch.cuda.synchronize()
    for i in list(range(0, len(sizes), 97)) + [7, 8, len(sizes) - 1]:
        o, n = int(src_off[i]), int(sizes[i])
        assert torch.equal(back[o:o + n], src[o:o + n])
        pad = (n + 255) // 256 * 256 - n
        if pad and i + 1 < len(sizes):
            assert bool((back[o + n:o + n + pad] == 0x55).all())


@pytest.mark.parametrize("shift", [0, 4, 1])
def test_pack_stress_shape_at_the_size_and_launch_the_bench_times(shift):
    # 4 GiB in 436 900 segments, tile index built once, one launch each way, as bench.py does it
    # (aligned, 4 bytes off, 1 byte off); sampled segments against the definition, one by one
    import bench
    L = bench.pack_stress_layout(torch, 4 << 30, shift)
    n, total = L["n"], L["total"]
    st = torch.cuda.current_stream().cuda_stream
    index = torch.empty(T.pack_tiles(total), dtype=torch.int32, device="cuda:0")
    T.pack_index(L["d_off"].data_ptr(), n, total, index.data_ptr(), st)
    L["slab"].fill_(0xEE)
    T.pack(L["slab"].data_ptr(), L["ptrs"].data_ptr(), L["d_bytes"].data_ptr(), L["d_off"].data_ptr(), n, total, st,
           index.data_ptr())
    torch.cuda.synchronize()
    rng = np.random.default_rng(shift)
    sample = sorted(set(rng.integers(0, n, size=300).tolist()) | {0, 1, n - 2, n - 1})
    for i in sample:
        o, so, k = int(L["slab_off"][i]), int(L["src_off"][i]), int(L["bytes"][i])
        piece = L["src"][so:so + k].cpu().numpy()
        want = po.pack([piece], np.asarray([0], dtype=np.uint64), np.zeros(k, dtype=np.uint8))
        assert np.array_equal(L["slab"][o:o + k].cpu().numpy(), want), (shift, i)
    # the way back, into a fresh image: sampled segments equal their slab pieces, the gaps stay
    back = torch.full_like(L["src"], 0x55)
    ptrs2 = _dev((L["src_off"] + np.uint64(back.data_ptr())).astype(np.int64))
    T.unpack(L["slab"].data_ptr(), ptrs2.data_ptr(), L["d_bytes"].data_ptr(), L["d_off"].data_ptr(), n, total, st,
             index.data_ptr())
    torch.cuda.synchronize()
    for i in sample:
        o, so, k = int(L["slab_off"][i]), int(L["src_off"][i]), int(L["bytes"][i])
        want = po.unpack(L["slab"][o:o + k].cpu().numpy(), np.asarray([k], dtype=np.uint64), np.asarray([0], dtype=np.uint64))[0]
        assert np.array_equal(back[so:so + k].cpu().numpy(), want), (shift, i)
    assert bool((back[:shift] == 0x55).all()) and bool((back[total + shift:] == 0x55).all())
    # and as a whole, on the device: every byte of the image came back
    assert torch.equal(back[shift:total + shift], L["src"][shift:total + shift])


def test_pack_and_copy_inside_a_captured_graph():
    # the stand-alone movers only launch kernels on the caller's stream (the copy's ticket counters
    # come from the stream-ordered allocator and are cleared by a kernel), so a caller may capture
    # them; every replay, with eager work and synchronisation between the replays, must give
    # what the eager call gives
    rng = np.random.default_rng(3)
    sizes = [4096, 100, 33000, 16384 * 2 + 48, 7, 12288]
    nb = np.asarray(sizes, dtype=np.uint64)
    src_off, src_total = _layout(rng, sizes, [0, 3, 16])
    slab_off, slab_total = _layout(rng, sizes, [0, 5])
    src = _dev(rng.integers(0, 256, size=src_total + 16, dtype=np.uint8))
    ptrs = _dev((src_off + np.uint64(src.data_ptr())).astype(np.int64))
    d_nb, d_off = _dev(nb.astype(np.int64)), _dev(slab_off.astype(np.int64))
    slab = torch.zeros(slab_total, dtype=torch.uint8, device="cuda:0")
    copy_dst = torch.zeros(src_total + 16, dtype=torch.uint8, device="cuda:0")
    seg = (np.asarray([src.data_ptr()], dtype=np.uint64), np.asarray([copy_dst.data_ptr()], dtype=np.uint64),
           np.asarray([(src_total + 16) // 16 * 16], dtype=np.uint64))
    st = torch.cuda.Stream()
    T.copy_batch(*seg, st.cuda_stream)                      # first use on the device: outside any capture
    st.synchronize()

    def want_now():
        tensors = [src[int(o):int(o) + int(k)].cpu().numpy() for o, k in zip(src_off, nb)]
        return po.pack(tensors, slab_off, np.zeros(slab_total, dtype=np.uint8)), src.cpu().numpy()[: int(seg[2][0])]

    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(st):
        with torch.cuda.graph(g, stream=st):
            T.pack(slab.data_ptr(), ptrs.data_ptr(), d_nb.data_ptr(), d_off.data_ptr(), len(sizes), slab_total, st.cuda_stream)
            T.copy_batch(*seg, st.cuda_stream)
    for replay in range(3):
        src.random_(0, 255)                                 # eager work between the replays
        slab.zero_()
        copy_dst.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        want_slab, want_copy = want_now()
        assert np.array_equal(slab.cpu().numpy(), want_slab), replay
        assert np.array_equal(copy_dst.cpu().numpy()[: len(want_copy)], want_copy), replay
