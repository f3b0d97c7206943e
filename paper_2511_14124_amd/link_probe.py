"""Host-link probe: what the PCIe link of this box gives the migration path.

Run as `python -m paper_2511_14124_amd.link_probe`.  Prints, in GB/s:

1. pinned hipMemcpyAsync host->HBM, HBM->host, and both at once on two streams
   (the "measured PCIe peak" the benchmark divides by);
2. the library's batched copy / exchange kernel over the same link, one launch
   per line: host->HBM only, HBM->host only, and exchange units (a tensor
   leaves a GPU buffer for a pinned buffer while another arrives), by unit size;
3. the exchange kernel by launch size (what a launch of a few MiB loses);
4. the exchange kernel by the number of working workgroups (all on one XCD)
   and by chunk size;
5. the exchange kernel while another stream runs small kernels the host waits
   for one by one (what a decision launch per hook call does to a running
   migration launch).

The numbers justify the defaults of the library (12 workgroups on one XCD,
16 KiB chunks, zero-copy kernel instead of DMA-engine copies, decisions in
windows).
"""

from __future__ import annotations

import time

import numpy as np


def measure_link_peak(torch, nbytes: int = 1 << 30, reps: int = 5) -> dict:
    """Best-of-N pinned hipMemcpyAsync H2D, D2H, and both at once on two
    streams (GB/s per direction).  The copies are issued straight through the
    HIP runtime on streams created here."""
    import ctypes as C
    hip = C.CDLL("libamdhip64.so")
    hip.hipMemcpyAsync.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int, C.c_void_p]
    hip.hipStreamCreateWithFlags.argtypes = [C.POINTER(C.c_void_p), C.c_uint]
    hip.hipStreamSynchronize.argtypes = [C.c_void_p]
    hip.hipStreamDestroy.argtypes = [C.c_void_p]
    H2D, D2H, NONBLOCKING = 1, 2, 1
    dev = torch.device("cuda:0")
    h1 = torch.empty(nbytes, dtype=torch.uint8, pin_memory=True)
    h2 = torch.empty(nbytes, dtype=torch.uint8, pin_memory=True)
    d1 = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    d2 = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    h1.fill_(1)
    h2.fill_(2)
    d2.fill_(3)
    s1, s2 = C.c_void_p(), C.c_void_p()
    assert hip.hipStreamCreateWithFlags(C.byref(s1), NONBLOCKING) == 0
    assert hip.hipStreamCreateWithFlags(C.byref(s2), NONBLOCKING) == 0

    def h2d():
        assert hip.hipMemcpyAsync(d1.data_ptr(), h1.data_ptr(), nbytes, H2D, s1) == 0

    def d2h():
        assert hip.hipMemcpyAsync(h2.data_ptr(), d2.data_ptr(), nbytes, D2H, s2) == 0

    def run(*fns):
        best = 0.0
        for _ in range(reps):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for fn in fns:
                fn()
            assert hip.hipStreamSynchronize(s1) == 0 and hip.hipStreamSynchronize(s2) == 0
            best = max(best, nbytes / (time.perf_counter() - t0) / 1e9)
        return best

    out = {"h2d": run(h2d), "d2h": run(d2h)}
    out["duplex_each"] = run(h2d, d2h)        # bytes per direction / time with both running
    hip.hipStreamDestroy(s1)
    hip.hipStreamDestroy(s2)
    del h1, h2, d1, d2
    return out


def main():
    import torch
    from . import binding as T
    T.load_library()
    link = measure_link_peak(torch)
    print(f"hipMemcpyAsync pinned, 1 GiB: H2D {link['h2d']:.2f}  D2H {link['d2h']:.2f}  "
          f"both at once {link['duplex_each']:.2f} per direction", flush=True)

    G, M = 1 << 30, 1 << 20
    dev = torch.device("cuda:0")
    pinned = torch.empty(2 * G, dtype=torch.uint8, pin_memory=True)
    hbm = torch.empty(2 * G, dtype=torch.uint8, device=dev)
    pinned.fill_(7)
    hbm.fill_(9)
    st = torch.cuda.Stream()
    P, H = pinned.data_ptr(), hbm.data_ptr()

    def timed(fn, reps=3):
        best = 1e9
        for _ in range(reps):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            fn()
            torch.cuda.synchronize()
            best = min(best, time.perf_counter() - t0)
        return best

    def units(size, total=G, cap=48):
        n = max(1, min(cap, total // size))
        off = np.arange(n, dtype=np.uint64) * np.uint64(size)
        return off, np.full(n, size, dtype=np.uint64)

    def exchange(size, wg=0, chunk=0, total=G):
        off, nb = units(size, total)
        # out: HBM half 0 -> pinned half 0 (swap in place with in: pinned half 0 -> HBM half 0)
        dt = timed(lambda: T.exchange_batch(off + np.uint64(H), off + np.uint64(P), off + np.uint64(P),
                                            off + np.uint64(H), nb, st.cuda_stream, wg, chunk))
        return float(nb.sum()) / dt / 1e9

    def oneway(size, h2d, wg=0, chunk=0):
        off, nb = units(size)
        src, dst = (P, H) if h2d else (H, P)
        dt = timed(lambda: T.copy_batch(off + np.uint64(src), off + np.uint64(dst), nb, st.cuda_stream, wg, chunk))
        return float(nb.sum()) / dt / 1e9

    import ctypes as C
    hip = C.CDLL("libamdhip64.so")
    hip.hipMemcpyAsync.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int, C.c_void_p]

    def dma(size, h2d):
        """The same units as one hipMemcpyAsync each, back to back on one stream."""
        off, nb = units(size)
        src, dst, kind = (P, H, 1) if h2d else (H, P, 2)

        def fn():
            for o, n in zip(off.tolist(), nb.tolist()):
                assert hip.hipMemcpyAsync(dst + o, src + o, n, kind, st.cuda_stream) == 0
        return float(nb.sum()) / timed(fn) / 1e9

    print("\nup to 48 units of one size: one launch of the batched kernel against one hipMemcpyAsync per unit"
          "\n(GB/s per direction):")
    print(f"{'unit':>10} {'units':>6} {'H2D only':>10} {'D2H only':>10} {'exchange':>10} {'DMA H2D':>10} {'DMA D2H':>10}")
    for size in (64 << 10, 1 * M, 4 * M, 16 * M, 64 * M, 256 * M, G):
        n = max(1, min(48, G // size))
        print(f"{size >> 10:>8}Ki {n:>6} {oneway(size, True):>10.2f} {oneway(size, False):>10.2f} {exchange(size):>10.2f}"
              f" {dma(size, True):>10.2f} {dma(size, False):>10.2f}", flush=True)

    print("\nexchange, one launch of 4 units, by bytes per direction (GB/s per direction; the call's own"
          "\nstream-ordered allocation of the ticket counters is inside the time):")
    for total in (1 * M, 2 * M, 4 * M, 8 * M, 16 * M, 32 * M, 64 * M, 256 * M):
        print(f"  {total >> 20:>5} MiB {exchange(total // 4, total=total):8.2f}", flush=True)
    print("\nexchange of 16 x 64 MiB by working workgroups (GB/s per direction):")
    for wg in (4, 8, 12, 16, 24, 32, 64, 256):
        print(f"  {wg:>5} workgroups {exchange(64 * M, wg):8.2f}", flush=True)
    print("\nexchange of 16 x 64 MiB by chunk size (12 workgroups):")
    for chunk in (4096, 16384, 65536, 262144, 1 << 20):
        print(f"  {chunk >> 10:>5} KiB chunks {exchange(64 * M, 12, chunk):8.2f}", flush=True)

    # a stream of small kernels the host waits for, while eight 1 GiB exchange launches run
    side = torch.cuda.Stream()
    x = torch.zeros(64, device=dev)
    off, nb = units(64 * M)

    def eight():
        for _ in range(8):
            T.exchange_batch(off + np.uint64(H), off + np.uint64(P), off + np.uint64(P), off + np.uint64(H), nb,
                             st.cuda_stream)

    def with_side(n_small, sync_each):
        def fn():
            eight()
            with torch.cuda.stream(side):
                for _ in range(n_small):
                    x.add_(1)
                    if sync_each:
                        side.synchronize()
        return 8.0 * float(nb.sum()) / timed(fn, reps=2) / 1e9

    print("\neight exchange launches of 1 GiB while another stream runs small kernels (GB/s per direction):")
    print(f"  nothing else running                     {with_side(0, False):8.2f}")
    print(f"  400 small kernels, host waits for none   {with_side(400, False):8.2f}")
    print(f"  400 small kernels, host waits for each   {with_side(400, True):8.2f}")
    print(f"  1600 small kernels, host waits for each  {with_side(1600, True):8.2f}", flush=True)

    # the other way round: what the copies cost compute that runs beside them.  A fixed burst
    # of bf16 GEMMs (8192 x 8192 x 8192, forty of them) on the current stream, alone and with
    # 2 GiB crossing the link per direction meanwhile, by the zero-copy kernel or by DMA copies
    a = torch.randn(8192, 8192, device=dev, dtype=torch.bfloat16)
    b = torch.randn(8192, 8192, device=dev, dtype=torch.bfloat16)
    c = torch.empty(8192, 8192, device=dev, dtype=torch.bfloat16)
    gb = 128 * M
    hbm2 = torch.empty(gb, dtype=torch.uint8, device=dev)
    pin_in = torch.empty(gb, dtype=torch.uint8).pin_memory()
    pin_out = torch.empty(gb, dtype=torch.uint8).pin_memory()
    side2 = torch.cuda.Stream()
    one = np.asarray([gb], dtype=np.uint64)
    p_h, p_i, p_o = (np.asarray([t.data_ptr()], dtype=np.uint64) for t in (hbm2, pin_in, pin_out))

    def gemms(copies):
        # time on the GEMMs' own stream (events), so that copies outlasting them do not count
        best = 1e9
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for _ in range(3):
            torch.cuda.synchronize()
            copies()
            e0.record()
            for _ in range(40):
                torch.matmul(a, b, out=c)
            e1.record()
            torch.cuda.synchronize()
            best = min(best, e0.elapsed_time(e1) * 1e-3)
        return best

    def by_kernel(n, both):
        def go():
            for _ in range(n):
                if both:
                    T.exchange_batch(p_h, p_o, p_i, p_h, one, side.cuda_stream)
                else:
                    T.copy_batch(p_i, p_h, one, side.cuda_stream)
        return go

    def by_dma(n, both):
        def go():
            for _ in range(n):
                with torch.cuda.stream(side):
                    hbm2.copy_(pin_in, non_blocking=True)
                if both:
                    with torch.cuda.stream(side2):
                        pin_out.copy_(hbm2, non_blocking=True)
        return go

    alone = gemms(lambda: None)
    print(f"\nforty bf16 GEMMs of 8192^3 ({40 * 2 * 8192**3 / alone / 1e12:.0f} TFLOP/s alone, {alone * 1e3:.1f} ms), and beside them:")
    for name, go in (("16 x 128 MiB host to HBM by the kernel", by_kernel(16, False)),
                     ("16 x 128 MiB each way by the kernel (exchange)", by_kernel(16, True)),
                     ("16 x 128 MiB host to HBM by DMA copies", by_dma(16, False)),
                     ("16 x 128 MiB each way by DMA copies", by_dma(16, True))):
        t = gemms(go)
        print(f"  {name:50s} {t * 1e3:7.1f} ms  (+{(t - alone) * 1e3:4.1f} ms, +{100.0 * (t - alone) / alone:4.1f} %)", flush=True)


if __name__ == "__main__":
    main()
