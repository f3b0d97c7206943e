"""The host link's measured peak: what the benchmark divides the migration rate by.

`measure_link_peak` times pinned hipMemcpyAsync copies of 1 GiB host->HBM,
HBM->host, and both at once on two streams, straight through the HIP runtime.
"""

from __future__ import annotations

import time


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

    # The runtime gives a stream its DMA engine at the stream's first copy, among the engines idle at
    # that moment, and keeps it: the two streams must make their first copies AT ONCE, or they share
    # one engine and the two directions take turns for good (28.7 instead of 48.6 GB/s per direction).
    out = {"duplex_each": run(h2d, d2h)}      # bytes per direction / time with both running
    out["h2d"], out["d2h"] = run(h2d), run(d2h)
    # for context (the paper's Table 2 sets pinned against pageable host memory, which the driver
    # stages through a buffer of its own): the same host->HBM copy from pageable memory
    n_page = min(nbytes, 256 << 20)
    pageable = torch.empty(n_page, dtype=torch.uint8)
    pageable.fill_(4)
    best = 0.0
    for _ in range(3):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        d1[:n_page].copy_(pageable)
        torch.cuda.synchronize()
        best = max(best, n_page / (time.perf_counter() - t0) / 1e9)
    out["h2d_from_pageable_memory"] = best
    hip.hipStreamDestroy(s1)
    hip.hipStreamDestroy(s2)
    del h1, h2, d1, d2
    return out
