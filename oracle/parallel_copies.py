"""The oracle's byte movement, replayed with one thread per core.

TEST INFRASTRUCTURE ONLY, like the rest of this package: the benchmark's
cpu_baseline leg reports it beside the single-threaded oracle so that one core's
memcpy rate is not mistaken for the host's limit.

It adds no method arithmetic.  The decisions are the oracle's own: an op log
produced by `tc_oracle.Replay` is taken as given and only its copies are
carried out again, in log order, over plain byte arrays laid out as the
oracle's tiers are (same offsets, same strides), each copy cut into equal
slices that a pool of threads moves concurrently.  An eviction followed by the
fetch into the GPU buffer it leaves is done the way the oracle's full-bytes
mode does it: the incoming bytes are read first (the two tensors may swap host
buffers), then the outgoing copy, then the incoming bytes land.
"""

from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from typing import List

import numpy as np

from . import tc_oracle as o


class Tiers:
    """Three byte arrays laid out like a full-bytes Replay's."""

    def __init__(self, r: o.Replay, payload=None):
        self.r = r
        self.hbm = np.zeros(r.plan.gpu_total, dtype=np.uint8)
        self.host = np.zeros(r.plan.cpu_total, dtype=np.uint8)
        self.file = np.zeros(r.pl.file_total, dtype=np.uint8)
        if payload is not None:
            for t in range(r.p.n_tensors):
                self.view(t, r.pl.final[t], r.pl.slot[t])[:] = payload(t)

    def view(self, t: int, tier: int, slot: int) -> np.ndarray:
        r = self.r
        s, n = r.p.class_of[t], r.bytes_of[t]
        if tier == o.GPU:
            a = r.plan.gpu_off[s] + slot * r.plan.stride[s]
            return self.hbm[a:a + n]
        if tier == o.CPU:
            a = r.plan.cpu_off[s] + slot * r.plan.stride[s]
            return self.host[a:a + n]
        a = r.pl.file_off[t]
        return self.file[a:a + n]


def replay_copies(tiers: Tiers, log: List[o.Op], threads: int) -> int:
    """Carries out the copies of `log` over `tiers`; returns the bytes copied into the HBM array."""
    pool = ThreadPoolExecutor(max_workers=threads)

    def copy(dst: np.ndarray, src: np.ndarray) -> None:
        n = dst.shape[0]
        if n < (1 << 16) or threads == 1:
            np.copyto(dst, src)
            return
        cut = [n * k // threads for k in range(threads + 1)]
        futs = [pool.submit(np.copyto, dst[a:b], src[a:b]) for a, b in zip(cut[:-1], cut[1:]) if b > a]
        for f in futs:
            f.result()

    into_hbm = 0
    i = 0
    try:
        while i < len(log):
            e = log[i]
            op, t = e[3], e[4]
            nxt = log[i + 1] if i + 1 < len(log) else None
            leaves_gpu = op in (o.EVICT, o.WRITEBACK) and e[5] == o.GPU
            if leaves_gpu and nxt is not None and nxt[3] in (o.PREFETCH, o.DEMAND) and nxt[:3] == e[:3] \
                    and nxt[8] == e[6] and tiers.r.p.class_of[nxt[4]] == tiers.r.p.class_of[t]:
                u = nxt[4]
                incoming = np.empty(tiers.r.bytes_of[u], dtype=np.uint8)
                copy(incoming, tiers.view(u, nxt[5], nxt[6]))
                copy(tiers.view(t, e[7], e[8]), tiers.view(t, e[5], e[6]))
                copy(tiers.view(u, o.GPU, nxt[8]), incoming)
                into_hbm += incoming.shape[0]
                i += 2
                continue
            if op in (o.EVICT, o.WRITEBACK, o.SPILL, o.RESTORE, o.PREFETCH, o.DEMAND):
                copy(tiers.view(t, e[7], e[8]), tiers.view(t, e[5], e[6]))
                if e[7] == o.GPU:
                    into_hbm += tiers.r.bytes_of[t]
            i += 1                                   # RELEASE, FAIL: no bytes move
    finally:
        pool.shutdown()
    return into_hbm
