"""What pre-allocated buffer pools save (the paper's "+M" step, Sec. 3.3 and 4.1.4).

Run as `python -m paper_2511_14124_amd.alloc_probe` on a GPU.  The library never
allocates on the hot path; a design without pools would take a pinned host
buffer for every tensor it evicts and a GPU buffer for every tensor it fetches,
and give them back afterwards.  This probe replays one iteration of a workload
with the null mover (decisions only), counts the evictions and fetches per size
class in the op log, times hipHostMalloc + hipHostFree and hipMalloc + hipFree
for each size, and prints what those calls would add to the iteration.
"""

from __future__ import annotations

import argparse
import ctypes as C
import time

import numpy as np


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=1)
    ap.add_argument("--reps", type=int, default=5)
    args = ap.parse_args()
    import torch
    import workloads as W
    from . import binding as T
    T.load_library()
    torch.cuda.init()
    hip = C.CDLL("libamdhip64.so")
    hip.hipHostMalloc.argtypes = [C.POINTER(C.c_void_p), C.c_size_t, C.c_uint]
    hip.hipHostFree.argtypes = [C.c_void_p]
    hip.hipMalloc.argtypes = [C.POINTER(C.c_void_p), C.c_size_t]
    hip.hipFree.argtypes = [C.c_void_p]

    wl = W.config(args.config)
    tc = T.TensorCache.from_workload(wl)
    tc.bind_torch(null_mover=True)
    tc.replay_iteration_c(wl.iterations[0], 0)
    log = tc.dump_oplog()
    tc.close()
    evict = log[log["op"] == T.OP_NAMES.index("EVICT")]
    fetch = log[(log["op"] == T.OP_NAMES.index("PREFETCH")) | (log["op"] == T.OP_NAMES.index("DEMAND"))]

    def cost(alloc, free, size):
        best = 1e9
        for _ in range(args.reps):
            p = C.c_void_p()
            t0 = time.perf_counter()
            assert alloc(p, size) == 0
            assert free(p) == 0
            best = min(best, time.perf_counter() - t0)
        return best

    host_alloc = lambda p, n: hip.hipHostMalloc(C.byref(p), n, 0)
    dev_alloc = lambda p, n: hip.hipMalloc(C.byref(p), n)
    print(f"{wl.name}: one iteration evicts {len(evict)} tensors and fetches {len(fetch)}")
    print(f"{'bytes':>12} {'evictions':>10} {'pinned alloc+free us':>22} {'fetches':>9} {'HBM alloc+free us':>19}")
    total_host = total_dev = 0.0
    for size in sorted(set(evict["bytes"].tolist()) | set(fetch["bytes"].tolist())):
        ne, nf = int((evict["bytes"] == size).sum()), int((fetch["bytes"] == size).sum())
        ch = cost(host_alloc, hip.hipHostFree, int(size)) if ne else 0.0
        cd = cost(dev_alloc, hip.hipFree, int(size)) if nf else 0.0
        total_host += ne * ch
        total_dev += nf * cd
        print(f"{int(size):>12} {ne:>10} {ch * 1e6:>22.1f} {nf:>9} {cd * 1e6:>19.1f}", flush=True)
    print(f"per iteration: {total_host * 1e3:.1f} ms of pinned allocation + {total_dev * 1e3:.1f} ms of HBM allocation "
          f"that the pools avoid (best of {args.reps} per size, nothing else running)")


if __name__ == "__main__":
    main()
