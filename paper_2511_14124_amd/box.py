"""What a GPU machine can hold of a file-tier configuration.

Configurations 4 and 5 (200 and 485 GiB of tensors) exceed one box, so they run
at a reduced layer count with the same tensor shapes.  This module derives that
count from the box instead of fixing it: free HBM, the host memory a command
may hold, and the free space of the directories the file tier is striped over.
bench.py and the GPU tests share it, so that the depth timed is the depth
checked against the oracle.  Only the library is used here (a dry replay with
its null mover tells which file extents a schedule really writes).
"""

import os
import shutil

import numpy as np

GiB = 1 << 30
FULL_LAYERS = (12, 24, 32, 40, 60)


def mem_available():
    try:
        with open("/proc/meminfo") as f:
            for line in f:
                if line.startswith("MemAvailable:"):
                    return int(line.split()[1]) * 1024
    except OSError:
        pass
    return 64 * GiB


def is_tmpfs(path):
    try:
        with open("/proc/mounts") as f:
            best, kind = "", ""
            rp = os.path.realpath(path)
            for line in f:
                _dev, mnt, fs = line.split()[:3]
                if (rp == mnt or rp.startswith(mnt.rstrip("/") + "/")) and len(mnt) > len(best):
                    best, kind = mnt, fs
            return kind in ("tmpfs", "ramfs")
    except OSError:
        return False


_pinned_limit = None

_PIN_PROBE = r"""
import ctypes as C, sys
hip = C.CDLL("libamdhip64.so")
hip.hipHostMalloc.argtypes = [C.POINTER(C.c_void_p), C.c_size_t, C.c_uint]
hip.hipHostFree.argtypes = [C.c_void_p]
GiB = 1 << 30
def holds(n):
    p = C.c_void_p()
    if hip.hipHostMalloc(C.byref(p), n * GiB, 0) != 0 or not p.value:
        return False
    hip.hipHostFree(p)
    return True
lo, hi = 1, max(2, int(sys.argv[1]))
if holds(hi):
    lo = hi
while hi - lo > 1:
    mid = (lo + hi) // 2
    if holds(mid):
        lo = mid
    else:
        hi = mid
print(lo)
"""


def pinned_limit():
    """Most page-locked host memory one process can hold here, found by trying (hipHostMalloc
    commits lazily, so a trial costs a second at most): boxes cap it well below their RAM (this
    pool's at about 66 GiB of 295).  Bisected to 1 GiB between 1 GiB and what the host has free,
    by a short-lived child process, so that whatever the trials leave behind in the runtime ends
    with it (a process that had just freed a 65 GiB trial region was refused its next, small
    pinned allocation).  Measured once per process; TC_PINNED_LIMIT_GIB overrides it."""
    global _pinned_limit
    if _pinned_limit is not None:
        return _pinned_limit
    import subprocess
    import sys
    env = os.environ.get("TC_PINNED_LIMIT_GIB")
    if env:
        _pinned_limit = int(float(env) * GiB)
        return _pinned_limit
    top = max(2, min(mem_available(), 250 * GiB) // GiB)
    try:
        out = subprocess.run([sys.executable, "-c", _PIN_PROBE, str(top)], capture_output=True, text=True, timeout=120)
        _pinned_limit = int(out.stdout.strip().splitlines()[-1]) * GiB
    except (subprocess.SubprocessError, ValueError, IndexError):
        _pinned_limit = 32 * GiB                     # could not be measured: a figure every box of this kind grants
    return _pinned_limit


def box_limits(torch, tier_dirs):
    """What bounds a file-tier configuration on this machine: HBM free, host memory a command may
    hold (at most 250 GiB whatever the box has, 220 GiB if part of the file tier is itself in
    memory: a run that exhausts the host loses the box), and
    free space in the directories the file tier is striped over."""
    free_hbm, _total = torch.cuda.mem_get_info()
    dirs = []
    for d in tier_dirs:
        dirs.append({"dir": d, "free": shutil.disk_usage(d).free, "in_memory": is_tmpfs(d)})
    # a tier directory in memory is unreclaimable like the pinned pools: leave more of the box alone
    cap = (220 if any(d["in_memory"] for d in dirs) else 250) * GiB
    return {"hbm_free": int(free_hbm), "host_memory": int(min(mem_available(), cap)), "pinned": int(pinned_limit()),
            "tier_dirs": dirs}


def file_tier_need(T, wl):
    """Bytes of the file tier a replay really occupies: the extents of the NVMe-final tensors plus
    those of every tensor the schedule ever spills or writes back (the files are sparse, an extent
    that is never written takes no space).  Found by a dry replay with the library's null mover:
    the decision kernel runs, no byte moves."""
    tc = T.TensorCache.from_workload(wl)
    tc.bind_torch(null_mover=True)
    for steps in wl.iterations:
        tc.replay_iteration_c(steps, 0)
    ops = tc.dump_oplog()
    written = set(np.nonzero(tc.placement["final_tier"] == T.NVME)[0].tolist())
    to_file = (ops["dst_tier"] == T.NVME) & (ops["bytes"] > 0)
    written |= set(ops["tensor"][to_file].tolist())
    plan = {"hbm_total": int(tc.plan.hbm_total), "host_total": int(tc.plan.host_total)}
    tc.close()
    need = sum((int(wl.tensor_bytes[t]) + 4095) // 4096 * 4096 for t in written)
    return need, plan


def depth_the_box_holds(T, W, index, limits, staging_depth):
    """Largest layer count of configuration `index` this box holds, and the arithmetic:
      HBM   : pool region + 2 GiB for the library's tables and PyTorch      <= 92 % of free HBM
      pinned: pinned pools + staging ring + 3 GiB                           <= what one process may pin
      host  : pinned pools + staging ring + the in-memory share of the file tier + 24 GiB
              (page cache in motion, the process itself)                     <= host memory
      files : file-tier bytes / number of directories                        <= free space of each
              directory less 12 GiB (directories in memory: bounded by the host line instead)
    The file tier is striped evenly over its directories, so each takes the same share."""
    full = FULL_LAYERS[index]
    dirs = limits["tier_dirs"]
    n_dirs = max(1, len(dirs))

    def fits(L):
        wl = W.config(index, layers=L)
        need, plan = file_tier_need(T, wl)
        big = (int(wl.tensor_bytes.max()) + 4095) // 4096 * 4096
        share = need / n_dirs
        in_mem = sum(share for d in dirs if d["in_memory"])
        rows = {"layers": L, "hbm_pool_GiB": plan["hbm_total"] / GiB, "pinned_pool_GiB": plan["host_total"] / GiB,
                "staging_GiB": staging_depth * big / GiB, "file_tier_GiB": need / GiB,
                "file_tier_in_memory_GiB": in_mem / GiB}
        ok = plan["hbm_total"] + 2 * GiB <= 0.92 * limits["hbm_free"]
        ok = ok and plan["host_total"] + staging_depth * big + 3 * GiB <= limits["pinned"]
        ok = ok and plan["host_total"] + staging_depth * big + in_mem + 24 * GiB <= limits["host_memory"]
        for d in dirs:
            if not d["in_memory"]:
                ok = ok and share <= d["free"] - 12 * GiB
        return ok, rows

    lo, hi, best = 1, full, None
    ok, rows = fits(full)
    if ok:
        return full, rows
    while lo <= hi:
        mid = (lo + hi) // 2
        ok, rows = fits(mid)
        if ok:
            best, lo = (mid, rows), mid + 1
        else:
            hi = mid - 1
    if best is None:
        raise SystemExit(f"configuration {index + 1} does not fit this box even one layer deep")
    return best
