"""ctypes binding of libtc.so.  Names follow include/tc.h one to one."""

from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libtc.so")

GPU, CPU, NVME = 0, 1, 2
PRE, POST, END, END_CPU = 0, 1, 2, 3
OP_NAMES = ["DEMAND", "PREFETCH", "EVICT", "RELEASE", "WRITEBACK", "SPILL", "RESTORE", "FAIL", "ALLOC"]
LITERAL_ALG2 = 1
NO_PREFETCH = 2
SMALLEST_FIRST = 4
ALLOC_WRITE_ONLY = 8
BIND_NULL_MOVER = 1
BIND_FILE_DIRECT = 2
BIND_HOST_TIER = 4
NONE = 0xFFFFFFFF
MAX_STEP_TENSORS = 64

TENSOR_DESC = np.dtype([("bytes", "<u8"), ("group", "u1"), ("kind", "u1"), ("pad_", "u1", (6,))])
EVENT = np.dtype([("step", "<u4"), ("tensor", "<u4"), ("compute_ns", "<u8"), ("rw", "u1"), ("pad_", "u1", (7,))])
POOL_CLASS = np.dtype([("bytes", "<u8"), ("stride", "<u8"), ("hbm_off", "<u8"), ("host_off", "<u8"),
                       ("group", "<u4"), ("count", "<u4"), ("used", "<u4"), ("step_max", "<u4"),
                       ("gpu_count", "<u4"), ("cpu_count", "<u4")])
PLACEMENT = np.dtype([("file_off", "<u8"), ("cls", "<u4"), ("slot", "<u4"), ("first_use", "<u4"),
                      ("final_tier", "u1"), ("pad_", "u1", (3,))])
OP = np.dtype([("iteration", "<u4"), ("step", "<u4"), ("tensor", "<u4"), ("src_slot", "<u4"),
               ("dst_slot", "<u4"), ("phase", "u1"), ("op", "u1"), ("src_tier", "u1"), ("dst_tier", "u1"),
               ("bytes", "<u8")])
SEGMENT = np.dtype([("src", "<u8"), ("dst", "<u8"), ("bytes", "<u8")])

assert TENSOR_DESC.itemsize == 16 and EVENT.itemsize == 24 and POOL_CLASS.itemsize == 56
assert PLACEMENT.itemsize == 24 and OP.itemsize == 32 and SEGMENT.itemsize == 24


class Budget(C.Structure):
    _fields_ = [("hbm_bytes", C.c_uint64), ("host_bytes", C.c_uint64 * 2), ("align", C.c_uint32), ("flags", C.c_uint32)]


class PoolPlan(C.Structure):
    _fields_ = [("n_classes", C.c_uint32), ("n_rows", C.c_uint32), ("n_steps", C.c_uint32), ("pad_", C.c_uint32),
                ("hbm_total", C.c_uint64), ("host_total", C.c_uint64), ("file_total", C.c_uint64)]


class Stats(C.Structure):
    _fields_ = [("hits", C.c_uint64), ("misses", C.c_uint64), ("fails", C.c_uint64), ("n_ops", C.c_uint64 * 8),
                ("bytes_h2d", C.c_uint64), ("bytes_d2h", C.c_uint64),
                ("bytes_file_read", C.c_uint64), ("bytes_file_write", C.c_uint64),
                ("file_read_ns", C.c_uint64), ("file_write_ns", C.c_uint64),
                ("mover_launches", C.c_uint64), ("mover_units", C.c_uint64), ("dma_copies", C.c_uint64),
                ("decide_launches", C.c_uint64),
                ("hbm_budget", C.c_uint64), ("hbm_pool_bytes", C.c_uint64),
                ("host_budget", C.c_uint64), ("host_pool_bytes", C.c_uint64),
                ("stall_ns", C.c_uint64), ("waits_under_30us", C.c_uint64), ("waits_total", C.c_uint64),
                ("waits_under_10us", C.c_uint64), ("waits_under_100us", C.c_uint64),
                ("cursor", C.c_uint32), ("iteration", C.c_uint32),
                ("n_alloc", C.c_uint64), ("bytes_not_fetched", C.c_uint64), ("undefined_reads", C.c_uint64),
                ("host_blocked_ns", C.c_uint64 * 4)]


class Timing(C.Structure):
    _fields_ = [("kernel_ns", C.c_double), ("kernel_launches", C.c_uint64), ("kernel_bytes", C.c_uint64),
                ("h2d_ns", C.c_double), ("h2d_copies", C.c_uint64), ("h2d_bytes", C.c_uint64),
                ("d2h_ns", C.c_double), ("d2h_copies", C.c_uint64), ("d2h_bytes", C.c_uint64),
                ("decide_ns", C.c_double), ("decide_launches", C.c_uint64), ("decide_calls", C.c_uint64)]


STATS_FIELDS = [f[0] for f in Stats._fields_]

_lib = None


class TcError(RuntimeError):
    def __init__(self, code: int, detail: str = ""):
        self.code = code
        name = lib().tc_strerror(code).decode() if _lib is not None else str(code)
        super().__init__(f"tc error {code} ({name}): {detail}")


def load_library(path: str = LIB_PATH):
    """Loads libtc.so.  There is no fallback: without the built library the
    product path does not exist."""
    global _lib
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} is missing: run `python -m paper_2511_14124_amd.build` first")
    try:
        # PyTorch ships its own HIP runtime under the same library name.  Whichever copy is
        # loaded first serves the whole process, and the device memory and streams handed to
        # the library come from PyTorch: let PyTorch's copy be that one.
        import torch  # noqa: F401
    except ImportError:
        pass
    L = C.CDLL(path)
    vp, u32, u64, i32 = C.c_void_p, C.c_uint32, C.c_uint64, C.c_int
    sig = {
        "tc_strerror": (C.c_char_p, [i32]),
        "tc_last_error": (C.c_char_p, [vp]),
        "tc_create": (i32, [C.POINTER(vp)]),
        "tc_destroy": (i32, [vp]),
        "tc_profile_order": (i32, [vp, vp, u32, vp, u64]),
        "tc_plan_pools": (i32, [vp, C.POINTER(Budget), C.POINTER(PoolPlan), vp, u32]),
        "tc_plan_schedule": (i32, [vp, vp]),
        "tc_bind_memory": (i32, [vp, vp, u64, vp, u64, vp, u64, i32, vp, u32]),
        "tc_load_tensor": (i32, [vp, u32, vp]),
        "tc_fill_payload": (i32, [vp, u32]),
        "tc_read_tensor": (i32, [vp, u32, vp]),
        "tc_migrate_step": (i32, [vp, u32, i32, vp, vp, u32, vp, vp]),
        "tc_end_iteration": (i32, [vp, vp]),
        "tc_emulate_compute": (i32, [vp, vp, u64]),
        "tc_set_stall_measurement": (i32, [vp, i32]),
        "tc_stall_by_step": (i32, [vp, vp, u32, i32]),
        "tc_replay_iteration": (i32, [vp, vp, vp, vp, u32, vp, vp, i32]),
        "tc_synchronize": (i32, [vp]),
        "tc_cache_stats": (i32, [vp, C.POINTER(Stats)]),
        "tc_dump_oplog": (i32, [vp, u64, vp, u64, C.POINTER(u64)]),
        "tc_dump_state": (i32, [vp, vp, vp, vp]),
        "tc_set_oplog": (i32, [vp, i32, i32]),
        "tc_set_mover": (i32, [vp, u32, u32]),
        "tc_mover_timing": (i32, [vp, i32, C.POINTER(Timing)]),
        "tc_set_dma_threshold": (i32, [vp, u64]),
        "tc_set_merge_bytes": (i32, [vp, u64]),
        "tc_set_dma_policy": (i32, [vp, i32]),
        "tc_set_gpu_dependencies": (i32, [vp, i32, u32]),
        "tc_tune_mover": (i32, [vp, C.POINTER(u32)]),
        "tc_set_io_threads": (i32, [vp, u32, u32]),
        "tc_add_stripe": (i32, [vp, i32]),
        "tc_set_io_chunk": (i32, [vp, u64]),
        "tc_set_replay_window": (i32, [vp, u32]),
        "tc_set_decide_ahead": (i32, [vp, u32]),
        "tc_copy_batch": (i32, [vp, u32, vp, u32, u32]),
        "tc_exchange_batch": (i32, [vp, vp, u32, vp, u32, u32]),
        "tc_pack_tiles": (u64, [u64]),
        "tc_pack_index": (i32, [vp, u32, u64, vp, vp]),
        "tc_pack": (i32, [vp, vp, vp, vp, u32, u64, vp, vp]),
        "tc_unpack": (i32, [vp, vp, vp, vp, u32, u64, vp, vp]),
        "tc_pack_static": (i32, [vp, vp, vp, vp, u32, u64, i32, vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype = res
        fn.argtypes = args
    _lib = L
    return L


def lib():
    return _lib if _lib is not None else load_library()


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


class _PinnedRegion:
    """Page-locked host memory from hipHostMalloc, freed explicitly."""

    _hip = None

    def __init__(self, nbytes: int):
        if _PinnedRegion._hip is None:
            hip = C.CDLL("libamdhip64.so")
            hip.hipHostMalloc.argtypes = [C.POINTER(C.c_void_p), C.c_size_t, C.c_uint]
            hip.hipHostFree.argtypes = [C.c_void_p]
            _PinnedRegion._hip = hip
        p = C.c_void_p()
        rc = _PinnedRegion._hip.hipHostMalloc(C.byref(p), int(nbytes), 0)
        if rc != 0 or not p.value:
            raise MemoryError(f"hipHostMalloc of {nbytes} bytes failed (HIP error {rc})")
        self.ptr, self.nbytes = int(p.value), int(nbytes)

    def data_ptr(self) -> int:
        return self.ptr

    def free(self):
        if self.ptr:
            _PinnedRegion._hip.hipHostFree(C.c_void_p(self.ptr))
            self.ptr = 0

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


class TensorCache:
    """One context of the library (one GPU).  Methods mirror the C calls."""

    def __init__(self):
        self._h = C.c_void_p()
        rc = lib().tc_create(C.byref(self._h))
        if rc:
            raise TcError(rc)
        self.n_tensors = 0
        self.n_steps = 0
        self._keep = []          # torch tensors / buffers that must outlive the context

    def close(self):
        if self._h:
            lib().tc_destroy(self._h)
            self._h = C.c_void_p()
        if getattr(self, "_fd", -1) >= 0:
            os.close(self._fd)
            self._fd = -1
        for sfd in getattr(self, "_stripe_fds", []):
            os.close(sfd)
        self._stripe_fds = []
        if self._keep:
            # regions bind_torch allocated: hand them back to the system, not to
            # PyTorch's caches (a pinned region can be tens of GiB)
            for r in self._keep:
                if isinstance(r, _PinnedRegion):
                    r.free()
            self._keep = []
            self.hbm = self.pinned = self.staging = self.mstream = None
            import torch
            torch.cuda.empty_cache()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc: int):
        if rc:
            raise TcError(rc, lib().tc_last_error(self._h).decode())

    # -- planning --------------------------------------------------------------
    def profile_order(self, tensor_bytes, tensor_group, ev_step, ev_tensor, ev_rw, ev_ns=None, tensor_kind=None):
        n_t = len(tensor_bytes)
        t = np.zeros(n_t, dtype=TENSOR_DESC)
        t["bytes"] = tensor_bytes
        t["group"] = tensor_group
        if tensor_kind is not None:
            t["kind"] = tensor_kind
        ev = np.zeros(len(ev_step), dtype=EVENT)
        ev["step"] = ev_step
        ev["tensor"] = ev_tensor
        ev["rw"] = ev_rw
        if ev_ns is not None:
            ev["compute_ns"] = ev_ns
        self._check(lib().tc_profile_order(self._h, _ptr(t), n_t, _ptr(ev), len(ev)))
        self.n_tensors = n_t
        self.tensor_bytes = np.asarray(tensor_bytes, dtype=np.uint64)

    def plan_pools(self, hbm_bytes: int, host_bytes: Sequence[int], align: int = 256, flags: int = 0):
        b = Budget(int(hbm_bytes), (C.c_uint64 * 2)(int(host_bytes[0]), int(host_bytes[1])), int(align), int(flags))
        plan = PoolPlan()
        classes = np.zeros(max(1, 2 * self.n_tensors), dtype=POOL_CLASS)
        self._check(lib().tc_plan_pools(self._h, C.byref(b), C.byref(plan), _ptr(classes), len(classes)))
        self.plan = plan
        self.classes = classes[: plan.n_classes].copy()
        self.n_steps = plan.n_steps
        return plan, self.classes

    def plan_schedule(self):
        out = np.zeros(self.n_tensors, dtype=PLACEMENT)
        self._check(lib().tc_plan_schedule(self._h, _ptr(out)))
        self.placement = out
        return out

    # -- memory ----------------------------------------------------------------
    def bind_memory(self, hbm_ptr: int, hbm_bytes: int, pinned_ptr: int, pinned_bytes: int,
                    staging_ptr: int = 0, staging_bytes: int = 0, file_fd: int = -1,
                    migrate_stream: int = 0, flags: int = 0):
        self._check(lib().tc_bind_memory(self._h, hbm_ptr or None, hbm_bytes, pinned_ptr or None, pinned_bytes,
                                         staging_ptr or None, staging_bytes, file_fd, migrate_stream or None, flags))

    def bind_torch(self, *, staging_bytes: int = 0, file_path: Optional[str] = None, null_mover: bool = False,
                   stream=None, direct: bool = False, file_fd: Optional[int] = None, stripes: int = 1,
                   host_tier: bool = False, stripe_paths: Optional[Sequence[str]] = None):
        """Allocates the regions and binds them: device memory and the streams
        come from PyTorch, the pinned regions straight from hipHostMalloc
        (PyTorch's pinned allocator rounds every request up to a power of two,
        which for a 60 GiB pool locks 64 GiB).  host_tier: the two-tier mode, the
        fast tier a pinned host region (self.hbm then is that region).
        stripe_paths: the files of the file tier named one by one (they may lie in
        different directories or on different devices) instead of file_path and
        file_path.1 .. file_path.(stripes-1)."""
        import torch
        if stripe_paths:
            file_path, stripes = stripe_paths[0], len(stripe_paths)
        mode = BIND_HOST_TIER if host_tier else 0
        if null_mover:
            self.bind_memory(0, 0, 0, 0, 0, 0, -1, 0, BIND_NULL_MOVER | mode)
            return
        dev = torch.device("cuda:0")
        if host_tier:
            hbm = _PinnedRegion(max(4096, int(self.plan.hbm_total)))
        else:
            hbm = torch.empty(max(256, int(self.plan.hbm_total)), dtype=torch.uint8, device=dev)
        pinned = _PinnedRegion(max(4096, int(self.plan.host_total)))
        if direct:
            staging_bytes = (int(staging_bytes) + 4095) // 4096 * 4096
        staging = _PinnedRegion(max(4096, int(staging_bytes)))
        self.mstream = stream if stream is not None else torch.cuda.Stream(device=dev)
        fd = -1
        if file_fd is not None:                 # an open descriptor of the caller's (closed with the context)
            fd = int(file_fd)
        elif file_path is not None:
            fd = os.open(file_path, os.O_RDWR | os.O_CREAT | (os.O_DIRECT if direct else 0), 0o600)
            os.ftruncate(fd, int(self.plan.file_total))
        self._fd = fd
        self._keep = [hbm, pinned, staging, self.mstream]
        self.hbm, self.pinned, self.staging = hbm, pinned, staging
        self.bind_memory(hbm.data_ptr(), hbm.nbytes if host_tier else hbm.numel(), pinned.data_ptr(), pinned.nbytes,
                         staging.data_ptr(), int(staging_bytes), fd, self.mstream.cuda_stream,
                         (BIND_FILE_DIRECT if (direct and fd >= 0) else 0) | mode)
        # further files the tier is striped over: file_path.1, file_path.2, ...
        self._stripe_fds = []
        for k in range(1, int(stripes) if file_path is not None and file_fd is None else 1):
            name = stripe_paths[k] if stripe_paths else f"{file_path}.{k}"
            sfd = os.open(name, os.O_RDWR | os.O_CREAT | (os.O_DIRECT if direct else 0), 0o600)
            self._stripe_fds.append(sfd)
            os.ftruncate(sfd, int(self.plan.file_total))
            self.add_stripe(sfd)

    def load_tensor(self, tensor: int, data: np.ndarray):
        data = np.ascontiguousarray(data, dtype=np.uint8)
        assert data.size == int(self.tensor_bytes[tensor])
        self._check(lib().tc_load_tensor(self._h, tensor, _ptr(data)))

    def fill_payload(self, seed: int = 0):
        self._check(lib().tc_fill_payload(self._h, seed))

    def read_tensor(self, tensor: int) -> np.ndarray:
        out = np.empty(int(self.tensor_bytes[tensor]), dtype=np.uint8)
        self._check(lib().tc_read_tensor(self._h, tensor, _ptr(out)))
        return out

    # -- hot path ---------------------------------------------------------------
    def migrate_step(self, step: int, phase: int, ids, rw=None, compute_stream: int = 0, want_ptrs: bool = False):
        ids = np.ascontiguousarray(ids, dtype=np.uint32)
        rwa = None if rw is None else np.ascontiguousarray(rw, dtype=np.uint8)
        ptrs = (C.c_void_p * max(1, len(ids)))() if want_ptrs else None
        self._check(lib().tc_migrate_step(self._h, step, phase, _ptr(ids), _ptr(rwa), len(ids),
                                          compute_stream or None, ptrs))
        if want_ptrs:
            return [p or 0 for p in ptrs[: len(ids)]]
        return None

    def end_iteration(self, compute_stream: int = 0):
        self._check(lib().tc_end_iteration(self._h, compute_stream or None))

    def emulate_compute(self, compute_stream: int = 0, busy_ns: int = 0):
        self._check(lib().tc_emulate_compute(self._h, compute_stream or None, int(busy_ns)))

    def set_stall_measurement(self, enable: bool):
        self._check(lib().tc_set_stall_measurement(self._h, int(enable)))

    def stall_by_step(self, clear: bool = False) -> np.ndarray:
        out = np.zeros(int(self.plan.n_steps), dtype=np.uint64)
        self._check(lib().tc_stall_by_step(self._h, _ptr(out), out.size, 1 if clear else 0))
        return out

    def synchronize(self):
        self._check(lib().tc_synchronize(self._h))

    def replay_iteration_c(self, steps, compute_stream: int = 0, busy_ns=None, measure_stall: bool = False):
        """The same sequence as replay_iteration, driven by tc_replay_iteration."""
        ptr = np.zeros(len(steps) + 1, dtype=np.uint32)
        ptr[1:] = np.cumsum([len(s) for s in steps])
        ids = np.asarray([t for s in steps for (t, _a) in s], dtype=np.uint32)
        rw = np.asarray([a for s in steps for (_t, a) in s], dtype=np.uint8)
        ns = None if busy_ns is None else np.ascontiguousarray(busy_ns, dtype=np.uint64)
        self._check(lib().tc_replay_iteration(self._h, _ptr(ptr), _ptr(ids), _ptr(rw), len(steps),
                                              compute_stream or None, _ptr(ns), int(measure_stall)))

    def replay_iteration(self, steps, compute_stream: int = 0, busy_ns=None, measure_stall: bool = False):
        """PRE, stand-in compute, POST for every step, then the end-of-iteration call."""
        self.set_stall_measurement(measure_stall)
        for k, access in enumerate(steps):
            ids = [t for (t, _a) in access]
            rw = [a for (_t, a) in access]
            self.migrate_step(k, PRE, ids, rw, compute_stream)
            self.emulate_compute(compute_stream, 0 if busy_ns is None else int(busy_ns[k]))
            self.migrate_step(k, POST, ids, rw, compute_stream)
        self.end_iteration(compute_stream)
        self.set_stall_measurement(False)

    # -- introspection -----------------------------------------------------------
    def cache_stats(self) -> dict:
        s = Stats()
        self._check(lib().tc_cache_stats(self._h, C.byref(s)))
        out = {}
        for name in STATS_FIELDS:
            v = getattr(s, name)
            out[name] = list(v) if name in ("n_ops", "host_blocked_ns") else int(v)
        return out

    def dump_oplog(self) -> np.ndarray:
        n = C.c_uint64()
        self._check(lib().tc_dump_oplog(self._h, 0, None, 0, C.byref(n)))
        buf = np.zeros(n.value, dtype=OP)
        if n.value:
            self._check(lib().tc_dump_oplog(self._h, 0, _ptr(buf), n.value, C.byref(n)))
        return buf

    def set_oplog(self, enable: bool = True, clear: bool = False):
        self._check(lib().tc_set_oplog(self._h, int(enable), int(clear)))

    def dump_state(self):
        tier = np.zeros(self.n_tensors, dtype=np.uint8)
        gs = np.zeros(self.n_tensors, dtype=np.uint32)
        cs = np.zeros(self.n_tensors, dtype=np.uint32)
        self._check(lib().tc_dump_state(self._h, _ptr(tier), _ptr(gs), _ptr(cs)))
        return tier, gs, cs

    def set_mover(self, workgroups: int = 0, chunk_bytes: int = 0):
        self._check(lib().tc_set_mover(self._h, workgroups, chunk_bytes))

    def mover_timing(self, enable: bool) -> dict:
        t = Timing()
        self._check(lib().tc_mover_timing(self._h, int(enable), C.byref(t)))
        return {f[0]: getattr(t, f[0]) for f in Timing._fields_}

    def tune_mover(self) -> int:
        """Times exchanges between the (still empty) regions and keeps the best workgroup count."""
        wg = C.c_uint32(0)
        self._check(lib().tc_tune_mover(self._h, C.byref(wg)))
        return int(wg.value)

    def set_merge_bytes(self, nbytes: int):
        self._check(lib().tc_set_merge_bytes(self._h, int(nbytes)))

    def set_gpu_dependencies(self, enable: bool, timeout_ms: int = 0):
        self._check(lib().tc_set_gpu_dependencies(self._h, int(bool(enable)), int(timeout_ms)))

    def set_dma_policy(self, when_behind: bool):
        self._check(lib().tc_set_dma_policy(self._h, int(bool(when_behind))))

    def set_io_chunk(self, nbytes: int):
        self._check(lib().tc_set_io_chunk(self._h, int(nbytes)))

    def add_stripe(self, fd: int):
        self._check(lib().tc_add_stripe(self._h, int(fd)))

    def set_io_threads(self, writers: int, readers: int):
        self._check(lib().tc_set_io_threads(self._h, int(writers), int(readers)))

    def set_decide_ahead(self, steps: int):
        self._check(lib().tc_set_decide_ahead(self._h, int(steps)))

    def set_replay_window(self, steps: int):
        self._check(lib().tc_set_replay_window(self._h, int(steps)))

    def set_dma_threshold(self, nbytes: int):
        self._check(lib().tc_set_dma_threshold(self._h, int(nbytes)))

    # -- convenience: a workload object from the workloads package ----------------
    @classmethod
    def from_workload(cls, wl) -> "TensorCache":
        tc = cls()
        st, te, rw, ns = wl.events()
        tc.profile_order(wl.tensor_bytes, wl.tensor_group, st, te, rw, ns, wl.tensor_kind)
        tc.plan_pools(wl.hbm_bytes, wl.host_bytes, wl.align,
                      (LITERAL_ALG2 if wl.literal_alg2 else 0) | (NO_PREFETCH if getattr(wl, "no_prefetch", False) else 0)
                      | (SMALLEST_FIRST if getattr(wl, "smallest_first", False) else 0)
                      | (ALLOC_WRITE_ONLY if getattr(wl, "alloc_write_only", False) else 0))
        tc.plan_schedule()
        return tc


def copy_batch(src_ptrs, dst_ptrs, nbytes, stream: int = 0, workgroups: int = 0, chunk_bytes: int = 0):
    segs = np.zeros(len(src_ptrs), dtype=SEGMENT)
    segs["src"] = src_ptrs
    segs["dst"] = dst_ptrs
    segs["bytes"] = nbytes
    rc = lib().tc_copy_batch(_ptr(segs), len(segs), stream or None, workgroups, chunk_bytes)
    if rc:
        raise TcError(rc)


def exchange_batch(out_src, out_dst, in_src, in_dst, nbytes, stream: int = 0, workgroups: int = 0,
                   chunk_bytes: int = 0):
    o = np.zeros(len(nbytes), dtype=SEGMENT)
    i = np.zeros(len(nbytes), dtype=SEGMENT)
    o["src"], o["dst"], o["bytes"] = out_src, out_dst, nbytes
    i["src"], i["dst"], i["bytes"] = in_src, in_dst, nbytes
    o["bytes"][np.asarray(out_src) == 0] = 0
    i["bytes"][np.asarray(in_src) == 0] = 0
    rc = lib().tc_exchange_batch(_ptr(o), _ptr(i), len(o), stream or None, workgroups, chunk_bytes)
    if rc:
        raise TcError(rc)


def pack_tiles(total: int) -> int:
    return int(lib().tc_pack_tiles(int(total)))


def pack_index(off_dev: int, n: int, total: int, tile_first_dev: int, stream: int = 0):
    rc = lib().tc_pack_index(off_dev or None, n, total, tile_first_dev or None, stream or None)
    if rc:
        raise TcError(rc)


def pack(slab_ptr: int, ptrs_dev: int, bytes_dev: int, off_dev: int, n: int, total: int, stream: int = 0,
         tile_first_dev: int = 0):
    rc = lib().tc_pack(slab_ptr or None, ptrs_dev or None, bytes_dev or None, off_dev or None, n, total,
                       tile_first_dev or None, stream or None)
    if rc:
        raise TcError(rc)


def unpack(slab_ptr: int, ptrs_dev: int, bytes_dev: int, off_dev: int, n: int, total: int, stream: int = 0,
           tile_first_dev: int = 0):
    rc = lib().tc_unpack(slab_ptr or None, ptrs_dev or None, bytes_dev or None, off_dev or None, n, total,
                         tile_first_dev or None, stream or None)
    if rc:
        raise TcError(rc)


PACK_STATIC_MAX_BYTES = 4 << 30


def pack_static(slab_ptr: int, ptrs_dev: int, bytes_dev: int, off_dev: int, n: int, total: int, unpack_: bool = False,
                stream: int = 0):
    rc = lib().tc_pack_static(slab_ptr or None, ptrs_dev or None, bytes_dev or None, off_dev or None, n, total,
                              1 if unpack_ else 0, stream or None)
    if rc:
        raise TcError(rc)
