"""Optimizer states of a model in the two-tier cache (pinned host cache over the
file tier) and an Adam update on the CPU over them.

`OptStateCache` keeps three fp32 tensors per parameter (master copy, momentum,
variance; ids 3j, 3j+1, 3j+2), profiled as one sweep over the parameters, and
hands them out as PyTorch CPU views of the cache's buffers between the PRE and
POST calls of `tc_migrate_step` (the paper's optimizer states scheduling policy,
Sec. 3.4.2).
"""

from __future__ import annotations

import ctypes as C
from typing import List, Optional

import numpy as np

from . import binding as T

RW = 3          # an access that reads and writes (TC_R | TC_W)


def adam_(torch, p, m, v, g, tmp, step, lr=1e-3, b1=0.9, b2=0.999, eps=1e-8):
    """Adam on fp32 CPU views, in place; tmp is scratch of the same length."""
    m.mul_(b1).add_(g, alpha=1 - b1)
    v.mul_(b2).addcmul_(g, g, value=1 - b2)
    torch.sqrt(v, out=tmp)
    tmp.div_((1 - b2 ** step) ** 0.5).add_(eps)
    p.addcdiv_(m, tmp, value=-lr / (1 - b1 ** step))


def host_view(torch, ptr: int, n: int):
    """n floats at a host address as a PyTorch tensor (no copy)."""
    return torch.from_numpy(np.ctypeslib.as_array((C.c_float * n).from_address(ptr)))


class OptStateCache:
    def __init__(self, elems: List[int], cache_bytes: int, file_path: str, *, stripes: int = 4, direct: bool = False,
                 prefetch: bool = True):
        import torch
        self.torch = torch
        self.elems = [int(e) for e in elems]
        n_p = len(self.elems)
        tensor_bytes = np.repeat(np.asarray(self.elems, dtype=np.uint64) * 4, 3)
        tc = self.tc = T.TensorCache()
        tc.profile_order(tensor_bytes, np.ones(3 * n_p, dtype=np.uint8), np.repeat(np.arange(n_p, dtype=np.uint32), 3),
                         np.arange(3 * n_p, dtype=np.uint32), np.full(3 * n_p, RW, dtype=np.uint8))
        tc.plan_pools(int(cache_bytes), (0, 0), 256, 0 if prefetch else T.NO_PREFETCH)
        tc.plan_schedule()
        tc.bind_torch(file_path=file_path, host_tier=True, stripes=stripes, direct=direct)
        tc.set_oplog(False, True)
        self._ids = [np.asarray([3 * j, 3 * j + 1, 3 * j + 2], dtype=np.uint32) for j in range(n_p)]
        self._rw = np.full(3, RW, dtype=np.uint8)
        self._views = {}

    def load(self, j: int, master, momentum=None, variance=None):
        """Initial states of parameter j (fp32 numpy arrays; zeros where None)."""
        n = self.elems[j]
        for k, a in enumerate((master, momentum, variance)):
            a = np.zeros(n, dtype=np.float32) if a is None else np.ascontiguousarray(a, dtype=np.float32).reshape(-1)
            self.tc.load_tensor(3 * j + k, a.view(np.uint8))

    def begin(self, j: int):
        """PRE: the three states of parameter j as CPU views, once their bytes are in the cache."""
        ptrs = self.tc.migrate_step(j, T.PRE, self._ids[j], self._rw, 0, want_ptrs=True)
        out = []
        for a in ptrs:
            if not a:
                raise RuntimeError(f"states of parameter {j} could not be given a buffer (cache too small)")
            v = self._views.get((a, self.elems[j]))
            if v is None:
                v = self._views[(a, self.elems[j])] = host_view(self.torch, a, self.elems[j])
            out.append(v)
        return out

    def end(self, j: int):
        """POST: the update of parameter j is complete."""
        self.tc.migrate_step(j, T.POST, self._ids[j], self._rw, 0)

    def end_iteration(self):
        self.tc.end_iteration(0)

    def read(self, j: int, k: int = 0) -> np.ndarray:
        return self.tc.read_tensor(3 * j + k).view(np.float32)

    def stats(self) -> dict:
        return self.tc.cache_stats()

    def close(self):
        self._views = {}
        if self.tc is not None:
            self.tc.close()
            self.tc = None
