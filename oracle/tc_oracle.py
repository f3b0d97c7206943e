"""Plain CPU oracle for order-driven tensor migration (10Cache, arXiv 2511.14124).

TEST INFRASTRUCTURE ONLY.  This file is the slow, sequential, obviously
correct statement of what the migration hot path computes.  It shares no code
with the HIP library and must never be imported by the product path: only
tests, the smoke check and the benchmark's cpu_baseline leg may use it.

What follows the paper, passage by passage:

* `profile`      Sec. 3.2.1 (prefetch table: execution order per tensor) and
                 Sec. 3.2.2 (size -> count dictionary TC).
* `tsd`          Alg. 1 (tensor size distribution).
* `plan_pools`   Alg. 2 (buffer counts) and Step 3 of Sec. 3.3.1 (one
                 contiguous region cut into per-size chunks, free list).
* `place`        Sec. 3.3.2 (tensor allocator: GPU first, then CPU, then NVMe,
                 in execution order; "final location").
* `Replay.post`  Alg. 3 (PrefetchTensor), called from the post-hook with the
                 tensors that just finished.
* `Replay._evict` Alg. 4 (EvictTensor).
* `Replay.end_iteration`  Sec. 3.2.1: after each iteration tensors return to
                 their final locations.

The paper is a heuristic state machine, not a faster route to a separately
defined result, so the oracle is the algorithm itself, step by step.  Where
the paper is silent or at odds with itself the reading taken is stated at the
place it is applied (search for "Reading").  Pins: tests/test_oracle_*.py check
this file against the paper's two worked examples (Sec. 3.4.1 and 3.4.2),
Alg. 1/2 closed forms, a single-class closed form, exhaustive search on tiny
traces and step-by-step invariants.

What the paper and the mathematics do not fix, and what stands in for them:
the prefetch table, the dictionary and the per-step maxima are pinned by a
hand-written trace; the end-of-iteration moves by "every displaced tensor
moves exactly once, nothing else moves" (any order satisfying it is a correct
restore; the order itself is a reading); keeping a finished tensor of another
size by Sec. 3.4.1 (nothing goes to NVMe while GPU and CPU hold the model; the
literal alternative spills); the "by this call" rules are shown to decide
nothing on the worked examples and the unperturbed configurations.

Parity unpinned (fixed only by the readings stated here, plus invariants):
victim tie-breaks, the demand-miss path, which of several valid
end-of-iteration orders is taken, the dirty rule for file-tier tensors (that
the log follows the rule is checked from the log and the trace alone; the rule
is a reading), and Alg. 2 with the working-set floor beyond its invariants, one
hand example and the reason it exists (no access of a profiled trace fails).
"""

from __future__ import annotations

import bisect
from dataclasses import dataclass
from fractions import Fraction
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

INF = 0xFFFFFFFF                     # "never used again"
NONE = 0xFFFFFFFF                    # no tensor / no slot

GPU, CPU, NVME = 0, 1, 2             # tiers
PRE, POST, END, END_CPU = 0, 1, 2, 3 # phases of the op log (END: two hook calls, END_CPU: a third)
R_FLAG, W_FLAG = 1, 2

# op codes of the op log
DEMAND, PREFETCH, EVICT, RELEASE, WRITEBACK, SPILL, RESTORE, FAIL, ALLOC = range(9)
OP_NAMES = ["DEMAND", "PREFETCH", "EVICT", "RELEASE", "WRITEBACK", "SPILL", "RESTORE", "FAIL", "ALLOC"]

FILE_ALIGN = 4096
STAMP_MAGIC = 0x10CAC4E5


def align_up(x: int, a: int) -> int:
    return (x + a - 1) // a * a


# ----------------------------------------------------------------------------
# Sec. 3.2: the tensor characteristic analyzer
# ----------------------------------------------------------------------------

@dataclass
class Profile:
    n_tensors: int
    rows_tensor: List[int]            # prefetch table: tensor id of row r (execution order)
    rows_rw: List[int]
    row_begin: List[int]              # first row of step k
    row_end: List[int]                # one past the last row of step k
    occ: List[List[int]]              # occ[t] = rows at which tensor t is used, ascending
    first_use: List[int]              # first row of t, INF if never used
    class_of: List[int]               # size class index of tensor t
    class_bytes: List[int]            # tensor size of class s
    class_group: List[int]            # 0 = 16-bit tensors, 1 = fp32 optimizer states
    count: List[int]                  # c_s: tensors of the class (the dictionary TC)
    used: List[int]                   # a_s: tensors of the class seen by the dry run
    step_max: List[int]               # m_s: most tensors of the class used by one step

    @property
    def n_rows(self) -> int:
        return len(self.rows_tensor)

    @property
    def n_steps(self) -> int:
        return len(self.row_begin)

    def next_use(self, t: int, row: int) -> int:
        """First row >= `row` at which tensor t is used, INF if none."""
        o = self.occ[t]
        i = bisect.bisect_left(o, row)
        return o[i] if i < len(o) else INF


def profile(tensor_bytes: Sequence[int], tensor_group: Sequence[int],
            ev_step: Sequence[int], ev_tensor: Sequence[int], ev_rw: Sequence[int]) -> Profile:
    """Build the prefetch table and TC from one profiled iteration (Sec. 3.2).

    Events arrive in execution order with non-decreasing step numbers.  A tensor
    named twice by one step is one row (flags OR-ed): a hook reports each tensor
    of its module once.

    Reading: a size class is a (bytes, group) pair.  The paper sizes 16-bit and
    fp32 buffers in separate runs of Alg. 2 (Sec. 3.3.1 Step 2), so a byte size
    shared by a 16-bit tensor and an fp32 state is two classes.
    """
    n_t = len(tensor_bytes)
    n_steps = (int(ev_step[-1]) + 1) if len(ev_step) else 0
    per_step: List[Dict[int, int]] = [dict() for _ in range(n_steps)]
    last = 0
    for k, t, a in zip(ev_step, ev_tensor, ev_rw):
        k, t, a = int(k), int(t), int(a)
        if k < last:
            raise ValueError("events must be ordered by step")
        if not (0 <= t < n_t) or not (1 <= a <= 3):
            raise ValueError("bad event")
        last = k
        per_step[k][t] = per_step[k].get(t, 0) | a      # dict keeps first-occurrence order
    rows_tensor, rows_rw, row_begin, row_end = [], [], [], []
    for k in range(n_steps):
        row_begin.append(len(rows_tensor))
        for t, a in per_step[k].items():
            rows_tensor.append(t)
            rows_rw.append(a)
        row_end.append(len(rows_tensor))
    occ: List[List[int]] = [[] for _ in range(n_t)]
    for r, t in enumerate(rows_tensor):
        occ[t].append(r)
    first_use = [o[0] if o else INF for o in occ]

    keys = sorted({(int(b), int(g)) for b, g in zip(tensor_bytes, tensor_group)})
    index = {k: i for i, k in enumerate(keys)}
    class_of = [index[(int(b), int(g))] for b, g in zip(tensor_bytes, tensor_group)]
    n_c = len(keys)
    count = [0] * n_c
    used = [0] * n_c
    for t in range(n_t):
        count[class_of[t]] += 1
        if occ[t]:
            used[class_of[t]] += 1
    step_max = [0] * n_c
    for k in range(n_steps):
        per = [0] * n_c
        for r in range(row_begin[k], row_end[k]):
            per[class_of[rows_tensor[r]]] += 1
        step_max = [max(a, b) for a, b in zip(step_max, per)]
    return Profile(n_t, rows_tensor, rows_rw, row_begin, row_end, occ, first_use, class_of,
                   [k[0] for k in keys], [k[1] for k in keys], count, used, step_max)


# ----------------------------------------------------------------------------
# Sec. 3.3.1: the cache allocator
# ----------------------------------------------------------------------------

def tsd(tc: Sequence[Tuple[int, int]]) -> List[Fraction]:
    """Alg. 1: share of the total bytes taken by each size, as exact rationals."""
    total = 0
    dist = []
    for (s, c) in tc:
        sc = s * c
        total += sc
        dist.append(sc)
    return [Fraction(sc, total) if total else Fraction(0) for sc in dist]


def buffer_count(tc: Sequence[Tuple[int, int]], avail: int, cap: Sequence[int]) -> List[int]:
    """One output of Alg. 2: min(TSD[s] * avail / s, cap[s]) per size.

    Reading: the quotient is rounded down (a buffer is whole) and evaluated in
    exact rationals; a floating-point TSD could differ by one at exact
    boundaries.
    """
    dist = tsd(tc)
    out = []
    for (s, _c), d, k in zip(tc, dist, cap):
        n = (d * avail / s).__floor__() if s else 0
        out.append(max(0, min(int(n), int(k))))
    return out


@dataclass
class PoolPlan:
    stride: List[int]                 # buffer size of class s (tensor size rounded up to `align`)
    gpu_count: List[int]              # GPU_BUFFER_COUNT
    cpu_count: List[int]              # CPU_BUFFER_COUNT
    gpu_off: List[int]                # byte offset of buffer 0 of class s in the HBM region
    cpu_off: List[int]                # ... in the pinned host region
    gpu_total: int
    cpu_total: int


class CapacityError(Exception):
    pass


def plan_pools(p: Profile, hbm_bytes: int, host_bytes: Sequence[int], align: int = 256,
               literal: bool = False, smallest_first: bool = False) -> PoolPlan:
    """Alg. 2 plus Step 3 of Sec. 3.3.1.

    The size s_i of Alg. 1/2 is the buffer size actually cut from the region
    (tensor bytes rounded up to `align`; the same number whenever sizes are
    multiples of `align`).

    GPU counts use the dictionary of the dry run: tensors the profiled
    iteration never touched are not in TC and get no GPU buffer.

    Reading (working-set floor): read literally, Alg. 2 gives
    floor(c_s * avail / total) buffers, which is zero for every class with
    fewer than total/avail tensors; a step using such a tensor could never
    run.  Unless `literal` is set, each class first receives m_s buffers (the
    most one step uses) and Alg. 2 is applied to what is left: counts
    (c_s - m_s) and memory avail - sum(m_s * s).  With every m_s = 0 the two
    agree.

    `smallest_first` is not the paper's allocator but the placement it argues
    against (Sec. 3.1 and the illustrative example of Sec. 3.3.2: the baseline
    places tensors by size, the large ones below the GPU wherever they stand in
    the execution order): GPU memory beyond the floor goes to the classes in
    ascending size, each taking as many buffers as it has tensors and the
    memory left allows, so the smallest tensors stay on the GPU and the
    largest live below it.  An ablation, used to state a hit-rate ratio of the
    kind the paper reports against that baseline.

    Host counts are Alg. 2's second line, run once per group with that group's
    budget and its own distribution (16-bit tensors first, fp32 states after).

    Step 3: classes ascending by (bytes, group); buffer k of class s sits at
    off[s] + k*stride[s]; offsets are running sums, so the smallest class's
    first chunk is "buffer0" at offset 0.
    """
    n_c = len(p.count)
    stride = [align_up(b, align) for b in p.class_bytes]
    if smallest_first:
        gpu = [0 if literal else min(p.step_max[s], p.used[s]) for s in range(n_c)]
        left = hbm_bytes - sum(gpu[s] * stride[s] for s in range(n_c))
        if left < 0:
            raise CapacityError("HBM budget below the per-step working set")
        for s in range(n_c):                              # classes are ascending by (bytes, group)
            more = min(p.used[s] - gpu[s], left // stride[s])
            gpu[s] += more
            left -= more * stride[s]
    elif literal:
        gpu = buffer_count([(stride[s], p.used[s]) for s in range(n_c)], hbm_bytes, p.used)
    else:
        floor_ = [min(p.step_max[s], p.used[s]) for s in range(n_c)]
        reserved = sum(floor_[s] * stride[s] for s in range(n_c))
        if reserved > hbm_bytes:
            raise CapacityError("HBM budget below the per-step working set")
        rest = [p.used[s] - floor_[s] for s in range(n_c)]
        extra = buffer_count([(stride[s], rest[s]) for s in range(n_c)], hbm_bytes - reserved, rest)
        gpu = [floor_[s] + extra[s] for s in range(n_c)]
    cpu = [0] * n_c
    for g in (0, 1):
        idx = [s for s in range(n_c) if p.class_group[s] == g]
        got = buffer_count([(stride[s], p.count[s]) for s in idx], int(host_bytes[g]),
                           [p.count[s] - gpu[s] for s in idx])
        for s, n in zip(idx, got):
            cpu[s] = n
    gpu_off, cpu_off, go, co = [], [], 0, 0
    for s in range(n_c):
        gpu_off.append(go)
        cpu_off.append(co)
        go += gpu[s] * stride[s]
        co += cpu[s] * stride[s]
    return PoolPlan(stride, gpu, cpu, gpu_off, cpu_off, go, co)


# ----------------------------------------------------------------------------
# Sec. 3.3.2: the tensor allocator
# ----------------------------------------------------------------------------

@dataclass
class Placement:
    final: List[int]                  # final location (tier) of tensor t
    slot: List[int]                   # buffer index within its class on that tier, NONE for NVMe
    file_off: List[int]               # byte offset of t's extent in the file tier
    file_total: int
    order: List[int]                  # tensors in placement order


def place(p: Profile, plan: PoolPlan) -> Placement:
    """Tensors in execution order take the fastest tier that still has a free
    buffer of their size: GPU, then CPU, then NVMe (Sec. 3.3.2).  Buffers are
    handed out lowest index first (the free list of Step 3 returns buffer0
    first).  Tensors the dry run never saw come last, by id, and never take a
    GPU buffer.  Every tensor also owns a file extent (4 KiB aligned, id order),
    used when it is NVMe-final or spilled.
    """
    order = sorted(range(p.n_tensors), key=lambda t: (p.first_use[t], t))
    gpu_next = [0] * len(plan.gpu_count)
    cpu_next = [0] * len(plan.cpu_count)
    final = [NVME] * p.n_tensors
    slot = [NONE] * p.n_tensors
    for t in order:
        s = p.class_of[t]
        if p.first_use[t] != INF and gpu_next[s] < plan.gpu_count[s]:
            final[t], slot[t] = GPU, gpu_next[s]
            gpu_next[s] += 1
        elif cpu_next[s] < plan.cpu_count[s]:
            final[t], slot[t] = CPU, cpu_next[s]
            cpu_next[s] += 1
    file_off, off = [], 0
    bytes_of = [p.class_bytes[p.class_of[t]] for t in range(p.n_tensors)]
    for t in range(p.n_tensors):
        file_off.append(off)
        off += align_up(bytes_of[t], FILE_ALIGN)
    return Placement(final, slot, file_off, off, order)


# ----------------------------------------------------------------------------
# Sec. 3.4: the prefetch-eviction scheduler, replayed
# ----------------------------------------------------------------------------

Op = Tuple[int, int, int, int, int, int, int, int, int, int]
# (iteration, step, phase, op, tensor, src_tier, src_slot, dst_tier, dst_slot, bytes)


def stamp16(iteration: int, step: int, tensor: int) -> np.ndarray:
    """The 16 bytes a write access XORs into the first and the last 16 bytes of
    a tensor: four little-endian 32-bit words (magic, iteration, step, tensor).
    It stands in for the module's kernel writing its output."""
    return np.asarray([STAMP_MAGIC, iteration, step, tensor], dtype="<u4").view(np.uint8).copy()


def write_seed(iteration: int, step: int) -> int:
    """Seed of the counter pattern a write-only access fills its tensor with when such accesses
    are declared whole-tensor writes (see Replay): one per (iteration, step)."""
    return 0x10000000 + iteration * 4096 + step


def apply_stamp(buf: np.ndarray, stamp: np.ndarray) -> None:
    n = buf.shape[0]
    assert n >= 16
    buf[:16] ^= stamp
    buf[n - 16:] ^= stamp


class Replay:
    """State of the scheduler while a trace is replayed.

    With `payload` given (a function tensor id -> uint8 array) the three tiers
    are real byte arrays and every op moves bytes ("full-bytes mode").  Without
    it only the bookkeeping runs and `expected_bytes` rebuilds any tensor from
    its initial payload and the stamps it received ("metadata mode").
    """

    def __init__(self, p: Profile, plan: PoolPlan, pl: Placement, payload=None, prefetch: bool = True,
                 alloc_write_only: bool = False, pattern=None):
        """alloc_write_only: a refinement the paper does not have.  An access that only writes
        (a gradient in the backward pass, a checkpoint in the forward pass, the 16-bit
        parameter in the optimizer sweep) is declared a whole-tensor write, so what the tensor
        held before is dead and bringing it in is wasted traffic: where Alg. 3 would prefetch
        such a tensor, or the pre-hook would fetch it on demand, it is given its GPU buffer
        without any bytes being copied (op ALLOC).  Every decision is what it is without the
        flag; only the copy is left out.  The stand-in for the module's kernel then fills the
        whole tensor with the counter pattern of seed write_seed(iteration, step) instead of
        stamping it.  `pattern(tensor, n_bytes, seed)` supplies that pattern (an input
        generator, like `payload`).  A tensor allocated this way is undefined until its
        write-only access really comes; on a replay that leaves the profile it may never
        come, and then the tensor's bytes are unspecified (`undefined[t]`; reads of such
        tensors are counted in `undefined_reads`)."""
        self.p, self.plan, self.pl = p, plan, pl
        self.prefetch = prefetch          # False: the "base" variant of Sec. 4.1.4, demand fetch only
        self.alloc_write_only = alloc_write_only
        self._pattern = pattern
        self.undefined = [False] * p.n_tensors
        self.undefined_reads = 0
        self.whole_write: List[Optional[Tuple[int, int]]] = [None] * p.n_tensors   # (iteration, step) of the last one
        n_t, n_c = p.n_tensors, len(p.count)
        self.bytes_of = [p.class_bytes[p.class_of[t]] for t in range(n_t)]
        self.cur = list(pl.final)
        self.gslot = [pl.slot[t] if pl.final[t] == GPU else NONE for t in range(n_t)]
        self.cslot = [pl.slot[t] if pl.final[t] == CPU else NONE for t in range(n_t)]
        self.gpu_owner = [[NONE] * plan.gpu_count[s] for s in range(n_c)]
        self.cpu_owner = [[NONE] * plan.cpu_count[s] for s in range(n_c)]
        self.designated = [[False] * plan.cpu_count[s] for s in range(n_c)]
        self.gpu_freed = [[0] * plan.gpu_count[s] for s in range(n_c)]   # hook call that freed the buffer
        self.cpu_freed = [[0] * plan.cpu_count[s] for s in range(n_c)]
        for t in range(n_t):
            if pl.final[t] == GPU:
                self.gpu_owner[p.class_of[t]][pl.slot[t]] = t
            elif pl.final[t] == CPU:
                self.cpu_owner[p.class_of[t]][pl.slot[t]] = t
        self.dirty = [False] * n_t
        self.moved = [0] * n_t            # id of the last hook call that moved t
        self.call = 0
        self.cursor = 0                   # prefetch_tab_cur_row
        self.iteration = 0
        self.log: List[Op] = []
        self.hits = 0
        self.misses = 0
        self.fails = 0
        self.step_hits: List[Tuple[int, int, int, int]] = []   # (iteration, step, hits, misses)
        self.bytes_h2d = self.bytes_d2h = self.bytes_file_read = self.bytes_file_write = 0
        self.stamps: List[List[Tuple[int, int]]] = [[] for _ in range(n_t)]
        self.resident_at_pre: List[List[Optional[Tuple[int, int]]]] = []
        self.full = payload is not None
        self._payload = payload
        if self.full:
            self.hbm = np.zeros(plan.gpu_total, dtype=np.uint8)
            self.host = np.zeros(plan.cpu_total, dtype=np.uint8)
            self.file = np.zeros(pl.file_total, dtype=np.uint8)
            for t in range(n_t):
                self._view(t)[:] = payload(t)

    # -- byte views ----------------------------------------------------------
    def _gpu_view(self, s: int, k: int, n: int) -> np.ndarray:
        o = self.plan.gpu_off[s] + k * self.plan.stride[s]
        return self.hbm[o:o + n]

    def _cpu_view(self, s: int, k: int, n: int) -> np.ndarray:
        o = self.plan.cpu_off[s] + k * self.plan.stride[s]
        return self.host[o:o + n]

    def _file_view(self, t: int) -> np.ndarray:
        o = self.pl.file_off[t]
        return self.file[o:o + self.bytes_of[t]]

    def _view(self, t: int) -> np.ndarray:
        """The bytes of tensor t where it currently lives."""
        s, n = self.p.class_of[t], self.bytes_of[t]
        if self.cur[t] == GPU:
            return self._gpu_view(s, self.gslot[t], n)
        if self.cur[t] == CPU:
            return self._cpu_view(s, self.cslot[t], n)
        return self._file_view(t)

    def read_tensor(self, t: int) -> np.ndarray:
        return self._view(t).copy()

    def expected_bytes(self, t: int, payload) -> Optional[np.ndarray]:
        """Initial payload of t (or what its last whole-tensor write put there) with every
        stamp it received since applied; None while the tensor's bytes are unspecified."""
        if self.undefined[t]:
            return None
        if self.whole_write[t] is not None:
            it, step = self.whole_write[t]
            buf = np.array(self._pattern(t, self.bytes_of[t], write_seed(it, step)), dtype=np.uint8, copy=True)
        else:
            buf = np.array(payload(t), dtype=np.uint8, copy=True)
        for (it, step) in self.stamps[t]:
            apply_stamp(buf, stamp16(it, step, t))
        return buf

    # -- small helpers -------------------------------------------------------
    def _emit(self, step, phase, op, t, st, ss, dt, ds, nbytes):
        self.log.append((self.iteration, step, phase, op, t, st, ss, dt, ds, nbytes))

    def _lowest_free(self, owner: List[int], freed: List[int]) -> int:
        """Lowest free buffer of a class (the free list returns buffer0 first).

        Reading: a buffer freed by the current hook call may still be the
        source of a copy that call issued, so it is handed out again only from
        the next call on."""
        for k, o in enumerate(owner):
            if o == NONE and freed[k] != self.call:
                return k
        return NONE

    def _farthest(self, cands: List[int], bound: int) -> int:
        """Among candidate tensors the one used farthest in the future, counted
        from row `bound`; never-again counts as farthest; ties -> lowest id."""
        best, best_key = NONE, None
        for x in cands:
            key = (-self.p.next_use(x, bound), x)
            if best_key is None or key < best_key:
                best, best_key = x, key
        return best

    # -- Alg. 4 ---------------------------------------------------------------
    def _evict(self, v: int, step: int, phase: int, bound: int, partner_cpu_slot: int) -> None:
        """EvictTensor(v).  `partner_cpu_slot` is the host buffer of the tensor
        about to take v's GPU buffer, or NONE.

        Reading (pair semantics): Alg. 3 calls EvictTensor before the prefetch
        frees the incoming tensor's host buffer, while Alg. 2 gives exactly
        c_s - G_s host buffers, so read literally even the CPU-GPU example of
        Sec. 3.4.1 (CPU {4,5,6} -> {1,5,6} with three buffers) would have to
        spill.  The evicted tensor therefore takes its partner's host buffer
        directly: the two tensors swap places.

        Reading (victim): of the occupied host buffers that qualify in Alg. 4
        the tensor used farthest in the future is spilled, ties -> lowest id;
        tensors already moved by this hook call do not qualify.

        Reading (dirty): an NVMe-final tensor is written back only if a write
        access touched it since it was last on the file tier; the paper's
        releasing the GPU buffer without a copy, as the text does, covers read-only parameters.
        """
        p, s, n = self.p, self.p.class_of[v], self.bytes_of[v]
        y = self.gslot[v]
        if self.pl.final[v] == NVME:                       # Alg. 4: final_loc is 'nvme'
            if self.dirty[v]:
                if self.full:
                    self._file_view(v)[:] = self._gpu_view(s, y, n)
                self._emit(step, phase, WRITEBACK, v, GPU, y, NVME, NONE, n)
                self.bytes_file_write += n
                self.dirty[v] = False
            else:
                self._emit(step, phase, RELEASE, v, GPU, y, NVME, NONE, 0)
            self.cur[v] = NVME
        else:
            x = partner_cpu_slot
            if x == NONE:
                x = self._lowest_free(self.cpu_owner[s], self.cpu_freed[s])   # "CPU has free buffer"
            if x == NONE:
                occupied = [k for k, o in enumerate(self.cpu_owner[s])
                            if o != NONE and self.moved[o] != self.call]
                pool = [k for k in occupied if self.designated[s][k]] or occupied
                if pool:                                   # spill its tensor to NVMe, reuse the buffer
                    w = self._farthest([self.cpu_owner[s][k] for k in pool], bound)
                    x = self.cslot[w]
                    if self.full:
                        self._file_view(w)[:] = self._cpu_view(s, x, n)
                    self._emit(step, phase, SPILL, w, CPU, x, NVME, NONE, n)
                    self.bytes_file_write += n
                    self.cur[w], self.cslot[w] = NVME, NONE
                    self.moved[w] = self.call
                    self.cpu_owner[s][x] = NONE
                    self.designated[s][x] = False
            if x == NONE:
                # no host buffer of this size at all: v goes to its file extent
                if self.full:
                    self._file_view(v)[:] = self._gpu_view(s, y, n)
                self._emit(step, phase, WRITEBACK, v, GPU, y, NVME, NONE, n)
                self.bytes_file_write += n
                self.cur[v] = NVME
            else:
                self.designated[s][x] = (self.pl.final[v] == GPU)   # "GPU-designated"
                self.cpu_owner[s][x] = v
                self.cslot[v] = x
                if self.full:
                    self._cpu_view(s, x, n)[:] = self._gpu_view(s, y, n)
                self._emit(step, phase, EVICT, v, GPU, y, CPU, x, n)
                self.bytes_d2h += n
                self.cur[v] = CPU
        self.gslot[v] = NONE
        self.gpu_owner[s][y] = NONE
        self.gpu_freed[s][y] = self.call
        self.moved[v] = self.call

    def _exchange(self, v: int, u: int, y: int, step: int, phase: int, op_in: int, bound: int) -> None:
        """Evict v (or nothing if v is NONE) and bring u into GPU buffer y of
        their common class.  Bytes leaving the GPU buffer are read before the
        incoming bytes land: in full-bytes mode the outgoing copy is taken
        first."""
        s, n = self.p.class_of[u], self.bytes_of[u]
        src_tier, src_slot = self.cur[u], self.cslot[u]
        incoming = None
        if self.full and op_in != ALLOC:
            incoming = self._view(u).copy()
        if v != NONE:
            swap = src_slot if (src_tier == CPU and self.pl.final[v] != NVME) else NONE
            if swap != NONE:                      # u leaves its host buffer to v
                self.cpu_owner[s][swap] = NONE
                self.designated[s][swap] = False
            self._evict(v, step, phase, bound, swap)
        if src_tier == CPU and self.cpu_owner[s][src_slot] == u:
            self.cpu_owner[s][src_slot] = NONE    # "release" u's host buffer
            self.designated[s][src_slot] = False
            self.cpu_freed[s][src_slot] = self.call
        if op_in == ALLOC:
            # the buffer is handed over as it is: nothing is copied, what the tensor held is dropped
            self._emit(step, phase, ALLOC, u, src_tier, src_slot if src_tier == CPU else NONE, GPU, y, 0)
            self.undefined[u] = True
        else:
            if self.full:
                self._gpu_view(s, y, n)[:] = incoming
            self._emit(step, phase, op_in, u, src_tier, src_slot if src_tier == CPU else NONE, GPU, y, n)
            if src_tier == CPU:
                self.bytes_h2d += n
            else:
                self.bytes_file_read += n
                self.bytes_h2d += n               # file -> staging -> GPU crosses the link too
        self.cur[u], self.gslot[u], self.cslot[u] = GPU, y, NONE
        self.gpu_owner[s][y] = u
        self.moved[u] = self.call

    # -- pre-hook ------------------------------------------------------------
    def pre(self, step: int, access: Sequence[Tuple[int, int]]) -> List[Optional[Tuple[int, int]]]:
        """Before a module runs every tensor it uses must be in a GPU buffer.

        A tensor already there is a hit; the decision is logical (it is in the
        active tensor window when the hook runs), lateness of an in-flight copy
        is stall time, not a miss.

        Reading (miss path, the paper only promises robustness to timing
        drift): a missing tensor is fetched on demand into the lowest free GPU
        buffer of its class, else in place of the resident tensor of the class,
        not used by this step and not moved by this call, whose next use
        counted from the step's first row is farthest (ties -> lowest id).  If
        neither exists the access FAILs and the tensor stays where it is.

        Returns (class, GPU buffer) per access, None for a failed one.
        """
        p = self.p
        self.call += 1
        bound = p.row_begin[step] if step < p.n_steps else p.n_rows
        in_step = {t for (t, _a) in access}
        h = m = 0
        out: List[Optional[Tuple[int, int]]] = []
        for (t, rw) in access:
            s = p.class_of[t]
            if self.cur[t] == GPU:
                h += 1
            else:
                m += 1
                y = self._lowest_free(self.gpu_owner[s], self.gpu_freed[s])
                v = NONE
                if y == NONE:
                    cands = [x for x in self.gpu_owner[s]
                             if x != NONE and x not in in_step and self.moved[x] != self.call]
                    v = self._farthest(cands, bound)
                    if v != NONE:
                        y = self.gslot[v]
                if y == NONE:
                    self.fails += 1
                    self._emit(step, PRE, FAIL, t, self.cur[t], NONE, GPU, NONE, 0)
                    out.append(None)
                    continue
                whole = self.alloc_write_only and rw == W_FLAG
                self._exchange(v, t, y, step, PRE, ALLOC if whole else DEMAND, bound)
            if (rw & R_FLAG) and self.undefined[t]:
                self.undefined_reads += 1
            if self.alloc_write_only and rw == W_FLAG:
                # the module's kernel writes the whole tensor: whatever it held is replaced
                self.dirty[t] = True
                self.undefined[t] = False
                self.whole_write[t] = (self.iteration, step)
                self.stamps[t] = []
                if self.full:
                    self._gpu_view(s, self.gslot[t], self.bytes_of[t])[:] = \
                        self._pattern(t, self.bytes_of[t], write_seed(self.iteration, step))
            elif rw & W_FLAG:
                # the module's kernel writes the tensor: stamp it, mark it dirty
                self.dirty[t] = True
                self.stamps[t].append((self.iteration, step))
                if self.full:
                    apply_stamp(self._gpu_view(s, self.gslot[t], self.bytes_of[t]),
                                stamp16(self.iteration, step, t))
            out.append((s, self.gslot[t]))
        self.hits += h
        self.misses += m
        self.step_hits.append((self.iteration, step, h, m))
        self.resident_at_pre.append(out)
        return out

    # -- post-hook: Alg. 3 -----------------------------------------------------
    def post(self, step: int, finished: Sequence[int]) -> None:
        """PrefetchTensor(finished tensors), Alg. 3.

        Reading (halt rule): Alg. 3 as printed evicts a finished tensor and
        may immediately prefetch it back, against the text of Sec. 3.4.1 (nothing
        is evicted or prefetched while the window holds what the backward pass
        needs next).  So the next non-resident row is
        found first, and a resident tensor gives up its buffer only if its
        own next use lies after that row.

        Reading (which buffer): the incoming tensor u needs a buffer of its
        own size.  The finished tensor t is evicted for it when t has u's size
        (and passes the halt rule); otherwise u takes the lowest free buffer of
        its class; otherwise the resident tensor of u's class used farthest in
        the future, provided that is later than u's own use (Sec. 3.4.2: the
        tensor evicted is one not needed for a while).  If none qualifies nothing moves and the row
        is tried again at the next call.  A finished tensor of another size
        keeps its buffer until a tensor of its own size needs it: evicting it
        would free nothing u can use, and with Alg. 2's c_s - G_s host buffers
        it could only be spilled to NVMe, which Sec. 3.4.1 rules out when GPU
        and CPU suffice.

        Reading: the cursor starts at row 0 and never lags the step that just
        finished; the bound of the skip loop is tested before the row is read;
        tensors moved by this call are in flight and are neither evicted nor
        prefetched again by it; rows of a class with no GPU buffer are skipped.
        """
        p = self.p
        self.call += 1
        if not self.prefetch:
            # the variant the paper calls the base version (Sec. 4.1.4: it does not
            # prefetch): the post-hook moves nothing, tensors arrive by the
            # pre-hook's demand fetch alone
            return
        n_rows = p.n_rows
        bound = p.row_end[step] if step < p.n_steps else n_rows
        self.cursor = max(self.cursor, bound)
        for t in finished:
            if self.cursor >= n_rows:                     # Alg. 3: the table has no row left
                break
            while self.cursor < n_rows and (
                    self.cur[p.rows_tensor[self.cursor]] == GPU
                    or self.plan.gpu_count[p.class_of[p.rows_tensor[self.cursor]]] == 0):
                self.cursor += 1                          # already in the active tensor window
            if self.cursor >= n_rows:
                break
            u = p.rows_tensor[self.cursor]
            if self.moved[u] == self.call:                # in flight
                break
            s = p.class_of[u]
            v, y = NONE, NONE
            if (p.class_of[t] == s and self.cur[t] == GPU and self.moved[t] != self.call
                    and p.next_use(t, bound) > self.cursor):
                v = t
                y = self.gslot[t]
            else:
                y = self._lowest_free(self.gpu_owner[s], self.gpu_freed[s])
                if y == NONE:
                    cands = [x for x in self.gpu_owner[s]
                             if x != NONE and self.moved[x] != self.call
                             and p.next_use(x, bound) > self.cursor]
                    v = self._farthest(cands, bound)
                    if v != NONE:
                        y = self.gslot[v]
            if y == NONE:
                continue                                  # nothing may leave: halt for this tensor
            whole = self.alloc_write_only and p.rows_rw[self.cursor] == W_FLAG
            self._exchange(v, u, y, step, POST, ALLOC if whole else PREFETCH, bound)
            self.cursor += 1

    # -- end of iteration ------------------------------------------------------
    def end_iteration(self) -> None:
        """Every tensor goes back to its final location (Sec. 3.2.1).

        Reading: the text gives no order.  The order taken moves every
        displaced tensor exactly once and no other tensor at all, so that
        restoring never writes a tensor to NVMe that GPU and CPU have room
        for (Sec. 3.4.1).  Three hook calls:

        1. class by class (ascending), GPU-final tensors sitting in host
           buffers come back, in placement order, into the lowest free GPU
           buffer or else in place of the lowest-id resident tensor whose
           final location is not the GPU.  That guest takes the host buffer
           the incoming tensor leaves (the two swap) or, if NVMe-final, goes
           to its file extent.
        2. GPU-final tensors on the file tier come back the same way; a
           CPU-final guest now finds a free host buffer, because every
           GPU-final tensor has left the host pool.
        3. CPU-final tensors on the file tier return to the lowest free host
           buffer, class by class in placement order.

        (Taking the tensors of calls 1 and 2 in one pass would make a CPU-final
        guest displaced by a tensor from the file tier spill a host tensor
        while GPU-final tensors still hold host buffers: that tensor would move
        twice.)  GPU-designated marks are cleared and the cursor returns to
        row 0.
        """
        p = self.p
        step = p.n_steps
        bound = p.n_rows
        n_c = len(p.count)
        members = [[t for t in self.pl.order if p.class_of[t] == s] for s in range(n_c)]
        for source in (CPU, NVME):
            self.call += 1
            for s in range(n_c):
                for u in members[s]:
                    if self.pl.final[u] != GPU or self.cur[u] != source:
                        continue
                    y = self._lowest_free(self.gpu_owner[s], self.gpu_freed[s])
                    v = NONE
                    if y == NONE:
                        guests = [x for x in self.gpu_owner[s]
                                  if x != NONE and self.pl.final[x] != GPU and self.moved[x] != self.call]
                        if not guests:
                            continue
                        v = min(guests)
                        y = self.gslot[v]
                    self._exchange(v, u, y, step, END, PREFETCH, bound)
        self.call += 1
        for s in range(n_c):
            for u in members[s]:
                if self.pl.final[u] != CPU or self.cur[u] != NVME:
                    continue
                x = self._lowest_free(self.cpu_owner[s], self.cpu_freed[s])
                if x == NONE:
                    continue
                n = self.bytes_of[u]
                if self.full:
                    self._cpu_view(s, x, n)[:] = self._file_view(u)
                self._emit(step, END_CPU, RESTORE, u, NVME, NONE, CPU, x, n)
                self.bytes_file_read += n
                self.cur[u], self.cslot[u] = CPU, x
                self.cpu_owner[s][x] = u
                self.moved[u] = self.call
            for k in range(len(self.designated[s])):
                self.designated[s][k] = False
        self.cursor = 0
        self.iteration += 1

    # -- whole-trace driver ----------------------------------------------------
    def run_iteration(self, steps: Sequence[Sequence[Tuple[int, int]]], check=None) -> None:
        for k, access in enumerate(steps):
            self.pre(k, access)
            if check:
                check(self, k, access, PRE)
            self.post(k, [t for (t, _a) in access])
            if check:
                check(self, k, access, POST)
        self.end_iteration()
        if check:
            check(self, len(steps), [], END)


def build(tensor_bytes, tensor_group, ev_step, ev_tensor, ev_rw, hbm_bytes, host_bytes,
          align=256, literal=False, payload=None, prefetch=True, smallest_first=False,
          alloc_write_only=False, pattern=None):
    """Profile, plan, place and return a Replay ready at iteration 0."""
    p = profile(tensor_bytes, tensor_group, ev_step, ev_tensor, ev_rw)
    plan = plan_pools(p, hbm_bytes, host_bytes, align, literal, smallest_first)
    pl = place(p, plan)
    return Replay(p, plan, pl, payload, prefetch, alloc_write_only, pattern)


def replay_workload(wl, payload=None, check=None, pattern=None) -> Replay:
    """Run every iteration of a workload object (see the workloads package)."""
    st, te, rw, _ns = wl.events()
    r = build(wl.tensor_bytes.tolist(), wl.tensor_group.tolist(), st, te, rw,
              wl.hbm_bytes, wl.host_bytes, wl.align, wl.literal_alg2, payload,
              prefetch=not getattr(wl, "no_prefetch", False),
              smallest_first=getattr(wl, "smallest_first", False),
              alloc_write_only=getattr(wl, "alloc_write_only", False), pattern=pattern)
    for steps in wl.iterations:
        r.run_iteration(steps, check)
    return r
