"""Tensor tables, access traces and budgets of the synthetic workloads.

Five transformer-shaped configurations stand in for the Hugging Face models
and GLUE/Wikitext runs the paper trained on (its Sec. 4.1): a migration path
sees only tensor sizes, the access order and the bytes, so the traces take the
shape of those workloads (layer-regular dense transformers; forward, then the
backward pass in reverse order, then the optimizer sweep: Sec. 2.1 and the
illustrative example of Sec. 3.3.2) and nothing else of them.

A *step* is one leaf-module hook pair (Sec. 3.2.1).  Every parameter tensor j
owns five tensors with ids 5j+k: k=0 16-bit parameter, 1 16-bit gradient,
2 fp32 master copy, 3 Adam momentum, 4 Adam variance (Sec. 2.1: 2N+2N+4N+4N+4N
bytes).  Activation-checkpoint tensors, where a configuration has them, take
the ids after the last parameter.

Only input generation lives here; nothing in this file sizes pools, places
tensors or decides a migration.
"""

from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Sequence, Tuple

import numpy as np

R, W, RW = 1, 2, 3
GROUP_16, GROUP_32 = 0, 1
KIND_P16, KIND_G16, KIND_MASTER, KIND_M, KIND_V, KIND_CKPT = range(6)
PHASE_FORWARD, PHASE_BACKWARD, PHASE_OPTIMIZER = range(3)

GiB = 1 << 30
VOCAB_SHARD_ROWS = 4096

Step = List[Tuple[int, int]]          # [(tensor id, rw), ...]


@dataclass
class Workload:
    """One synthetic workload: what the profiler saw and what is replayed."""

    name: str
    tensor_bytes: np.ndarray                  # uint64 [n_tensors]
    tensor_group: np.ndarray                  # uint8  [n_tensors] 0 = 16-bit, 1 = fp32
    tensor_kind: np.ndarray                   # uint8  [n_tensors] KIND_*
    profile: List[Step]                       # the profiled iteration
    compute_ns: np.ndarray                    # uint64 [n_steps] modelled compute per step
    hbm_bytes: int                            # HBM cache budget
    host_bytes: Tuple[int, int]               # pinned-host budget per group
    iterations: List[List[Step]] = field(default_factory=list)   # replayed iterations
    align: int = 256
    literal_alg2: bool = False                # Alg. 2 without the working-set floor
    no_prefetch: bool = False                 # replay the paper's base variant: demand fetch only
    smallest_first: bool = False              # GPU buffers to the smallest tensors first (the baseline placement)
    alloc_write_only: bool = False            # write-only accesses are whole-tensor writes: no fetch for them
    gaussian_p16: bool = False                # 16-bit params are fp16(N(0, 0.02))
    notes: str = ""
    step_phase: np.ndarray | None = None      # uint8 [n_steps]: 0 forward, 1 backward, 2 optimizer sweep (None: not known)

    @property
    def n_tensors(self) -> int:
        return int(self.tensor_bytes.shape[0])

    @property
    def n_steps(self) -> int:
        return len(self.profile)

    def events(self):
        """The profiled iteration as flat event arrays (step, tensor, rw, compute_ns)."""
        step, tensor, rw, ns = [], [], [], []
        for k, st in enumerate(self.profile):
            for (t, a) in st:
                step.append(k)
                tensor.append(t)
                rw.append(a)
                ns.append(int(self.compute_ns[k]))
        return (np.asarray(step, dtype=np.uint32), np.asarray(tensor, dtype=np.uint32),
                np.asarray(rw, dtype=np.uint8), np.asarray(ns, dtype=np.uint64))

    def total_bytes(self) -> int:
        return int(self.tensor_bytes.sum())


# --------------------------------------------------------------------------
# counter-based generator used for the seeded perturbation of config 5
# --------------------------------------------------------------------------

class splitmix64:
    """SplitMix64 (Steele, Lea, Flood 2014): a 64-bit counter-based generator."""

    MASK = (1 << 64) - 1

    def __init__(self, seed: int):
        self.state = seed & self.MASK

    def next(self) -> int:
        self.state = (self.state + 0x9E3779B97F4A7C15) & self.MASK
        z = self.state
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & self.MASK
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & self.MASK
        return z ^ (z >> 31)


def perturb_iteration(steps: List[Step], n_tensors: int, seed: int, one_in: int = 100) -> List[Step]:
    """Replace the accessed tensor id of about one row in `one_in` by a random id.

    One draw per row decides; a second draw picks the replacement.  Row
    positions and rw flags stay aligned with the profiled iteration: only the
    id changes (order drift, not timing drift).
    """
    g = splitmix64(seed)
    out: List[Step] = []
    for st in steps:
        new: Step = []
        for (t, a) in st:
            if g.next() % one_in == 0:
                t = g.next() % n_tensors
            new.append((int(t), a))
        out.append(new)
    return out


# --------------------------------------------------------------------------
# transformer-shaped tensor tables
# --------------------------------------------------------------------------

def _vocab_shards(vocab: int) -> List[int]:
    rows, left = [], vocab
    while left > 0:
        rows.append(min(VOCAB_SHARD_ROWS, left))
        left -= rows[-1]
    return rows


class _Builder:
    def __init__(self):
        self.param_elems: List[int] = []     # elements of parameter tensor j
        self.modules: List[List[int]] = []   # forward-order leaf modules -> param indices
        self.block_end: List[int] = []       # module index after which block l ends

    def module(self, *elems: int) -> int:
        idx = []
        for e in elems:
            idx.append(len(self.param_elems))
            self.param_elems.append(int(e))
        self.modules.append(idx)
        return len(self.modules) - 1


def _assemble(name, b: _Builder, head_modules: List[List[int]], *, ckpt_bytes: int, n_blocks: int,
              first_block_module: int, modules_per_block: int, with_optimizer: bool,
              tokens: int, hbm_bytes, host_bytes, n_iterations: int, gaussian_p16=False,
              notes="") -> Workload:
    n_p = len(b.param_elems)
    n_ckpt = n_blocks if ckpt_bytes else 0
    n_t = 5 * n_p + n_ckpt
    tb = np.zeros(n_t, dtype=np.uint64)
    tg = np.zeros(n_t, dtype=np.uint8)
    tk = np.zeros(n_t, dtype=np.uint8)
    for j, e in enumerate(b.param_elems):
        for k in range(5):
            tb[5 * j + k] = e * (2 if k < 2 else 4)
            tg[5 * j + k] = GROUP_16 if k < 2 else GROUP_32
            tk[5 * j + k] = k
    for l in range(n_ckpt):
        tb[5 * n_p + l] = ckpt_bytes
        tg[5 * n_p + l] = GROUP_16
        tk[5 * n_p + l] = KIND_CKPT

    # modelled compute: 2*elems*tokens flops forward, 4*... backward at a fixed
    # effective rate; optimizer steps are elementwise and HBM-bound.
    FLOP_RATE = 1.0e15          # flop/s, effective dense 16-bit rate assumed for the model
    HBM_RATE = 4.0e12           # B/s, effective elementwise rate assumed for the optimizer
    fwd: List[Step] = []
    fwd_ns: List[int] = []
    all_modules = list(b.modules) + head_modules
    n_body = len(b.modules)
    for mi, params in enumerate(all_modules):
        fwd.append([(5 * j, R) for j in params])
        fwd_ns.append(int(sum(2.0 * b.param_elems[j] * tokens for j in params) / FLOP_RATE * 1e9))
        if ckpt_bytes and mi < n_body and mi >= first_block_module:
            l, pos = divmod(mi - first_block_module, modules_per_block)
            if l < n_blocks and pos == modules_per_block - 1:
                fwd.append([(5 * n_p + l, W)])
                fwd_ns.append(int(ckpt_bytes / HBM_RATE * 1e9))
    bwd: List[Step] = []
    bwd_ns: List[int] = []
    for st, ns in zip(reversed(fwd), reversed(fwd_ns)):
        if st[0][0] >= 5 * n_p:                      # checkpoint step: read it back
            bwd.append([(st[0][0], R)])
            bwd_ns.append(ns)
        else:
            new: Step = []
            for (t, _a) in st:
                new.append((t, R))
                new.append((t + 1, W))
            bwd.append(new)
            bwd_ns.append(2 * ns)
    steps = fwd + bwd
    ns_all = fwd_ns + bwd_ns
    phase = [PHASE_FORWARD] * len(fwd) + [PHASE_BACKWARD] * len(bwd)
    if with_optimizer:
        for j in range(n_p):
            steps.append([(5 * j + 1, R), (5 * j + 2, RW), (5 * j + 3, RW), (5 * j + 4, RW), (5 * j, W)])
            ns_all.append(int(16.0 * b.param_elems[j] * 2 / HBM_RATE * 1e9))
            phase.append(PHASE_OPTIMIZER)
    wl = Workload(name=name, tensor_bytes=tb, tensor_group=tg, tensor_kind=tk, profile=steps,
                  compute_ns=np.asarray(ns_all, dtype=np.uint64),
                  hbm_bytes=0, host_bytes=(0, 0), gaussian_p16=gaussian_p16, notes=notes,
                  step_phase=np.asarray(phase, dtype=np.uint8))
    wl.hbm_bytes = int(hbm_bytes(wl) if callable(hbm_bytes) else hbm_bytes)
    hb = host_bytes(wl) if callable(host_bytes) else host_bytes
    wl.host_bytes = (int(hb[0]), int(hb[1]))
    wl.iterations = [steps for _ in range(n_iterations)]
    return wl


def gpt_shaped(name: str, *, layers: int, hidden: int, ffn: int, vocab: int, positions: int = 1024,
               ckpt_bytes: int = 0, with_optimizer: bool = True, tokens: int = 8192,
               hbm_bytes=0, host_bytes=(0, 0), n_iterations: int = 1, gaussian_p16=False,
               notes="") -> Workload:
    """GPT-shaped table: sharded token table, position table, per layer
    ln1{w,b} qkv{W,b} out{W,b} ln2{w,b} fc1{W,b} fc2{W,b}, final ln{w,b}, and a
    tied output head that re-reads the token-table shards."""
    h, f = hidden, ffn
    b = _Builder()
    shards = [b.module(rows * h) for rows in _vocab_shards(vocab)]
    b.module(positions * h)
    first_block = len(b.modules)
    for _ in range(layers):
        b.module(h, h)
        b.module(h * 3 * h, 3 * h)
        b.module(h * h, h)
        b.module(h, h)
        b.module(h * f, f)
        b.module(f * h, h)
    b.module(h, h)
    head = [list(b.modules[m]) for m in shards]       # tied: same parameter tensors again
    return _assemble(name, b, head, ckpt_bytes=ckpt_bytes, n_blocks=layers,
                     first_block_module=first_block, modules_per_block=6,
                     with_optimizer=with_optimizer, tokens=tokens, hbm_bytes=hbm_bytes,
                     host_bytes=host_bytes, n_iterations=n_iterations,
                     gaussian_p16=gaussian_p16, notes=notes)


def llama_shaped(name: str, *, layers: int, hidden: int, ffn: int, vocab: int,
                 ckpt_bytes: int = 0, with_optimizer: bool = True, tokens: int = 8192,
                 hbm_bytes=0, host_bytes=(0, 0), n_iterations: int = 1, notes="") -> Workload:
    """Llama-shaped table: sharded embedding, per layer rms1 wq wk wv wo rms2
    gate up down (no biases, one tensor per leaf module), final rms, and an
    untied sharded output head."""
    h, f = hidden, ffn
    b = _Builder()
    for rows in _vocab_shards(vocab):
        b.module(rows * h)
    first_block = len(b.modules)
    for _ in range(layers):
        b.module(h)
        for _q in range(4):
            b.module(h * h)
        b.module(h)
        b.module(h * f)
        b.module(h * f)
        b.module(f * h)
    b.module(h)
    for rows in _vocab_shards(vocab):
        b.module(rows * h)                              # untied head: its own tensors
    return _assemble(name, b, [], ckpt_bytes=ckpt_bytes, n_blocks=layers,
                     first_block_module=first_block, modules_per_block=9,
                     with_optimizer=with_optimizer, tokens=tokens, hbm_bytes=hbm_bytes,
                     host_bytes=host_bytes, n_iterations=n_iterations, notes=notes)


def optimizer_sweep(name: str, *, layers: int, hidden: int, ffn: int, vocab: int, cache_frac: float,
                    n_iterations: int = 2, cpu_bytes_per_s: float = 20.0e9, notes="") -> Workload:
    """The optimizer step on the CPU as a workload of its own (Sec. 3.4.2,
    optimizer states scheduling policy): per parameter tensor of a
    Llama-shaped model three fp32 state tensors (master copy, momentum,
    variance; ids 3j, 3j+1, 3j+2), read and written by step j of a sweep over
    the parameters.  Two tiers: `hbm_bytes` is the budget of the fast tier (the
    CPU cache), cache_frac of all states; both host budgets are 0, so whatever
    does not fit lives on the file tier.  compute_ns models the CPU's Adam
    update as bound by memory traffic (28 bytes per element: gradient and three
    states read, three states written) at cpu_bytes_per_s."""
    h, f = hidden, ffn
    elems: List[int] = [rows * h for rows in _vocab_shards(vocab)]
    for _ in range(layers):
        elems += [h, h * h, h * h, h * h, h * h, h, h * f, h * f, f * h]
    elems += [h] + [rows * h for rows in _vocab_shards(vocab)]
    n_p = len(elems)
    tb = np.repeat(np.asarray(elems, dtype=np.uint64) * 4, 3)
    kinds = np.tile(np.asarray([KIND_MASTER, KIND_M, KIND_V], dtype=np.uint8), n_p)
    steps: List[Step] = [[(3 * j, RW), (3 * j + 1, RW), (3 * j + 2, RW)] for j in range(n_p)]
    ns = np.asarray([int(28.0 * e / cpu_bytes_per_s * 1e9) for e in elems], dtype=np.uint64)
    wl = Workload(name=name, tensor_bytes=tb, tensor_group=np.full(3 * n_p, GROUP_32, dtype=np.uint8),
                  tensor_kind=kinds, profile=steps, compute_ns=ns,
                  hbm_bytes=int(float(tb.sum()) * cache_frac), host_bytes=(0, 0), notes=notes)
    wl.iterations = [steps for _ in range(n_iterations)]
    return wl


def _ample_host(wl: Workload):
    g = wl.tensor_group
    return (int(wl.tensor_bytes[g == 0].sum()) + (1 << 20), int(wl.tensor_bytes[g == 1].sum()) + (1 << 20))


_CONFIGS = ("gpt2_small", "gpt_1p3b_ckpt", "llama_7b", "llama_13b_ckpt_nvme", "llama_30b_perturbed")


def config_names() -> Sequence[str]:
    return _CONFIGS


def config(index: int, *, layers: int | None = None) -> Workload:
    """The five benchmark configurations (index 0..4).

    `layers` overrides the layer count (same shapes, shallower model) for runs
    on boxes that cannot hold the full footprint; budgets that are fractions
    scale with it, absolute ones scale in proportion to the layer count.
    """
    if index == 0:
        L = 12 if layers is None else layers
        # The optimizer sweep is not replayed here: with per-class working
        # sets (2 slots per 16-bit class, 3 per fp32 class) it alone needs
        # about 152 MB of HBM, more than this configuration's 25 % cache.
        return gpt_shaped(
            "gpt2_small", layers=L, hidden=768, ffn=3072, vocab=50257, with_optimizer=False,
            tokens=8 * 1024,
            hbm_bytes=lambda w: int(w.tensor_bytes[w.tensor_kind == KIND_P16].sum()) // 4,
            host_bytes=_ample_host, gaussian_p16=True,
            notes="forward + reverse backward; Adam states exist but are never accessed on the GPU")
    if index == 1:
        L = 24 if layers is None else layers
        return gpt_shaped(
            "gpt_1p3b_ckpt", layers=L, hidden=2048, ffn=8192, vocab=50257,
            ckpt_bytes=4 * 1024 * 2048 * 2, tokens=4 * 1024,
            hbm_bytes=lambda w: w.total_bytes() * 15 // 100, host_bytes=_ample_host)
    if index == 2:
        L = 32 if layers is None else layers
        return llama_shaped(
            "llama_7b", layers=L, hidden=4096, ffn=11008, vocab=32000, tokens=4 * 2048,
            hbm_bytes=40 * GiB * L // 32, host_bytes=_ample_host, n_iterations=3)
    if index == 3:
        L = 40 if layers is None else layers
        return llama_shaped(
            "llama_13b_ckpt_nvme", layers=L, hidden=5120, ffn=13824, vocab=32000,
            ckpt_bytes=8 * 2048 * 5120 * 2, tokens=8 * 2048,
            hbm_bytes=60 * GiB * L // 40,
            host_bytes=lambda w: (_ample_host(w)[0], 0),
            notes="fp32 optimizer states have no host pool: file tier")
    if index == 4:
        L = 60 if layers is None else layers
        wl = llama_shaped(
            "llama_30b_perturbed", layers=L, hidden=6656, ffn=17920, vocab=32000, tokens=4 * 2048,
            hbm_bytes=200 * GiB * L // 60, host_bytes=(64 * GiB * L // 60, 96 * GiB * L // 60),
            notes="1 % of accesses replaced by seeded random ids")
        wl.iterations = [perturb_iteration(wl.profile, wl.n_tensors, seed=0)]
        return wl
    raise IndexError(index)


def scaled_config(index: int, layers: int) -> Workload:
    return config(index, layers=layers)


# --------------------------------------------------------------------------
# tiny hand traces
# --------------------------------------------------------------------------

def _simple(name, sizes, groups, steps, hbm_bytes, host_bytes, *, literal=True, align=256,
            n_iterations=1) -> Workload:
    n = len(sizes)
    wl = Workload(name=name, tensor_bytes=np.asarray(sizes, dtype=np.uint64),
                  tensor_group=np.asarray(groups, dtype=np.uint8),
                  tensor_kind=np.zeros(n, dtype=np.uint8), profile=steps,
                  compute_ns=np.full(len(steps), 1000, dtype=np.uint64),
                  hbm_bytes=int(hbm_bytes), host_bytes=(int(host_bytes[0]), int(host_bytes[1])),
                  align=align, literal_alg2=literal)
    wl.iterations = [steps for _ in range(n_iterations)]
    return wl


def single_class_fwd_bwd(n: int, k_gpu: int, k_cpu: int, *, size: int = 512, n_iterations: int = 1,
                         rw_bwd: int = R) -> Workload:
    """n equal-size tensors used 0..n-1 forward then n-1..0 backward, with room
    for exactly k_gpu tensors in HBM and k_cpu in host buffers (Alg. 2 without
    the working-set floor, so the closed form applies)."""
    steps = [[(t, R)] for t in range(n)] + [[(t, rw_bwd)] for t in reversed(range(n))]
    return _simple(f"single{n}_{k_gpu}_{k_cpu}", [size] * n, [0] * n, steps,
                   hbm_bytes=k_gpu * size, host_bytes=(k_cpu * size, 0), n_iterations=n_iterations)


def single_class_sweep(n: int, k_fast: int, *, size: int = 512, n_iterations: int = 1) -> Workload:
    """n equal-size fp32 state tensors updated (read and written) one per step
    in the order 0..n-1, a fast tier with room for exactly k_fast of them and
    no host buffers below it: the optimizer-state example of Sec. 3.4.2 (its
    figure has n = 8, k_fast = 5; ids here are the paper's minus 1)."""
    steps = [[(t, RW)] for t in range(n)]
    return _simple(f"sweep{n}_{k_fast}", [size] * n, [GROUP_32] * n, steps,
                   hbm_bytes=k_fast * size, host_bytes=(0, 0), n_iterations=n_iterations)


def example_cpu_gpu() -> Workload:
    """Six equal tensors, three HBM buffers, three host buffers: the CPU-GPU
    offloading example of Sec. 3.4.1 (tensor ids here are the paper's minus 1)."""
    return single_class_fwd_bwd(6, 3, 3)


def example_cpu_gpu_nvme() -> Workload:
    """Seven equal tensors, three HBM buffers, three host buffers, the seventh
    tensor on the file tier: the equal-size variant of the CPU-GPU-NVMe example
    of Sec. 3.4.2 (ids are the paper's minus 1)."""
    return single_class_fwd_bwd(7, 3, 3)


def example_cpu_gpu_nvme_two_sizes() -> Workload:
    """The CPU-GPU-NVMe example of Sec. 3.4.2 with the sizes its text implies: the text
    spills tensor 2 because it "has the same size as tensor 4", so not every tensor has
    that size.  Tensors 2, 4 and 7 (paper ids) are 1024 bytes, tensors 1, 3, 5 and 6 are
    512; budgets of half of all bytes on the GPU and half below it give Alg. 2 two + one
    GPU buffers and two + one host buffers, and the allocator GPU {1,2,3}, CPU {4,5,6},
    NVMe {7} as the figure has it.  Ids here are the paper's minus 1."""
    small, large = 512, 1024
    sizes = [small, large, small, large, small, small, large]
    n = len(sizes)
    steps = [[(t, R)] for t in range(n)] + [[(t, R)] for t in reversed(range(n))]
    total = sum(sizes)
    return _simple("example_cpu_gpu_nvme_two_sizes", sizes, [0] * n, steps, hbm_bytes=total // 2,
                   host_bytes=(total // 2, 0))


def random_workload(seed: int, *, n_tensors: int = 24, n_steps: int = 40, max_per_step: int = 3,
                    sizes: Sequence[int] = (512, 1024, 4096, 100, 33000), hbm_frac: float = 0.4,
                    host_frac: float = 0.4, two_groups: bool = True, n_iterations: int = 2,
                    literal: bool = False, perturb_one_in: int = 0) -> Workload:
    """A seeded random multi-class trace: random sizes from a small set, random
    steps of 1..max_per_step distinct tensors with random rw flags."""
    rng = np.random.default_rng(seed)
    sz = rng.choice(np.asarray(sizes), size=n_tensors)
    gr = rng.integers(0, 2, size=n_tensors) if two_groups else np.zeros(n_tensors, dtype=np.int64)
    steps: List[Step] = []
    for _ in range(n_steps):
        m = int(rng.integers(1, max_per_step + 1))
        ids = rng.choice(n_tensors, size=m, replace=False)
        steps.append([(int(t), int(rng.integers(1, 4))) for t in ids])
    total = int(sz.sum())
    stride = (sz + 255) // 256 * 256
    hb0 = int(stride[gr == 0].sum() * host_frac)
    hb1 = int(stride[gr == 1].sum() * host_frac)
    # HBM budget: a fraction of all bytes plus max_per_step buffers of every
    # distinct (size, group) pair, so that any one step always fits.
    pairs = sorted({(int(s), int(g)) for s, g in zip(stride, gr)})
    hbm = int(total * hbm_frac)
    if not literal:
        hbm += max_per_step * sum(s for s, _g in pairs)
    wl = _simple(f"random{seed}", sz.tolist(), gr.tolist(), steps, hbm_bytes=hbm,
                 host_bytes=(hb0, hb1), literal=literal, n_iterations=n_iterations)
    if perturb_one_in:
        wl.iterations = [perturb_iteration(steps, n_tensors, seed=seed + 1000 + i, one_in=perturb_one_in)
                         for i in range(n_iterations)]
    return wl
