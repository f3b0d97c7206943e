"""Live profiling and hook-driven migration for a PyTorch module.

The paper's tensor characteristic analyzer (Sec. 3.2.1) registers a pre-hook
and a post-hook on every module, records execution order and tensor sizes in
one dry-run iteration, and the scheduler (Sec. 3.4) is then driven by the same
hooks.  `ParamCache` does that for the parameters of an `nn.Module` on top of
the C-ABI library:

    pc = ParamCache(model, hbm_bytes=...)
    pc.profile(lambda: loss_fn(model(x), y).backward())   # dry run: order + sizes
    pc.install()                                          # plan, place, move the parameters out
    for batch in data:
        loss_fn(model(x), y).backward()                   # hooks fetch / evict around every module
        pc.sgd_step(lr)                                   # parameters pass through the cache once more
        pc.end_iteration()

`ParamCache(..., dma_threshold=65536)` sends the larger parameters through the DMA engines
while there is compute to hide the copies behind (the zero-copy kernel is faster on the link but
slows the compute that runs beside it); `autotune_dma(step)` lets a few training steps choose.

With `ParamCache(..., fused_sgd_lr=lr)` the update of a module's parameters is
applied in its backward post-hook instead, while they are still in their cache
buffers: no third pass, a third less traffic; `sgd_step` is then not called.

With `ParamCache(..., host_bytes=..., file_path=...)` what neither the HBM cache nor that much pinned
host memory hold lives in a file (the paper's CPU-GPU-NVMe set-up, Sec. 3.4.2): fetched through a
pinned staging ring by the library's reader threads, spilled and written back by its writer threads.

With `ParamCache(..., manage_grads=True)` the gradients are tensors of the cache
too (Sec. 3.2.1's hooks cover every tensor a layer touches; Sec. 2.1 counts the
16-bit gradients beside the parameters): a module's backward step names its
parameters (read) and their gradients (written), each gradient autograd hands
over is copied into its cache buffer and dropped, and the optimizer sweep's
step for a parameter names the gradient (read) and the parameter (read and
written).  Outside those steps a gradient lives wherever the scheduler put it,
and `p.grad` is None.

With `ParamCache(..., state_tensors=2)` every managed parameter has that many fp32 optimizer-state
tensors of its shape in the cache as well (the north star's "parameter, gradient and optimizer
tensors"): the parameter's step of the update sweep names them read and written, `update_sweep`
hands them to the update, and `adam_step` is Adam over them (first and second moment).

A parameter shared by two modules (tied weights) and a module that runs twice in
a pass are handled in the parameters-only mode: such a use's backward step is
closed when the gradients of its own inputs arrive, not when its parameters'
gradients do (those are complete only after the last use).

What is managed are the parameters of the modules that own parameters and call no other module that
does (the leaves of the model as far as parameters go: Linear, LayerNorm, Embedding ...).  A module
that owns parameters AND calls such modules (a root module with a position table of its own, say)
uses its parameters across its children's steps, where nothing protects them from eviction: its own
parameters stay ordinary resident tensors (`ParamCache.resident`), and so do those of the modules
named in `resident_modules` (for a module whose parameters are used without its forward being called,
as the output projection inside `nn.MultiheadAttention` is; the dry run refuses such a module
otherwise).  `sgd_step` and `gather` cover the resident parameters too.

Between its pre-hook and its post-hook a module's parameters are views into
the HBM cache buffers the library returned; outside that window they point
nowhere useful and must not be touched.  A parameter may come back for the
backward pass in another buffer than the one it had in the forward pass, and
autograd keeps for the backward whatever tensor the forward handed it (for a
Linear layer a transposed view of the weight, tied to the old buffer).  During
a managed module's forward the helper therefore installs saved-tensor hooks:
a tensor that aliases one of the module's parameters is saved as "parameter t,
this shape, stride and offset" and rebuilt from the parameter's current buffer
when the backward pass asks for it.  Without `manage_grads` gradients stay
ordinary PyTorch tensors (the FP16-parameter policy of Sec. 3.4.2).  This is a
way to drive the library from real modules, not a training framework.

Only argument marshalling and hook bookkeeping happen here; decisions and
copies are the library's kernels.
"""

from __future__ import annotations

import time
from typing import Callable, Dict, List, Optional, Tuple

import numpy as np

from . import binding as T

R, W, RW = 1, 2, 3


class _ParamRef:
    """What autograd keeps in place of a tensor that aliases managed parameter t."""
    __slots__ = ("t", "shape", "stride", "offset")

    def __init__(self, t, shape, stride, offset):
        self.t, self.shape, self.stride, self.offset = t, shape, stride, offset


class ParamCache:
    def __init__(self, model, hbm_bytes: int, host_bytes: Optional[int] = None, align: int = 256,
                 fused_sgd_lr: Optional[float] = None, dma_threshold: Optional[int] = None,
                 manage_grads: bool = False, resident_modules=(), file_path: Optional[str] = None,
                 stripes: int = 1, state_tensors: int = 0, keep_oplog: bool = False):
        import torch
        self.torch = torch
        self.model = model
        self.hbm_bytes = int(hbm_bytes)
        self.host_bytes = host_bytes
        self.align = align
        self.fused_sgd_lr = fused_sgd_lr                  # plain SGD applied in the backward post-hook
        if manage_grads and fused_sgd_lr is not None:
            raise ValueError("with the update in the backward hooks no gradient outlives its module: nothing to manage")
        self.manage_grads = manage_grads                  # gradients are tensors of the cache too (ids n_params + t)
        # a file for what neither the HBM cache nor `host_bytes` of pinned memory hold (the paper's
        # CPU-GPU-NVMe set-up, Sec. 3.4.2), optionally striped over file_path, file_path.1, ...
        self.file_path, self.stripes = file_path, int(stripes)
        self.keep_oplog = keep_oplog                      # the library's op log: 32 bytes per decision, for ever (for tests)
        # optimizer states through the same cache: per managed parameter this many fp32 tensors of its
        # shape, zero at first, named (read and written) by the parameter's step of the update sweep
        self.state_tensors = int(state_tensors)
        if self.state_tensors and fused_sgd_lr is not None:
            raise ValueError("optimizer states are tensors of the update sweep; with the update in the backward hooks there is none")
        # parameters of at least this many bytes travel as DMA-engine copies instead of through the
        # zero-copy kernel: slower on the link, but compute running beside them is hardly slowed
        self.dma_threshold = dma_threshold
        # managed: the modules that own parameters and call no other module that does.  A module above such
        # a module uses its own parameters across its children's steps (nothing would keep them in their
        # buffers there): those stay resident, like the parameters of the modules the caller names.
        def owns(m):
            return any(True for _ in m.parameters(recurse=False))
        keep_out = {id(m) for r in resident_modules for m in r.modules()}
        owners = [m for m in model.modules() if owns(m)]
        self.mods = [m for m in owners
                     if id(m) not in keep_out and not any(c is not m and owns(c) for c in m.modules())]
        self.params: List = []
        self.pid: Dict[int, int] = {}
        for m in self.mods:
            for p in m.parameters(recurse=False):
                if id(p) not in self.pid:
                    self.pid[id(p)] = len(self.params)
                    self.params.append(p)
        if not self.params:
            raise ValueError("no module of this model owns parameters the cache could manage")
        self.resident: List = []                          # parameters left where they are
        for p in model.parameters():
            if id(p) not in self.pid:
                self.resident.append(p)
        # model.parameters() order -> managed index or resident tensor (for gather)
        self._order = [self.pid.get(id(p), p) for p in model.parameters()]
        per_step = 2 if manage_grads else 1
        if any(per_step * len(list(m.parameters(recurse=False))) > T.MAX_STEP_TENSORS for m in self.mods):
            raise ValueError("a module owns more parameters than one hook call may name")
        self.mod_ids = {id(m): [self.pid[id(p)] for p in m.parameters(recurse=False)] for m in self.mods}
        n_p = len(self.params)
        # what a module's steps name: forward its parameters (read); backward the same, or, with managed
        # gradients, the parameters (read) and behind them their gradients (written)
        self._step_lists: Dict[Tuple[int, str], Tuple[list, np.ndarray, np.ndarray]] = {}
        for k, ids in self.mod_ids.items():
            self._step_lists[(k, "fwd")] = (ids, np.asarray(ids, dtype=np.uint32), np.full(len(ids), R, dtype=np.uint8))
            if manage_grads:
                both = ids + [n_p + t for t in ids]
                flags = [R] * len(ids) + [W] * len(ids)
            else:
                both, flags = ids, [R if fused_sgd_lr is None else RW] * len(ids)
            self._step_lists[(k, "bwd")] = (both, np.asarray(both, dtype=np.uint32), np.asarray(flags, dtype=np.uint8))
        self._grad_view: Dict[int, object] = {}           # parameter -> its gradient's cache buffer, during a step that names it
        self._views: Dict[Tuple[int, int], object] = {}   # (parameter, buffer address) -> view into the HBM region
        self._hbm_base = 0
        self.steps: List[List[Tuple[int, int]]] = []      # the profiled iteration
        self.tc: Optional[T.TensorCache] = None
        self._handles: list = []
        self._k = 0                                       # next step of the running iteration
        self._recording = False
        self._pending_bwd: Dict[int, int] = {}            # module -> parameters whose gradient is still due
        self._bwd_step: Dict[int, int] = {}               # module -> step index of its running backward
        self._fwd_step: Dict[int, int] = {}               # module -> step index of its running forward
        self._saving_for: Tuple[int, ...] = ()            # parameters of the module whose forward is running
        self._saved_ctx: Dict[int, object] = {}           # module -> its saved-tensor hooks, while its forward runs
        if any(not p.requires_grad for p in self.params):
            raise ValueError("every managed parameter must require a gradient (its post-hook waits for it)")
        # A module's backward step is normally closed when the gradients of its parameters have arrived.
        # That does not work where a parameter is shared by two modules (tied weights) or a module runs
        # twice in a pass: the gradient arrives only after the last of the uses, and the steps of the
        # earlier ones would stay open across other modules' steps.  Such a use is closed instead when
        # the gradients of its own inputs arrive (the kernels that read its parameters are queued by
        # then); a use without an input that needs a gradient (an embedding) falls back to the rule above.
        owned_by: Dict[int, list] = {}
        for m in self.mods:
            for p in m.parameters(recurse=False):
                owned_by.setdefault(id(p), []).append(m)
        self._by_input = {id(m) for ms in owned_by.values() if len(ms) > 1 for m in ms}
        self._uses: Dict[int, int] = {}                   # module -> forward calls in the running iteration
        self._next_use = 0
        self._open_use: Dict[int, int] = {}               # module -> the use whose forward is running
        self._use_inputs: Dict[int, int] = {}             # use -> input gradients still due
        self._use_step: Dict[int, int] = {}               # use -> step index of its running backward
        self._ran: Dict[int, bool] = {}                   # module -> its forward ran in the dry run
        self._check_by_input()

    def _check_by_input(self):
        if self._by_input and (self.fused_sgd_lr is not None or self.manage_grads):
            raise ValueError("shared parameters and modules used twice in a pass are supported for parameters with a "
                             "separate update sweep only (their gradients are complete only after the last use)")

    # ------------------------------------------------------------------ hooks
    def _register(self):
        for m in self.mods:
            self._handles.append(m.register_forward_pre_hook(self._fwd_pre))
            self._handles.append(m.register_forward_hook(self._fwd_post))
            for p in m.parameters(recurse=False):
                self._handles.append(p.register_post_accumulate_grad_hook(self._make_grad_done(m, self.pid[id(p)])))

    def _remove(self):
        for h in self._handles:
            h.remove()
        self._handles = []

    def _begin(self, m, kind: str) -> int:
        """Opens the next step for module m (steps are numbered in the order they open)."""
        ids, ids_np, rw_np = self._step_lists[(id(m), kind)]
        k = self._k
        self._k += 1
        if self._recording:
            self.steps.append([(t, int(a)) for t, a in zip(ids, rw_np)])
        else:
            self._fetch(k, ids, ids_np, rw_np)
        return k

    def _end(self, m, k: int, kind: str):
        if not self._recording:
            _ids, ids_np, rw_np = self._step_lists[(id(m), kind)]
            stream = self.torch.cuda.current_stream().cuda_stream
            self.tc.migrate_step(k, T.POST, ids_np, rw_np, stream)

    def _fetch(self, k: int, ids, ids_np, rw_np):
        stream = self.torch.cuda.current_stream().cuda_stream
        ptrs = self.tc.migrate_step(k, T.PRE, ids_np, rw_np, stream, want_ptrs=True)
        for t, ptr in zip(ids, ptrs):
            if not ptr:
                raise RuntimeError(f"tensor {t} could not be given a GPU buffer (cache too small for this module)")
            # a tensor comes back to the same few buffers iteration after iteration: keep the views
            view = self._views.get((t, ptr))
            if view is None:
                off, n = ptr - self._hbm_base, self._nbytes[t]
                view = self._views[(t, ptr)] = self.tc.hbm[off: off + n].view(self._dtype[t]).view(self._shape[t])
            if t < len(self.params):
                self.params[t].data = view
            elif t < self._state_base:
                self._grad_view[t - len(self.params)] = view
            else:
                self._state_view[t] = view

    def _pack_saved(self, x):
        """A tensor the running forward saves for the backward pass: if it aliases one of
        the module's parameters, keep a reference to the parameter instead of the buffer."""
        if not x.is_cuda:
            return x
        ptr = x.data_ptr()
        for t in self._saving_for:
            d = self.params[t].data
            base = d.data_ptr()
            if base <= ptr < base + self._nbytes[t] and x.dtype == d.dtype:
                return _ParamRef(t, tuple(x.shape), tuple(x.stride()), (ptr - base) // x.element_size())
        return x

    def _unpack_saved(self, r):
        if isinstance(r, _ParamRef):
            d = self.params[r.t].data                     # the buffer the backward pre-hook fetched it into
            return self.torch.as_strided(d, r.shape, r.stride, d.storage_offset() + r.offset)
        return r

    def _fwd_pre(self, m, args):
        if self._recording:
            self._ran[id(m)] = True
        self._uses[id(m)] = self._uses.get(id(m), 0) + 1
        if self._uses[id(m)] > 1 and id(m) not in self._by_input:
            if not self._recording:
                raise RuntimeError("a module ran twice in a pass but only once in the profiled iteration")
            self._by_input.add(id(m))                     # (its first use's backward comes later: it will see this)
            self._check_by_input()
        self._fwd_step[id(m)] = self._begin(m, "fwd")
        new_args = None
        if id(m) in self._by_input and self.torch.is_grad_enabled():
            # this use's own view of every input that needs a gradient: the gradient of the view is this
            # module's contribution alone, and its arrival closes the use's backward step
            u = self._next_use
            self._next_use += 1
            self._open_use[id(m)] = u
            views = []
            for a in args:
                if self.torch.is_tensor(a) and a.requires_grad:
                    a = a.view_as(a)
                    a.register_hook(self._make_input_grad(m, u))
                    self._use_inputs[u] = self._use_inputs.get(u, 0) + 1
                views.append(a)
            self._use_inputs.setdefault(u, 0)
            new_args = tuple(views)
        if not self._recording and self.torch.is_grad_enabled():
            ctx = self.torch.autograd.graph.saved_tensors_hooks(self._pack_saved, self._unpack_saved)
            ctx.__enter__()
            self._saved_ctx[id(m)] = ctx
            self._saving_for = tuple(self.mod_ids[id(m)])
        return new_args

    def _fwd_post(self, m, args, out):
        ctx = self._saved_ctx.pop(id(m), None)
        if ctx is not None:
            ctx.__exit__(None, None, None)
            self._saving_for = ()
        self._end(m, self._fwd_step.pop(id(m)), "fwd")
        # the module's backward starts when the gradient of its output arrives
        outs = out if isinstance(out, (tuple, list)) else (out,)
        u = self._open_use.pop(id(m), None)
        for o in outs:
            if self.torch.is_tensor(o) and o.requires_grad:
                o.register_hook(self._make_bwd_start(m) if u is None else self._make_use_bwd_start(m, u))
                break

    def _make_use_bwd_start(self, m, u):
        def hook(grad):
            if u in self._use_step or u not in self._use_inputs:
                return grad
            if self._use_inputs[u] == 0:                  # no input to wait for: the parameters' gradients close it
                del self._use_inputs[u]
                if id(m) not in self._bwd_step:
                    self._bwd_step[id(m)] = self._begin(m, "bwd")
                    self._pending_bwd[id(m)] = len(self.mod_ids[id(m)])
                return grad
            self._use_step[u] = self._begin(m, "bwd")
            return grad
        return hook

    def _make_input_grad(self, m, u):
        def hook(grad):
            if u in self._use_step:
                self._use_inputs[u] -= 1
                if self._use_inputs[u] == 0:
                    del self._use_inputs[u]
                    self._end(m, self._use_step.pop(u), "bwd")
            return grad
        return hook

    def _make_bwd_start(self, m):
        def hook(grad):
            if id(m) not in self._bwd_step:               # several outputs: the first gradient opens the step
                self._bwd_step[id(m)] = self._begin(m, "bwd")
                self._pending_bwd[id(m)] = len(self.mod_ids[id(m)])
            return grad
        return hook

    def _make_grad_done(self, m, t):
        def hook(param):
            if id(m) not in self._bwd_step:
                return
            if self.manage_grads and not self._recording:
                # the gradient goes into its cache buffer; the tensor autograd made is dropped
                self._grad_view.pop(t).copy_(param.grad)
                param.grad = None
            self._pending_bwd[id(m)] -= 1
            if self._pending_bwd[id(m)] == 0:
                if self.fused_sgd_lr is not None and not self._recording:
                    with self.torch.no_grad():            # the parameters are still in their cache buffers
                        for p in m.parameters(recurse=False):
                            p.data.add_(p.grad, alpha=-self.fused_sgd_lr)
                self._end(m, self._bwd_step.pop(id(m)), "bwd")
        return hook

    # ---------------------------------------------------------------- profile
    def profile(self, run_iteration: Callable[[], None]):
        """Dry run (Sec. 3.2.1): one forward + backward under recording hooks.  Parameters are not
        updated, gradients are dropped, the model's buffers and the random number generators are put
        back as they were: training after it starts from the state before it."""
        self.steps = []
        self._k = 0
        self._uses, self._next_use, self._open_use, self._use_inputs, self._use_step = {}, 0, {}, {}, {}
        self._recording = True
        self._ran: Dict[int, bool] = {}
        self._register()
        # the dry run leaves nothing behind: what its forward changes besides gradients (running statistics
        # of normalisation layers, the random number generators a dropout draws from) is put back
        torch = self.torch
        buffers = [(b, b.detach().clone()) for b in self.model.buffers()]
        rng_cpu = torch.get_rng_state()
        rng_gpu = torch.cuda.get_rng_state_all() if torch.cuda.is_available() else None
        try:
            run_iteration()
        finally:
            self._remove()
            self._recording = False
            with torch.no_grad():
                for b, saved in buffers:
                    b.copy_(saved)
            torch.set_rng_state(rng_cpu)
            if rng_gpu is not None:
                torch.cuda.set_rng_state_all(rng_gpu)
        if self._bwd_step or self._use_step:
            raise RuntimeError("a module's backward did not finish during the dry run")
        ran = {id(m) for m in self.mods if self._ran.get(id(m))}
        # (a module that never runs but shares every parameter with modules that do, like a container's
        # handle on a tied embedding, needs no step of its own)
        covered = {id(p) for m in self.mods if id(m) in ran for p in m.parameters(recurse=False)}
        idle = [type(m).__name__ for m in self.mods
                if id(m) not in ran and any(id(p) not in covered for p in m.parameters(recurse=False))]
        if idle:
            raise ValueError("modules whose forward never ran in the dry run own parameters: " + ", ".join(sorted(set(idle))) +
                             " (if their parameters are used by another module's forward, name them in resident_modules)")
        self._uses, self._next_use, self._use_inputs = {}, 0, {}
        self._n_model_steps = len(self.steps)
        # the optimizer sweep: every parameter once, read and written
        if self.fused_sgd_lr is None:
            n_p = len(self.params)
            base = n_p * (2 if self.manage_grads else 1)
            for t in range(n_p):
                step = [(n_p + t, R), (t, RW)] if self.manage_grads else [(t, RW)]
                self.steps.append(step + [(base + j * n_p + t, RW) for j in range(self.state_tensors)])
        for p in self.params + self.resident:             # what the dry run left behind is no gradient of a step
            p.grad = None

    # ---------------------------------------------------------------- install
    def install(self):
        torch = self.torch
        rep = 2 if self.manage_grads else 1                # gradients: the same sizes once more, ids behind the parameters
        self._nbytes = [p.numel() * p.element_size() for p in self.params] * rep
        self._dtype = [p.dtype for p in self.params] * rep
        self._shape = [tuple(p.shape) for p in self.params] * rep
        self._state_base = len(self._nbytes)              # optimizer states: fp32, ids behind those
        for _ in range(self.state_tensors):
            self._nbytes += [p.numel() * 4 for p in self.params]
            self._dtype += [torch.float32] * len(self.params)
            self._shape += [tuple(p.shape) for p in self.params]
        n_p = len(self.params)
        self._sweep = []                                  # per parameter: the ids and flags of its sweep step
        for t in range(n_p):
            ids = ([n_p + t] if self.manage_grads else []) + [t] + \
                  [self._state_base + j * n_p + t for j in range(self.state_tensors)]
            flags = ([R] if self.manage_grads else []) + [RW] * (1 + self.state_tensors)
            self._sweep.append((tuple(ids), np.asarray(ids, dtype=np.uint32), np.asarray(flags, dtype=np.uint8)))
        self._state_view: Dict[int, object] = {}          # state tensor id -> its cache buffer, during a step that names it
        if min(self._nbytes) < 16:
            raise ValueError("parameters smaller than 16 bytes are not supported")
        st, te, rw = [], [], []
        for k, step in enumerate(self.steps):
            for (t, a) in step:
                st.append(k)
                te.append(t)
                rw.append(a)
        tc = T.TensorCache()
        tc.profile_order(self._nbytes, [0] * len(self._nbytes), st, te, rw)
        host = self.host_bytes if self.host_bytes is not None else sum((n + 255) // 256 * 256 for n in self._nbytes) + 4096
        tc.plan_pools(self.hbm_bytes, (host, 0), self.align)
        tc.plan_schedule()
        if self.file_path is not None:
            largest = (max(self._nbytes) + 4095) // 4096 * 4096
            tc.bind_torch(file_path=self.file_path, staging_bytes=8 * largest, stripes=self.stripes)
        else:
            tc.bind_torch()
        tc.tune_mover()                                   # the regions are still empty: measure the workgroup count
        if self.dma_threshold:
            tc.set_dma_threshold(int(self.dma_threshold))
            tc.set_dma_policy(True)                       # only while there is compute to hide the copies behind
        for t, p in enumerate(self.params):
            tc.load_tensor(t, p.detach().cpu().contiguous().view(torch.uint8).numpy().reshape(-1))
            p.data = torch.empty(0, dtype=self._dtype[t], device=p.device)
        for t in range(len(self.params), len(self._nbytes)):
            tc.load_tensor(t, np.zeros(self._nbytes[t], dtype=np.uint8))
        tc.set_oplog(self.keep_oplog, True)               # a training run of a million steps must not keep every decision
        self.tc = tc
        self._hbm_base = tc.hbm.data_ptr()
        self._views = {}
        self._k = 0
        self._register()

    # ------------------------------------------------------------- iteration
    def update_sweep(self, update: Callable[[int, object], None]):
        """The optimizer sweep through the cache: each parameter in turn is fetched (read +
        write), `update(t, p)` changes `p.data` in its cache buffer (p.grad holds the
        gradient), and the parameter is left to the scheduler.  With state_tensors the call is
        `update(t, p, states)`, states being the parameter's fp32 state tensors in their cache buffers."""
        torch = self.torch
        if self.fused_sgd_lr is not None:
            raise RuntimeError("the update is applied in the backward hooks (fused_sgd_lr): there is no sweep")
        stream = torch.cuda.current_stream().cuda_stream
        k = self._n_model_steps
        n_p = len(self.params)
        with torch.no_grad():
            for t, p in enumerate(self.params):
                ids, ids_np, rw = self._sweep[t]
                self._fetch(k, ids, ids_np, rw)
                states = [self._state_view.pop(self._state_base + j * n_p + t) for j in range(self.state_tensors)]
                if self.manage_grads:
                    p.grad = self._grad_view.pop(t)        # the gradient, in its cache buffer, for this step only
                if p.grad is not None:
                    if self.state_tensors:
                        update(t, p, states)
                    else:
                        update(t, p)
                if self.manage_grads:
                    p.grad = None
                self.tc.migrate_step(k, T.POST, ids_np, rw, stream)
                k += 1

    def autotune_dma(self, step: Callable[[], None], threshold: int = 64 << 10, steps: int = 2) -> Optional[int]:
        """Which path suits this training loop: `step()` (one whole training step, end_iteration
        included) is timed `steps` times after a first one with every large parameter through the
        zero-copy kernel, then with those of at least `threshold` bytes as DMA copies while the
        compute stream has a backlog; the faster setting stays.  The steps are ordinary training
        steps.  Returns the threshold kept (None: the kernel alone)."""
        torch = self.torch
        best = None
        for thr in (0, int(threshold)):
            self.tc.set_dma_threshold(thr)
            self.tc.set_dma_policy(True)
            step()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                step()
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            if best is None or dt < best[0]:
                best = (dt, thr)
        self.tc.set_dma_threshold(best[1])
        self.dma_threshold = best[1] or None
        return self.dma_threshold

    def sgd_step(self, lr: float):
        """Plain SGD: the managed parameters through the cache, the resident ones where they are."""
        self.update_sweep(lambda t, p, *_: p.data.add_(p.grad, alpha=-lr))
        with self.torch.no_grad():
            for p in self.resident:
                if p.grad is not None:
                    p.add_(p.grad, alpha=-lr)

    @staticmethod
    def adam_update(p, grad, m, v, step: int, lr: float, beta1: float, beta2: float, eps: float):
        """One Adam update of p (any float dtype) from grad, over fp32 moments m and v, in place."""
        g = grad.float()
        m.mul_(beta1).add_(g, alpha=1.0 - beta1)
        v.mul_(beta2).addcmul_(g, g, value=1.0 - beta2)
        denom = (v / (1.0 - beta2 ** step)).sqrt_().add_(eps)
        p.add_((m / (1.0 - beta1 ** step)).div_(denom).mul_(-lr).to(p.dtype))

    def adam_step(self, lr: float, betas=(0.9, 0.999), eps: float = 1e-8):
        """Adam with its two moments as tensors of the cache (needs state_tensors >= 2); the resident
        parameters keep theirs as ordinary tensors."""
        if self.state_tensors < 2:
            raise RuntimeError("adam_step needs ParamCache(state_tensors=2)")
        self._adam_step = getattr(self, "_adam_step", 0) + 1
        k = self._adam_step
        self.update_sweep(lambda t, p, st: self.adam_update(p.data, p.grad, st[0], st[1], k, lr, betas[0], betas[1], eps))
        with self.torch.no_grad():
            if not hasattr(self, "_resident_moments"):
                self._resident_moments = [(self.torch.zeros_like(p, dtype=self.torch.float32),
                                           self.torch.zeros_like(p, dtype=self.torch.float32)) for p in self.resident]
            for p, (m, v) in zip(self.resident, self._resident_moments):
                if p.grad is not None:
                    self.adam_update(p, p.grad, m, v, k, lr, betas[0], betas[1], eps)

    def end_iteration(self):
        self.tc.end_iteration(self.torch.cuda.current_stream().cuda_stream)
        self._k = 0
        self._uses, self._next_use, self._open_use, self._use_inputs, self._use_step = {}, 0, {}, {}, {}
        if self.fused_sgd_lr is not None:                 # the resident parameters have no hook to be updated in
            with self.torch.no_grad():
                for p in self.resident:
                    if p.grad is not None:
                        p.add_(p.grad, alpha=-self.fused_sgd_lr)
        for p in self.params:
            p.grad = None
        for p in self.resident:
            p.grad = None

    def gather(self) -> list:
        """Current value of every parameter of the model, in the order of `model.parameters()`, wherever
        it lives (CPU tensors)."""
        torch = self.torch
        return [torch.from_numpy(self.tc.read_tensor(t)).view(self._dtype[t]).view(self._shape[t])
                if isinstance(t, int) else t.detach().cpu() for t in self._order]

    def state_dict(self) -> dict:
        """`model.state_dict()` with the managed parameters' current values in place of the empty tensors
        the module holds outside its steps (every name of a shared parameter included); CPU tensors for
        the parameters, the model's own tensors for its buffers."""
        value = {id(p): v for p, v in zip(self.model.parameters(), self.gather())}
        sd = self.model.state_dict()
        for name, p in self.model.named_parameters(remove_duplicate=False):
            if name in sd:
                sd[name] = value[id(p)]
        return sd

    def gather_grads(self) -> list:
        """With managed gradients: every gradient as the cache holds it now (CPU tensors)."""
        torch, n_p = self.torch, len(self.params)
        if not self.manage_grads:
            raise RuntimeError("gradients are not tensors of this cache")
        return [torch.from_numpy(self.tc.read_tensor(n_p + t)).view(self._dtype[t]).view(self._shape[t])
                for t in range(n_p)]

    def gather_states(self) -> list:
        """Every optimizer-state tensor as the cache holds it now: one list per state, in the order of
        the managed parameters (CPU tensors)."""
        torch, n_p = self.torch, len(self.params)
        return [[torch.from_numpy(self.tc.read_tensor(self._state_base + j * n_p + t)).view(torch.float32).view(self._shape[t])
                 for t in range(n_p)] for j in range(self.state_tensors)]

    def close(self, restore: bool = False):
        """Hooks off, the cache's memory released.  restore: first give every managed parameter its
        current value back as an ordinary tensor on its device, so that the model works without the
        cache again (otherwise its managed parameters stay the empty tensors they are outside a step)."""
        self._remove()
        if restore and self.tc is not None:
            for t, p in enumerate(self.params):
                value = self.torch.from_numpy(self.tc.read_tensor(t)).view(self._dtype[t]).view(self._shape[t])
                p.data = value.to(p.device)
                p.grad = None
        self._views = {}
        if self.tc is not None:
            self.tc.close()
            self.tc = None
