"""Live profiling and hook-driven migration on a real PyTorch model: a small
MLP whose parameters live in the tensor cache (an HBM budget of about a third
of their bytes) must train exactly like the same model with its parameters
resident, step for step."""

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2511_14124_amd as T                          # noqa: E402
from paper_2511_14124_amd.torch_hooks import ParamCache   # noqa: E402
from oracle import tc_oracle as o                         # noqa: E402


def _model(seed):
    torch.manual_seed(seed)
    layers = [torch.nn.Linear(64, 128)]
    for _ in range(5):
        layers += [torch.nn.LayerNorm(128), torch.nn.ReLU(), torch.nn.Linear(128, 128)]
    layers += [torch.nn.ReLU(), torch.nn.Linear(128, 10)]
    return torch.nn.Sequential(*layers).to("cuda:0")


@pytest.mark.parametrize("mode", ["sweep", "fused", "grads"])
def test_training_through_the_cache_equals_resident_training(mode):
    # sweep: parameters through the cache, plain SGD as a third pass; fused: the update in the backward hooks;
    # grads: the gradients are tensors of the cache as well (written in the backward step, read in the sweep)
    fused, grads = mode == "fused", mode == "grads"
    lr, iters = 0.05, 4
    torch.manual_seed(0)
    xs = [torch.randn(32, 64, device="cuda:0") for _ in range(iters + 1)]
    ys = [torch.randint(0, 10, (32,), device="cuda:0") for _ in range(iters + 1)]
    loss_fn = torch.nn.CrossEntropyLoss()

    ref = _model(7)
    ref_losses = []
    for i in range(iters):
        for p in ref.parameters():
            p.grad = None
        loss = loss_fn(ref(xs[i]), ys[i])
        loss.backward()
        ref_losses.append(float(loss.detach()))
        with torch.no_grad():
            for p in ref.parameters():
                p.add_(p.grad, alpha=-lr)

    model = _model(7)
    total = sum(p.numel() * p.element_size() for p in model.parameters())
    budget = int(total * (0.8 if grads else 0.4))          # 40 % of the bytes the cache manages
    pc = ParamCache(model, hbm_bytes=budget, fused_sgd_lr=lr if fused else None, manage_grads=grads, keep_oplog=True)
    pc.profile(lambda: loss_fn(model(xs[-1]), ys[-1]).backward())
    n_mod = len(pc.mods)
    assert len(pc.steps) == 2 * n_mod + (0 if fused else len(pc.params))   # forward, backward, one sweep
    # backward order recorded by the hooks is the reverse of the forward order
    n_p = len(pc.params)
    fwd = [tuple(t for t, _ in s) for s in pc.steps[:n_mod]]
    bwd = [tuple(t for t, _ in s if t < n_p) for s in pc.steps[n_mod:2 * n_mod]]
    assert bwd == fwd[::-1]
    if grads:
        # a backward step names the parameters (read) and behind them their gradients (written);
        # a sweep step the gradient (read) and the parameter (read and written)
        for s_f, s_b in zip(pc.steps[:n_mod][::-1], pc.steps[n_mod:2 * n_mod]):
            assert s_b == [(t, 1) for t, _ in s_f] + [(n_p + t, 2) for t, _ in s_f]
        assert pc.steps[2 * n_mod:] == [[(n_p + t, 1), (t, 3)] for t in range(n_p)]
    pc.install()
    losses = []
    for i in range(iters):
        loss = loss_fn(model(xs[i]), ys[i])
        loss.backward()
        losses.append(float(loss.detach()))
        if grads:
            assert all(p.grad is None for p in model.parameters())   # they live in the cache, not beside it
        if not fused:
            pc.sgd_step(lr)
        pc.end_iteration()
    got = pc.gather()
    got_grads = pc.gather_grads() if grads else None
    st = pc.tc.cache_stats()
    log = pc.tc.dump_oplog()
    pc.close()

    assert losses == ref_losses
    for a, b in zip(got, [p.detach().cpu() for p in ref.parameters()]):
        assert torch.equal(a, b)
    # the cache really was smaller than the model: tensors moved, and the schedule is the oracle's
    assert st["n_ops"][1] > 0 and st["n_ops"][2] > 0 and st["misses"] == 0
    if grads:                                                # the last iteration's gradients, wherever they ended up
        for a, b in zip(got_grads, [p.grad.detach().cpu() for p in ref.parameters()]):
            assert torch.equal(a, b)
    nbytes = [p.numel() * p.element_size() for p in ref.parameters()] * (2 if grads else 1)
    stp, te, rw = [], [], []
    for k, step in enumerate(pc.steps):
        for (t, a) in step:
            stp.append(k), te.append(t), rw.append(a)
    host = sum((n + 255) // 256 * 256 for n in nbytes) + 4096
    r = o.build(nbytes, [0] * len(nbytes), stp, te, rw, budget, (host, 0))
    for _ in range(iters):
        r.run_iteration(pc.steps)
    assert len(log) == len(r.log)
    assert [(int(x["step"]), int(x["op"]), int(x["tensor"]), int(x["dst_slot"])) for x in log] == \
        [(e[1], e[3], e[4], e[8]) for e in r.log]
    assert (st["hits"], st["misses"]) == (r.hits, r.misses)


class _Tied(torch.nn.Module):
    """Token embedding tied to the output projection (one parameter, two modules), and one block
    that runs twice in a pass."""

    def __init__(self, vocab=96, d=64):
        super().__init__()
        self.emb = torch.nn.Embedding(vocab, d)
        self.inp = torch.nn.Linear(d, d)
        self.block = torch.nn.Sequential(torch.nn.LayerNorm(d), torch.nn.Linear(d, d), torch.nn.ReLU())
        self.mid = torch.nn.Linear(d, d)
        self.head = torch.nn.Linear(d, vocab, bias=False)
        self.head.weight = self.emb.weight

    def forward(self, tok):
        x = self.inp(self.emb(tok))
        x = x + self.block(x)
        x = self.mid(x)
        x = x + self.block(x)                             # the same modules a second time
        return self.head(x)


def test_tied_weights_and_a_block_used_twice_train_like_the_resident_model():
    lr, iters = 0.05, 4
    torch.manual_seed(1)
    toks = [torch.randint(0, 96, (8, 16), device="cuda:0") for _ in range(iters + 1)]
    tgts = [torch.randint(0, 96, (8 * 16,), device="cuda:0") for _ in range(iters + 1)]
    loss_fn = torch.nn.CrossEntropyLoss()

    def make():
        torch.manual_seed(3)
        return _Tied().to("cuda:0")

    ref = make()
    ref_losses = []
    for i in range(iters):
        for p in ref.parameters():
            p.grad = None
        loss = loss_fn(ref(toks[i]).view(-1, 96), tgts[i])
        loss.backward()
        ref_losses.append(float(loss.detach()))
        with torch.no_grad():
            for p in ref.parameters():
                p.add_(p.grad, alpha=-lr)

    model = make()
    assert model.head.weight is model.emb.weight
    total = sum(p.numel() * p.element_size() for p in model.parameters())
    pc = ParamCache(model, hbm_bytes=int(total * 0.75), keep_oplog=True)
    assert len(pc.params) == len(list(model.parameters()))          # the shared parameter is one tensor of the cache
    pc.profile(lambda: loss_fn(model(toks[-1]).view(-1, 96), tgts[-1]).backward())
    n_p = len(pc.params)
    fwd_bwd = pc.steps[:-n_p]
    # emb, inp, (ln, lin), mid, (ln, lin), head forward = 8 module uses, as many backward
    assert len(fwd_bwd) == 16
    shared = pc.pid[id(model.emb.weight)]
    assert [k for k, st in enumerate(fwd_bwd) if any(t == shared for t, _ in st)] == [0, 7, 8, 15]
    pc.install()
    losses = []
    for i in range(iters):
        loss = loss_fn(model(toks[i]).view(-1, 96), tgts[i])
        loss.backward()
        losses.append(float(loss.detach()))
        pc.sgd_step(lr)
        pc.end_iteration()
    got = pc.gather()
    st = pc.tc.cache_stats()
    log = pc.tc.dump_oplog()
    pc.close()
    assert losses == ref_losses
    for a, b in zip(got, [p.detach().cpu() for p in ref.parameters()]):
        assert torch.equal(a, b)
    assert st["n_ops"][1] > 0 and st["misses"] == 0
    nbytes = [p.numel() * p.element_size() for p in ref.parameters()]
    stp, te, rw = [], [], []
    for k, step in enumerate(pc.steps):
        for (t, a) in step:
            stp.append(k), te.append(t), rw.append(a)
    host = sum((n + 255) // 256 * 256 for n in nbytes) + 4096
    r = o.build(nbytes, [0] * len(nbytes), stp, te, rw, int(total * 0.75), (host, 0))
    for _ in range(iters):
        r.run_iteration(pc.steps)
    assert [(int(x["step"]), int(x["op"]), int(x["tensor"]), int(x["dst_slot"])) for x in log] == \
        [(e[1], e[3], e[4], e[8]) for e in r.log]
    # the update in the hooks and managed gradients need every gradient complete at the module's own step
    for kw in (dict(fused_sgd_lr=0.1), dict(manage_grads=True)):
        with pytest.raises(ValueError):
            ParamCache(make(), hbm_bytes=int(total * 0.75), **kw)


class _Rooted(torch.nn.Module):
    """A root module with parameters of its own (a position table, a scale) that calls modules with
    parameters, and optionally nn.MultiheadAttention, which uses its output projection's parameters
    without calling that module."""

    def __init__(self, mha):
        super().__init__()
        self.pos = torch.nn.Parameter(torch.randn(16, 64) * 0.02)
        self.scale = torch.nn.Parameter(torch.ones(64))
        self.emb = torch.nn.Embedding(96, 64)
        self.blocks = torch.nn.ModuleList([torch.nn.Sequential(torch.nn.LayerNorm(64), torch.nn.Linear(64, 64),
                                                               torch.nn.GELU()) for _ in range(4)])
        self.mha = torch.nn.MultiheadAttention(64, 4, batch_first=True) if mha else None
        self.out = torch.nn.Linear(64, 96)

    def forward(self, x):
        h = self.emb(x) + self.pos
        for b in self.blocks:
            h = h + b(h)
        if self.mha is not None:
            h = h + self.mha(h, h, h, need_weights=False)[0]
        return self.out(h * self.scale)


@pytest.mark.parametrize("mha", [False, True])
@pytest.mark.parametrize("mode", ["sweep", "fused", "grads"])
def test_parameters_of_a_module_that_calls_managed_modules_stay_resident(mha, mode):
    # the root's own parameters are in use across its children's steps, where nothing would keep them in
    # their buffers: they stay ordinary tensors (managed naively the model trained to other bytes, without
    # an error); a module whose parameters are used without its forward being called is refused by the dry
    # run until the caller names it
    lr = 0.05
    x = torch.randint(0, 96, (4, 16), device="cuda:0", generator=torch.Generator(device="cuda:0").manual_seed(1))
    y = torch.randint(0, 96, (64,), device="cuda:0", generator=torch.Generator(device="cuda:0").manual_seed(2))
    loss_fn = torch.nn.CrossEntropyLoss()

    def iteration(m):
        loss_fn(m(x).view(-1, 96), y).backward()

    def make():
        torch.manual_seed(3)
        return _Rooted(mha).to("cuda:0")

    kw = {"fused": dict(fused_sgd_lr=lr), "grads": dict(manage_grads=True), "sweep": {}}[mode]
    ref, model = make(), make()
    total = sum(p.numel() * p.element_size() for p in model.parameters())
    budget = int(total * (1.2 if mode == "grads" else 0.6))
    pc = ParamCache(model, hbm_bytes=budget, **kw)
    if mha:
        with pytest.raises(ValueError, match="resident_modules"):
            pc.profile(lambda: iteration(model))
        pc.close()
        pc = ParamCache(model, hbm_bytes=budget, resident_modules=[model.mha], **kw)
    pc.profile(lambda: iteration(model))
    assert [id(p) for p in pc.resident[:2]] == [id(model.pos), id(model.scale)]
    assert len(pc.resident) == (6 if mha else 2) and len(pc.params) + len(pc.resident) == len(list(model.parameters()))
    pc.install()
    for _ in range(3):
        for p in ref.parameters():
            p.grad = None
        iteration(ref)
        with torch.no_grad():
            for p in ref.parameters():
                p.add_(p.grad, alpha=-lr)
        iteration(model)
        if mode != "fused":
            pc.sgd_step(lr)
        pc.end_iteration()
    got = pc.gather()
    st = pc.tc.cache_stats()
    pc.close()
    assert len(got) == len(list(ref.parameters()))
    for a, b in zip(got, ref.parameters()):
        assert torch.equal(a, b.detach().cpu())
    assert st["misses"] == 0 and st["n_ops"][1] > 0


def test_gradients_accumulated_over_two_micro_batches_train_like_the_resident_model():
    # two forward + backward passes before the update: every module runs twice in the iteration, which the
    # hooks treat like a module used twice in a pass; with the update in the hooks or managed gradients
    # (a gradient complete only after the last pass) the dry run refuses instead of training to other bytes
    from paper_2511_14124_amd.train_demo import build_model
    vocab, lr = 256, 0.05
    xs = [torch.randint(0, vocab, (2, 32), device="cuda:0", generator=torch.Generator(device="cuda:0").manual_seed(s))
          for s in (1, 2)]
    loss_fn = torch.nn.CrossEntropyLoss()

    def iteration(m):
        for x in xs:
            loss_fn(m(x).float().view(-1, vocab), x.view(-1)).backward()

    def make():
        torch.manual_seed(3)
        return build_model(torch, 64, 3, 4, vocab, torch.float32)

    ref, model = make(), make()
    total = sum(p.numel() * p.element_size() for p in model.parameters())
    pc = ParamCache(model, hbm_bytes=int(total * 0.5))
    pc.profile(lambda: iteration(model))
    pc.install()
    for _ in range(3):
        for p in ref.parameters():
            p.grad = None
        iteration(ref)
        with torch.no_grad():
            for p in ref.parameters():
                p.add_(p.grad, alpha=-lr)
        iteration(model)
        pc.sgd_step(lr)
        pc.end_iteration()
    got = pc.gather()
    pc.close()
    for a, b in zip(got, ref.parameters()):
        assert torch.equal(a, b.detach().cpu())
    for kw in (dict(manage_grads=True), dict(fused_sgd_lr=lr)):
        other = make()
        pc = ParamCache(other, hbm_bytes=int(total * 1.0), **kw)
        with pytest.raises(ValueError, match="separate update sweep"):
            pc.profile(lambda: iteration(other))
        pc.close()


class _Plain(torch.nn.Module):
    def __init__(self, ckpt=False, unused=False):
        super().__init__()
        self.emb = torch.nn.Embedding(96, 64)
        self.blocks = torch.nn.ModuleList([torch.nn.Sequential(torch.nn.LayerNorm(64), torch.nn.Linear(64, 64),
                                                               torch.nn.GELU()) for _ in range(4)])
        self.side = torch.nn.Linear(64, 64) if unused else None
        self.out = torch.nn.Linear(64, 96)
        self.ckpt, self.skip = ckpt, False

    def forward(self, x):
        from torch.utils.checkpoint import checkpoint
        h = self.emb(x)
        for i, b in enumerate(self.blocks):
            if self.skip and i == 2:
                continue
            h = h + (checkpoint(b, h, use_reentrant=False) if self.ckpt else b(h))
        if self.side is not None:
            self.side(h.detach())                          # computed, not part of the loss
        return self.out(h)


@pytest.mark.parametrize("case", ["eval_between", "block_skipped", "module_outside_the_loss", "activation_checkpointing"])
def test_passes_that_are_not_the_profiled_one_still_train_like_the_resident_model(case):
    # a forward-only pass between training iterations, an iteration that skips a block (demand misses),
    # a module whose output the loss does not use, blocks recomputed in the backward pass
    lr = 0.05
    x = torch.randint(0, 96, (4, 16), device="cuda:0", generator=torch.Generator(device="cuda:0").manual_seed(1))
    y = torch.randint(0, 96, (64,), device="cuda:0", generator=torch.Generator(device="cuda:0").manual_seed(2))
    loss_fn = torch.nn.CrossEntropyLoss()

    def iteration(m):
        loss_fn(m(x).view(-1, 96), y).backward()

    def make():
        torch.manual_seed(3)
        return _Plain(ckpt=case == "activation_checkpointing", unused=case == "module_outside_the_loss").to("cuda:0")

    script = {"eval_between": ["train", "eval", "train", "eval", "train"],
              "block_skipped": ["train", "skip", "train"]}.get(case, ["train"] * 3)
    ref, model = make(), make()
    total = sum(p.numel() * p.element_size() for p in model.parameters())
    pc = ParamCache(model, hbm_bytes=int(total * 0.5))
    pc.profile(lambda: iteration(model))
    pc.install()
    for what in script:
        if what == "eval":
            with torch.no_grad():
                want, got = ref(x), model(x)
            pc.end_iteration()
            assert torch.equal(want, got)
            continue
        ref.skip = model.skip = what == "skip"
        for p in ref.parameters():
            p.grad = None
        iteration(ref)
        with torch.no_grad():
            for p in ref.parameters():
                if p.grad is not None:
                    p.add_(p.grad, alpha=-lr)
        iteration(model)
        pc.sgd_step(lr)
        pc.end_iteration()
    got = pc.gather()
    st = pc.tc.cache_stats()
    pc.close()
    for a, b in zip(got, ref.parameters()):
        assert torch.equal(a, b.detach().cpu())
    assert (st["misses"] > 0) == (case == "block_skipped")


@pytest.mark.parametrize("mode", ["sweep", "fused", "grads"])
@pytest.mark.parametrize("weights", ["fp32_under_autocast", "bf16_linears_fp32_norms"])
def test_mixed_precision_trains_like_the_resident_model(mode, weights):
    # autocast makes 16-bit copies of fp32 weights inside the forward (nothing autograd saves aliases the
    # parameter then); with 16-bit Linear layers beside fp32 norms the cache has size classes of both widths
    from paper_2511_14124_amd.train_demo import build_model
    vocab, lr = 256, 0.05
    x = torch.randint(0, vocab, (2, 32), device="cuda:0", generator=torch.Generator(device="cuda:0").manual_seed(1))
    loss_fn = torch.nn.CrossEntropyLoss()

    def iteration(m):
        with torch.autocast("cuda", dtype=torch.bfloat16):
            out = m(x)
        loss_fn(out.float().view(-1, vocab), x.view(-1)).backward()

    def make():
        torch.manual_seed(3)
        m = build_model(torch, 64, 3, 4, vocab, torch.float32)
        if weights == "bf16_linears_fp32_norms":
            for mod in m.modules():
                if isinstance(mod, torch.nn.Linear):
                    mod.to(torch.bfloat16)
        return m

    kw = {"fused": dict(fused_sgd_lr=lr), "grads": dict(manage_grads=True), "sweep": {}}[mode]
    ref, model = make(), make()
    total = sum(p.numel() * p.element_size() for p in model.parameters())
    pc = ParamCache(model, hbm_bytes=int(total * (1.0 if mode == "grads" else 0.5)), **kw)
    pc.profile(lambda: iteration(model))
    pc.install()
    for _ in range(3):
        for p in ref.parameters():
            p.grad = None
        iteration(ref)
        with torch.no_grad():
            for p in ref.parameters():
                p.add_(p.grad, alpha=-lr)
        iteration(model)
        if mode != "fused":
            pc.sgd_step(lr)
        pc.end_iteration()
    got = pc.gather()
    st = pc.tc.cache_stats()
    pc.close()
    for a, b in zip(got, ref.parameters()):
        assert a.dtype == b.dtype and torch.equal(a.view(torch.uint8), b.detach().cpu().view(torch.uint8))
    assert st["misses"] == 0 and st["n_ops"][1] > 0


class _Stateful(torch.nn.Module):
    """Modules whose forward changes more than activations: batch-norm statistics (buffers), dropout
    (the random number generator); and a recurrent layer, which owns eight parameters in one step."""

    def __init__(self, kind):
        super().__init__()
        self.emb = torch.nn.Embedding(96, 64)
        self.rnn = {"lstm": torch.nn.LSTM, "gru": torch.nn.GRU}[kind](64, 64, num_layers=2, batch_first=True)
        self.drop = torch.nn.Dropout(0.1)
        self.conv = torch.nn.Conv1d(64, 64, 3, padding=1)
        self.bn = torch.nn.BatchNorm1d(64)
        self.out = torch.nn.Linear(64, 96)

    def forward(self, x):
        h, _ = self.rnn(self.emb(x))
        h = self.bn(self.conv(self.drop(h).transpose(1, 2))).transpose(1, 2)
        return self.out(h)


@pytest.mark.parametrize("kind", ["lstm", "gru"])
def test_the_dry_run_leaves_buffers_and_random_number_generators_as_they_were(kind):
    # the resident model trains first, from a seeded generator; then the generator is seeded again, the
    # other model is profiled (a whole forward and backward: batch-norm statistics move, dropout draws)
    # and trained through the cache: same parameters, same running statistics, same dropout masks
    lr = 0.05
    x = torch.randint(0, 96, (4, 16), device="cuda:0", generator=torch.Generator(device="cuda:0").manual_seed(1))
    y = torch.randint(0, 96, (64,), device="cuda:0", generator=torch.Generator(device="cuda:0").manual_seed(2))
    loss_fn = torch.nn.CrossEntropyLoss()

    def iteration(m):
        loss_fn(m(x).reshape(-1, 96), y).backward()

    def make():
        torch.manual_seed(3)
        return _Stateful(kind).to("cuda:0")

    ref = make()
    torch.manual_seed(11)
    for _ in range(3):
        for p in ref.parameters():
            p.grad = None
        iteration(ref)
        with torch.no_grad():
            for p in ref.parameters():
                p.add_(p.grad, alpha=-lr)
    model = make()
    total = sum(p.numel() * p.element_size() for p in model.parameters())
    torch.manual_seed(11)
    pc = ParamCache(model, hbm_bytes=int(total * 0.95))
    pc.profile(lambda: iteration(model))
    pc.install()
    for _ in range(3):
        iteration(model)
        pc.sgd_step(lr)
        pc.end_iteration()
    got = pc.gather()
    pc.close()
    for a, b in zip(got, ref.parameters()):
        assert torch.equal(a, b.detach().cpu())
    for (name, a), (_, b) in zip(model.named_buffers(), ref.named_buffers()):
        assert torch.equal(a, b), name


@pytest.mark.parametrize("mode", ["sweep", "fused", "grads"])
def test_training_with_parameters_in_hbm_host_memory_and_a_file(mode, tmp_path):
    # the paper's CPU-GPU-NVMe set-up driven by the hooks: 30 % of the managed bytes in the HBM cache,
    # 30 % in pinned host memory, the rest in a file striped over three files
    from paper_2511_14124_amd.train_demo import build_model
    vocab, lr = 512, 0.05
    x = torch.randint(0, vocab, (2, 64), device="cuda:0", generator=torch.Generator(device="cuda:0").manual_seed(1))
    loss_fn = torch.nn.CrossEntropyLoss()

    def iteration(m):
        loss_fn(m(x).float().view(-1, vocab), x.view(-1)).backward()

    def make():
        torch.manual_seed(3)
        return build_model(torch, 128, 4, 4, vocab, torch.bfloat16)

    kw = {"fused": dict(fused_sgd_lr=lr), "grads": dict(manage_grads=True), "sweep": {}}[mode]
    ref, model = make(), make()
    managed = sum(p.numel() * p.element_size() for p in model.parameters()) * (2 if mode == "grads" else 1)
    pc = ParamCache(model, hbm_bytes=int(managed * 0.3), host_bytes=int(managed * 0.3),
                    file_path=str(tmp_path / "tier.bin"), stripes=3, **kw)
    pc.profile(lambda: iteration(model))
    pc.install()
    assert (pc.tc.placement["final_tier"] == T.NVME).sum() > 0
    for _ in range(3):
        for p in ref.parameters():
            p.grad = None
        iteration(ref)
        with torch.no_grad():
            for p in ref.parameters():
                p.add_(p.grad, alpha=-lr)
        iteration(model)
        if mode != "fused":
            pc.sgd_step(lr)
        pc.end_iteration()
    got = pc.gather()
    st = pc.tc.cache_stats()
    pc.close()
    for a, b in zip(got, ref.parameters()):
        assert torch.equal(a.view(torch.int16), b.detach().cpu().view(torch.int16))
    assert st["misses"] == 0 and st["bytes_file_read"] > 0 and st["bytes_file_write"] > 0


@pytest.mark.parametrize("grads", [False, True], ids=["parameters_and_moments", "parameters_gradients_and_moments"])
@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_adam_with_its_moments_in_the_cache_equals_resident_adam(dtype, grads):
    # parameter, gradient and optimizer tensors all through one HBM cache of 30 % of their bytes: the fp32
    # first and second moments are tensors of the cache, named by each parameter's step of the update
    # sweep; parameters and moments after three steps are those of Adam with everything resident (the
    # reference spells the update out op by op)
    from paper_2511_14124_amd.train_demo import build_model
    vocab, lr, b1, b2, eps = 512, 1e-3, 0.9, 0.999, 1e-8
    dt = {"bf16": torch.bfloat16, "fp32": torch.float32}[dtype]
    x = torch.randint(0, vocab, (2, 64), device="cuda:0", generator=torch.Generator(device="cuda:0").manual_seed(1))
    loss_fn = torch.nn.CrossEntropyLoss()

    def iteration(m):
        loss_fn(m(x).float().view(-1, vocab), x.view(-1)).backward()

    def make():
        torch.manual_seed(3)
        return build_model(torch, 128, 4, 4, vocab, dt)

    ref, model = make(), make()
    ms = [torch.zeros_like(p, dtype=torch.float32) for p in ref.parameters()]
    vs = [torch.zeros_like(p, dtype=torch.float32) for p in ref.parameters()]
    managed = sum(p.numel() * (p.element_size() * (2 if grads else 1) + 8) for p in model.parameters())
    pc = ParamCache(model, hbm_bytes=int(managed * 0.3), state_tensors=2, manage_grads=grads)
    pc.profile(lambda: iteration(model))
    n_p = len(pc.params)
    assert len(pc.steps[-1]) == (4 if grads else 3) and len(pc.steps) == pc._n_model_steps + n_p
    pc.install()
    for k in range(1, 4):
        for p in ref.parameters():
            p.grad = None
        iteration(ref)
        with torch.no_grad():
            for p, m, v in zip(ref.parameters(), ms, vs):
                g = p.grad.float()
                m.mul_(b1).add_(g, alpha=1.0 - b1)
                v.mul_(b2).addcmul_(g, g, value=1.0 - b2)
                denom = (v / (1.0 - b2 ** k)).sqrt_().add_(eps)
                p.add_((m / (1.0 - b1 ** k)).div_(denom).mul_(-lr).to(p.dtype))
        iteration(model)
        pc.adam_step(lr, (b1, b2), eps)
        pc.end_iteration()
    got, states, st = pc.gather(), pc.gather_states(), pc.tc.cache_stats()
    pc.close()
    for a, b in zip(got, ref.parameters()):
        assert torch.equal(a.view(torch.uint8), b.detach().cpu().view(torch.uint8))
    for have, want in ((states[0], ms), (states[1], vs)):
        for a, b in zip(have, want):
            assert torch.equal(a, b.cpu())
    assert st["misses"] == 0 and st["bytes_h2d"] > managed
    with pytest.raises(ValueError):
        ParamCache(make(), hbm_bytes=managed, state_tensors=2, fused_sgd_lr=lr)


@pytest.mark.parametrize("family", ["gpt2", "llama", "llama_tied", "bert", "t5", "mixtral", "vit"])
def test_models_defined_by_a_model_library_train_like_the_resident_models(family):
    # Not models written for this cache: the GPT-2, Llama, BERT and T5 classes of the transformers package at
    # a small size with random weights (nothing is downloaded).  GPT-2 ties its head to the token table,
    # Llama has grouped-query attention, a rotary module without parameters and RMS norms; three
    # steps through a cache of 35 % of the parameters leave the bytes of resident training.
    tf = pytest.importorskip("transformers")
    if family == "gpt2":
        cfg = tf.GPT2Config(vocab_size=512, n_positions=64, n_embd=128, n_layer=4, n_head=4, resid_pdrop=0.0,
                            embd_pdrop=0.0, attn_pdrop=0.0, bos_token_id=0, eos_token_id=0,
                            attn_implementation="eager")
        cls = tf.GPT2LMHeadModel
    elif family == "bert":                                 # an encoder; decoder weight tied to the token table, a bias of its own
        cfg = tf.BertConfig(vocab_size=512, hidden_size=128, num_hidden_layers=2, num_attention_heads=4,
                            intermediate_size=256, max_position_embeddings=64, hidden_dropout_prob=0.0,
                            attention_probs_dropout_prob=0.0, attn_implementation="eager")
        cls = tf.BertForMaskedLM
    elif family == "mixtral":                              # mixture of experts: which experts run depends on the tokens
        cfg = tf.MixtralConfig(vocab_size=512, hidden_size=64, intermediate_size=128, num_hidden_layers=2,
                               num_attention_heads=4, num_key_value_heads=2, num_local_experts=4, num_experts_per_tok=2,
                               max_position_embeddings=64, attn_implementation="eager", bos_token_id=0, eos_token_id=0)
        cls = tf.MixtralForCausalLM
    elif family == "vit":                                  # class token and position table belong to a module that calls the patch convolution
        cfg = tf.ViTConfig(hidden_size=64, num_hidden_layers=2, num_attention_heads=4, intermediate_size=128, image_size=32,
                           patch_size=8, num_labels=10, hidden_dropout_prob=0.0, attention_probs_dropout_prob=0.0,
                           attn_implementation="eager")
        cls = tf.ViTForImageClassification
    elif family == "t5":                                   # encoder and decoder with cross-attention; one table used by both and by the head
        cfg = tf.T5Config(vocab_size=512, d_model=128, d_kv=32, d_ff=256, num_layers=2, num_heads=4, dropout_rate=0.0,
                          decoder_start_token_id=0)
        cls = tf.T5ForConditionalGeneration
    else:
        cfg = tf.LlamaConfig(vocab_size=512, hidden_size=128, intermediate_size=256, num_hidden_layers=4,
                             num_attention_heads=4, num_key_value_heads=2, max_position_embeddings=64,
                             tie_word_embeddings=family == "llama_tied", attn_implementation="eager",
                             bos_token_id=0, eos_token_id=0)
        cls = tf.LlamaForCausalLM

    def make():
        torch.manual_seed(3)
        return cls(cfg).to(device="cuda:0", dtype=torch.bfloat16)

    x = torch.randint(1, 512, (2, 32), device="cuda:0", generator=torch.Generator(device="cuda:0").manual_seed(5))

    inputs = dict(input_ids=x, labels=x)
    if family == "vit":
        gen = torch.Generator(device="cuda:0").manual_seed(7)
        inputs = dict(pixel_values=torch.randn(2, 3, 32, 32, device="cuda:0", generator=gen).to(torch.bfloat16),
                      labels=torch.randint(0, 10, (2,), device="cuda:0", generator=gen))

    def iteration(m):
        m(**inputs).loss.backward()

    lr = 1e-2
    ref, model = make(), make()
    total = sum(p.numel() * p.element_size() for p in model.parameters())
    # (35 % of the parameter bytes, or 60 % where one module's fused experts alone are more than that)
    pc = ParamCache(model, hbm_bytes=int(total * (0.6 if family in ("mixtral", "vit") else 0.35)))
    pc.profile(lambda: iteration(model))
    pc.install()
    for _ in range(3):
        for p in ref.parameters():
            p.grad = None
        iteration(ref)
        with torch.no_grad():
            for p in ref.parameters():
                if p.grad is not None:
                    p.add_(p.grad, alpha=-lr)
        iteration(model)
        pc.sgd_step(lr)
        pc.end_iteration()
    got = pc.gather()
    sd = pc.state_dict()
    st = pc.tc.cache_stats()
    pc.close(restore=True)
    with torch.no_grad():                                  # the model works without the cache again
        assert torch.equal(model(**inputs).logits, ref(**inputs).logits)
    assert len(got) == len(list(ref.parameters()))
    for a, b in zip(got, ref.parameters()):
        assert torch.equal(a.view(torch.uint8), b.detach().cpu().view(torch.uint8))
    assert st["misses"] == 0 and st["n_ops"][1] > 50 and st["bytes_h2d"] > total
    # a checkpoint written from the cache: every name of the model's own state_dict, tied names included
    want = ref.state_dict()
    assert list(sd) == list(want)
    for name in want:
        assert torch.equal(sd[name].cpu().view(torch.uint8), want[name].cpu().view(torch.uint8)), name


def test_training_demo_runs_a_gpt_shaped_model_through_the_cache(capsys, monkeypatch):
    # the demonstration script, at a size that takes a second: attention blocks, embedding,
    # untied head, bf16; every parameter passes through the cache and nothing misses
    import json
    import sys
    from paper_2511_14124_amd import train_demo
    monkeypatch.setattr(sys, "argv", ["train_demo", "--layers", "2", "--d-model", "128", "--heads", "4", "--vocab", "512",
                                      "--batch", "2", "--seq", "64", "--steps", "2", "--cache", "0.4"])
    train_demo.main()
    out = json.loads(capsys.readouterr().out.strip().splitlines()[-1])
    assert out["through_cache"]["hit_rate"] == 1.0 and out["final_parameters_equal_resident_training"]
    assert out["through_cache"]["h2d_GiB_per_step"] > 0 and out["cache_fraction"] < 0.8
    assert out["model"]["modules_with_hooks"] == 2 * 6 + 3


def test_training_demo_with_the_gradients_in_the_cache():
    from paper_2511_14124_amd import train_demo
    out = train_demo.main(["--layers", "2", "--d-model", "128", "--heads", "4", "--vocab", "512", "--batch", "2",
                           "--seq", "64", "--steps", "2", "--cache", "0.4", "--manage-grads"])
    assert out["managed"] == "parameters and gradients" and out["final_parameters_equal_resident_training"]
    assert out["through_cache"]["hit_rate"] == 1.0 and out["cache_fraction"] < 0.8


def test_training_demo_with_a_model_of_the_transformers_package():
    pytest.importorskip("transformers")
    from paper_2511_14124_amd import train_demo
    out = train_demo.main(["--hf", "gpt2", "--layers", "2", "--d-model", "128", "--heads", "4", "--vocab", "512",
                           "--batch", "2", "--seq", "64", "--steps", "2", "--cache", "0.4"])
    assert out["model"]["class"] == "transformers.GPT2LMHeadModel" and out["final_parameters_equal_resident_training"]
    assert out["through_cache"]["hit_rate"] == 1.0 and out["cache_fraction"] < 0.8


def test_train_demo_with_cpu_adam_over_the_two_tier_cache():
    # the whole pipeline on a small model: 16-bit parameters through the HBM cache, fp32 Adam
    # states through the host cache over a file, the update on the CPU; three steps give the
    # parameters and master copies of the same training with everything resident, bit for bit
    from paper_2511_14124_amd import train_demo
    out = train_demo.main(["--layers", "2", "--d-model", "128", "--heads", "4", "--vocab", "512", "--batch", "2",
                           "--seq", "64", "--steps", "2", "--cache", "0.4", "--cpu-adam", "--state-cache", "0.4",
                           "--threads", "4"])
    assert out["final_parameters_equal_resident_training"] and out["sampled_master_copies_equal"]
    assert out["steps_checked"] == 3
    both = out["through_both_caches"]
    assert both["param_hit_rate"] == 1.0 and both["state_miss_rate"] == 0.0
    assert both["state_file_read_GiB_per_step"] > 0 and out["state_cache_fraction"] < 0.8


def test_a_parameter_that_returns_in_another_buffer_is_read_from_there_in_the_backward_pass():
    # A transformer block's Linear layers keep a transposed view of their weight for the backward
    # pass.  With several size classes and a small cache a weight evicted after its forward comes
    # back for its backward in another buffer: the saved view must follow it there, or the
    # gradients of everything below that layer are computed from bytes of some other tensor.
    from paper_2511_14124_amd.train_demo import build_model
    vocab = 512

    def make():
        torch.manual_seed(3)
        return build_model(torch, 128, 6, 4, vocab, torch.bfloat16)

    gen = torch.Generator(device="cuda:0").manual_seed(5)
    tokens = torch.randint(0, vocab, (2, 64), device="cuda:0", generator=gen)
    target = torch.randint(0, vocab, (2, 64), device="cuda:0", generator=gen)
    loss_fn = torch.nn.CrossEntropyLoss()

    def iteration(m):
        loss_fn(m(tokens).float().view(-1, vocab), target.view(-1)).backward()

    ref = make()
    iteration(ref)
    want = [p.grad.clone() for p in ref.parameters()]
    model = make()
    total = sum(p.numel() * p.element_size() for p in model.parameters())
    pc = ParamCache(model, hbm_bytes=int(total * 0.26))
    pc.profile(lambda: iteration(model))
    pc.install()
    for _ in range(2):                                     # the second iteration starts from restored buffers
        iteration(model)
        torch.cuda.synchronize()
        got = [p.grad.clone() for p in pc.params]
        pc.end_iteration()
        assert all(torch.equal(a, b) for a, b in zip(got, want))
    buffers = {}
    for (t, ptr) in pc._views:
        buffers.setdefault(t, set()).add(ptr)
    assert any(len(v) > 1 for v in buffers.values())       # some parameter did change buffers
    pc.close()


def test_train_demo_chooses_its_copy_path_by_timing():
    # six steps time the kernel alone against DMA copies behind a compute backlog and the faster
    # setting stays; whichever it is, training equals resident training bit for bit
    from paper_2511_14124_amd import train_demo
    out = train_demo.main(["--layers", "2", "--d-model", "128", "--heads", "4", "--vocab", "512", "--batch", "2",
                           "--seq", "64", "--steps", "2", "--cache", "0.4", "--dma-auto", "--fused-sgd"])
    assert out["final_parameters_equal_resident_training"]
    assert out["through_cache"]["chosen_by_timing"] and out["through_cache"]["dma_copies_from_KiB"] in (None, 64)
