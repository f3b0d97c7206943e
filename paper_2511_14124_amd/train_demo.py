"""Hook-driven migration under real compute: a GPT-shaped decoder trained with
its parameters in the tensor cache, against the same model with its parameters
resident.

Run as `python -m paper_2511_14124_amd.train_demo` on a GPU.  The model is built
from leaf modules that own their parameters (LayerNorm, Linear, Embedding), so
that the pre- and post-hooks of the paper's analyzer (Sec. 3.2.1) see every
parameter; `ParamCache` profiles one iteration, plans the pools for an HBM
budget of `--cache` times the parameter bytes and then fetches and evicts the
parameters around every module.  Gradients and activations stay ordinary
PyTorch tensors.  Prints one JSON line: step time of both runs, tokens/s, what
moved per step and the cache's hit rate.
"""

from __future__ import annotations

import argparse
import json
import time


def build_model(torch, d_model, n_layers, n_heads, vocab, dtype):
    nn, F = torch.nn, torch.nn.functional

    class Block(nn.Module):
        def __init__(self):
            super().__init__()
            self.ln1 = nn.LayerNorm(d_model)
            self.qkv = nn.Linear(d_model, 3 * d_model)
            self.proj = nn.Linear(d_model, d_model)
            self.ln2 = nn.LayerNorm(d_model)
            self.fc1 = nn.Linear(d_model, 4 * d_model)
            self.fc2 = nn.Linear(4 * d_model, d_model)

        def forward(self, x):
            b, s, d = x.shape
            q, k, v = self.qkv(self.ln1(x)).view(b, s, 3, n_heads, d // n_heads).permute(2, 0, 3, 1, 4)
            a = F.scaled_dot_product_attention(q, k, v, is_causal=True)
            x = x + self.proj(a.transpose(1, 2).reshape(b, s, d))
            return x + self.fc2(F.gelu(self.fc1(self.ln2(x))))

    class Model(nn.Module):
        def __init__(self):
            super().__init__()
            self.emb = nn.Embedding(vocab, d_model)
            self.blocks = nn.ModuleList([Block() for _ in range(n_layers)])
            self.lnf = nn.LayerNorm(d_model)
            self.head = nn.Linear(d_model, vocab, bias=False)

        def forward(self, tokens):
            x = self.emb(tokens)
            for blk in self.blocks:
                x = blk(x)
            return self.head(self.lnf(x))

    return Model().to(device="cuda:0", dtype=dtype)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--layers", type=int, default=12)
    ap.add_argument("--d-model", type=int, default=2048)
    ap.add_argument("--heads", type=int, default=16)
    ap.add_argument("--vocab", type=int, default=8192)
    ap.add_argument("--batch", type=int, default=4)
    ap.add_argument("--seq", type=int, default=1024)
    ap.add_argument("--cache", type=float, default=0.3, help="HBM cache as a fraction of the parameter bytes")
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--lr", type=float, default=1e-3)
    ap.add_argument("--fused-sgd", action="store_true",
                    help="apply the update in the backward hooks, while the parameters are still in the cache")
    args = ap.parse_args()

    import torch
    from .torch_hooks import ParamCache
    from . import binding as T
    T.load_library()
    dtype = torch.bfloat16
    torch.manual_seed(0)
    tokens = torch.randint(0, args.vocab, (args.batch, args.seq), device="cuda:0")
    target = torch.randint(0, args.vocab, (args.batch, args.seq), device="cuda:0")
    loss_fn = torch.nn.CrossEntropyLoss()

    def iteration(model):
        logits = model(tokens)
        loss_fn(logits.float().view(-1, args.vocab), target.view(-1)).backward()

    def timed(step_fn):
        step_fn()                                          # warm-up (allocator, kernel selection)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step_fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / args.steps

    # ---- parameters resident
    model = build_model(torch, args.d_model, args.layers, args.heads, args.vocab, dtype)
    n_params = sum(p.numel() for p in model.parameters())
    param_bytes = sum(p.numel() * p.element_size() for p in model.parameters())

    def resident_step():
        for p in model.parameters():
            p.grad = None
        iteration(model)
        with torch.no_grad():
            for p in model.parameters():
                p.add_(p.grad, alpha=-args.lr)

    t_res = timed(resident_step)
    del model
    torch.cuda.empty_cache()

    # ---- parameters in the tensor cache
    torch.manual_seed(0)
    model = build_model(torch, args.d_model, args.layers, args.heads, args.vocab, dtype)
    pc = ParamCache(model, hbm_bytes=int(param_bytes * args.cache), fused_sgd_lr=args.lr if args.fused_sgd else None)
    pc.profile(lambda: iteration(model))
    pc.install()
    pc.tc.set_oplog(False, True)

    def cached_step():
        iteration(model)
        if not args.fused_sgd:
            pc.sgd_step(args.lr)
        pc.end_iteration()

    s0 = None

    def cached_step_counted():
        nonlocal s0
        if s0 is None:
            s0 = pc.tc.cache_stats()
        cached_step()

    cached_step()                                          # first pass through the hooks
    torch.cuda.synchronize()
    t_off = timed(cached_step_counted)
    pc.tc.synchronize()
    s1 = pc.tc.cache_stats()
    n_counted = args.steps + 1                             # timed() runs one warm-up step after s0 is taken
    plan = pc.tc.plan
    out = {
        "model": {"layers": args.layers, "d_model": args.d_model, "params": n_params, "param_GiB": param_bytes / 2**30,
                  "dtype": "bf16", "tokens_per_step": args.batch * args.seq, "modules_with_hooks": len(pc.mods)},
        "hbm_cache_GiB": float(plan.hbm_total) / 2**30, "cache_fraction": float(plan.hbm_total) / param_bytes,
        "resident": {"ms_per_step": t_res * 1e3, "tokens_per_s": args.batch * args.seq / t_res},
        "through_cache": {"ms_per_step": t_off * 1e3, "tokens_per_s": args.batch * args.seq / t_off,
                          "slowdown": t_off / t_res,
                          "hit_rate": (s1["hits"] - s0["hits"]) / max(1, s1["hits"] - s0["hits"] + s1["misses"] - s0["misses"]),
                          "h2d_GiB_per_step": (s1["bytes_h2d"] - s0["bytes_h2d"]) / n_counted / 2**30,
                          "d2h_GiB_per_step": (s1["bytes_d2h"] - s0["bytes_d2h"]) / n_counted / 2**30,
                          "h2d_GBps_over_the_step": (s1["bytes_h2d"] - s0["bytes_h2d"]) / n_counted / t_off / 1e9,
                          "hook_calls_per_step": 4 * len(pc.mods) + (0 if args.fused_sgd else 2 * len(pc.params)),
                          "update": "in the backward hooks" if args.fused_sgd else "a sweep over the parameters"},
        "note": "parameters only are managed (gradients and activations stay resident); plain SGD; hooks drive "
                "tc_migrate_step one call at a time",
    }
    pc.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
