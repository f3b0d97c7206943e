"""Hook-driven migration under real compute: a GPT-shaped decoder trained with
its parameters in the tensor cache, against the same model with its parameters
resident.

Run as `python -m paper_2511_14124_amd.train_demo` on a GPU.  The model is built
from leaf modules that own their parameters (LayerNorm, Linear, Embedding), so
that the pre- and post-hooks of the paper's analyzer (Sec. 3.2.1) see every
parameter; `ParamCache` profiles one iteration, plans the pools for an HBM
budget of `--cache` times the parameter bytes and then fetches and evicts the
parameters around every module.  Activations stay ordinary PyTorch tensors;
gradients do too unless `--manage-grads` puts them into the cache, and `--adam`
keeps Adam's two fp32 moments there as well (`--file PATH` adds a file tier
below pinned host memory, `--hf gpt2|llama` trains the transformers package's
classes).  Prints one JSON line: step time of both runs, tokens/s, what
moved per step and the cache's hit rate.

With `--cpu-adam` the update is the paper's whole pipeline in miniature
(Sec. 3.4.2): the 16-bit parameters go through the HBM cache as before, and per
parameter an fp32 master copy, momentum and variance live in a second,
two-tier cache (pinned host memory over a file); the sweep brings each
gradient to the host, runs Adam on the CPU over the cached states and writes
the rounded master copy back into the parameter's HBM buffer.  The reference
run does the same arithmetic with everything resident, and the final
parameters of the two must be equal bit for bit.
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


def build_library_model(torch, family, d_model, n_layers, n_heads, vocab, seq, dtype):
    """A model this package did not write: the GPT-2 (head tied to the token table) or Llama class of the
    transformers package at the given size, random weights, no dropout; nothing is downloaded."""
    import transformers as tf
    if family == "gpt2":
        cfg = tf.GPT2Config(vocab_size=vocab, n_positions=seq, n_embd=d_model, n_layer=n_layers, n_head=n_heads,
                            resid_pdrop=0.0, embd_pdrop=0.0, attn_pdrop=0.0, bos_token_id=0, eos_token_id=0)
        model = tf.GPT2LMHeadModel(cfg)
    else:
        cfg = tf.LlamaConfig(vocab_size=vocab, hidden_size=d_model, intermediate_size=(8 * d_model // 3 + 255) // 256 * 256,
                             num_hidden_layers=n_layers, num_attention_heads=n_heads, num_key_value_heads=n_heads,
                             max_position_embeddings=seq, bos_token_id=0, eos_token_id=0)
        model = tf.LlamaForCausalLM(cfg)
    return model.to(device="cuda:0", dtype=dtype)


def main(argv=None):
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
    ap.add_argument("--cpu-adam", action="store_true",
                    help="Adam on the CPU, its fp32 states in a two-tier cache (host memory over a file)")
    ap.add_argument("--state-cache", type=float, default=0.5, help="host cache as a fraction of the state bytes")
    ap.add_argument("--threads", type=int, default=8, help="PyTorch CPU threads for the CPU update")
    ap.add_argument("--dma-kib", type=int, default=0,
                    help="parameters of at least this many KiB travel as DMA-engine copies (0: all through the kernel)")
    ap.add_argument("--dma-auto", action="store_true",
                    help="let the first six steps decide between the kernel alone and DMA copies from 64 KiB")
    ap.add_argument("--fused-sgd", action="store_true",
                    help="apply the update in the backward hooks, while the parameters are still in the cache")
    ap.add_argument("--hf", choices=["gpt2", "llama"], default=None,
                    help="train the transformers package's GPT-2 or Llama class at this size instead of the built-in model")
    ap.add_argument("--adam", action="store_true",
                    help="Adam on the GPU with its two fp32 moments as tensors of the cache too "
                         "(--cache is then a fraction of parameters + moments)")
    ap.add_argument("--file", default=None,
                    help="a file for what neither the HBM cache nor --host of pinned memory hold (three tiers)")
    ap.add_argument("--host", type=float, default=0.3, help="with --file: pinned host memory as a fraction of the managed bytes")
    ap.add_argument("--gpu-deps", action="store_true",
                    help="modules and migration launches wait for each other on the GPU (tc_set_gpu_dependencies)")
    ap.add_argument("--manage-grads", action="store_true",
                    help="the gradients are tensors of the cache too (--cache is then a fraction of parameters + gradients)")
    args = ap.parse_args(argv)

    import torch
    from .torch_hooks import ParamCache
    from . import binding as T
    T.load_library()
    if args.cpu_adam:
        return cpu_adam_demo(args, torch, T)
    dtype = torch.bfloat16
    torch.manual_seed(0)
    tokens = torch.randint(0, args.vocab, (args.batch, args.seq), device="cuda:0")
    target = torch.randint(0, args.vocab, (args.batch, args.seq), device="cuda:0")
    loss_fn = torch.nn.CrossEntropyLoss()

    def iteration(model):
        if args.hf:
            model(input_ids=tokens, labels=target).loss.backward()
            return
        logits = model(tokens)
        loss_fn(logits.float().view(-1, args.vocab), target.view(-1)).backward()

    def build():
        if args.hf:
            return build_library_model(torch, args.hf, args.d_model, args.layers, args.heads, args.vocab, args.seq, dtype)
        return build_model(torch, args.d_model, args.layers, args.heads, args.vocab, dtype)

    def timed(step_fn):
        step_fn()                                          # warm-up (allocator, kernel selection)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step_fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / args.steps

    # ---- parameters resident
    torch.manual_seed(0)
    model = build()
    n_params = sum(p.numel() for p in model.parameters())
    param_bytes = sum(p.numel() * p.element_size() for p in model.parameters())

    moments = None
    res_k = 0

    def resident_step():
        nonlocal moments, res_k
        for p in model.parameters():
            p.grad = None
        iteration(model)
        with torch.no_grad():
            if args.adam:
                if moments is None:
                    moments = [(torch.zeros_like(p, dtype=torch.float32), torch.zeros_like(p, dtype=torch.float32))
                               for p in model.parameters()]
                res_k += 1
                for p, (m, v) in zip(model.parameters(), moments):
                    ParamCache.adam_update(p, p.grad, m, v, res_k, args.lr, 0.9, 0.999, 1e-8)
                return
            for p in model.parameters():
                p.add_(p.grad, alpha=-args.lr)

    for _ in range(6 if args.dma_auto else 0):             # as many steps as the tuning of the cached run takes
        resident_step()
    t_res = timed(resident_step)
    want = [p.detach().cpu().clone() for p in model.parameters()]
    del model
    moments = None
    torch.cuda.empty_cache()

    # ---- parameters in the tensor cache
    torch.manual_seed(0)
    model = build()
    managed_bytes = param_bytes * (2 if args.manage_grads else 1) + (8 * n_params if args.adam else 0)
    pc = ParamCache(model, hbm_bytes=int(managed_bytes * args.cache), fused_sgd_lr=args.lr if args.fused_sgd else None,
                    dma_threshold=(args.dma_kib << 10) or None, manage_grads=args.manage_grads,
                    host_bytes=int(managed_bytes * args.host) if args.file else None, file_path=args.file,
                    state_tensors=2 if args.adam else 0)
    pc.profile(lambda: iteration(model))
    pc.install()
    if args.gpu_deps:
        pc.tc.set_gpu_dependencies(True)

    def cached_step():
        iteration(model)
        if args.adam:
            pc.adam_step(args.lr)
        elif not args.fused_sgd:
            pc.sgd_step(args.lr)
        pc.end_iteration()

    s0 = None

    def cached_step_counted():
        nonlocal s0
        if s0 is None:
            s0 = pc.tc.cache_stats()
        cached_step()

    kept = pc.autotune_dma(cached_step) if args.dma_auto else ((args.dma_kib << 10) or None)
    t_off = timed(cached_step_counted)                     # as many steps as the resident run: one warm-up, then timed
    pc.tc.synchronize()
    s1 = pc.tc.cache_stats()
    same = all(torch.equal(a.view(torch.int16), b.view(torch.int16)) for a, b in zip(pc.gather(), want))
    n_counted = args.steps + 1                             # timed() runs one warm-up step after s0 is taken
    plan = pc.tc.plan
    out = {
        "model": {"class": {"gpt2": "transformers.GPT2LMHeadModel", "llama": "transformers.LlamaForCausalLM",
                            None: "built-in GPT-shaped decoder"}[args.hf],
                  "layers": args.layers, "d_model": args.d_model, "params": n_params, "param_GiB": param_bytes / 2**30,
                  "dtype": "bf16", "tokens_per_step": args.batch * args.seq, "modules_with_hooks": len(pc.mods)},
        "hbm_cache_GiB": float(plan.hbm_total) / 2**30, "cache_fraction": float(plan.hbm_total) / managed_bytes,
        "resident": {"ms_per_step": t_res * 1e3, "tokens_per_s": args.batch * args.seq / t_res},
        "through_cache": {"ms_per_step": t_off * 1e3, "tokens_per_s": args.batch * args.seq / t_off,
                          "slowdown": t_off / t_res,
                          "hit_rate": (s1["hits"] - s0["hits"]) / max(1, s1["hits"] - s0["hits"] + s1["misses"] - s0["misses"]),
                          "h2d_GiB_per_step": (s1["bytes_h2d"] - s0["bytes_h2d"]) / n_counted / 2**30,
                          "d2h_GiB_per_step": (s1["bytes_d2h"] - s0["bytes_d2h"]) / n_counted / 2**30,
                          "h2d_GBps_over_the_step": (s1["bytes_h2d"] - s0["bytes_h2d"]) / n_counted / t_off / 1e9,
                          "hook_calls_per_step": 4 * len(pc.mods) + (0 if args.fused_sgd else 2 * len(pc.params)),
                          "update": "in the backward hooks" if args.fused_sgd else "a sweep over the parameters",
                          "dma_copies_from_KiB": (kept >> 10) if kept else None, "chosen_by_timing": bool(args.dma_auto),
                          "file_read_GiB_per_step": (s1["bytes_file_read"] - s0["bytes_file_read"]) / n_counted / 2**30,
                          "file_write_GiB_per_step": (s1["bytes_file_write"] - s0["bytes_file_write"]) / n_counted / 2**30},
        "final_parameters_equal_resident_training": bool(same),
        "managed": ("parameters and gradients" if args.manage_grads else "parameters") + (" and Adam's moments" if args.adam else ""),
        "note": ("parameters and their gradients are managed (activations stay resident)" if args.manage_grads else
                 "of parameters and gradients only the parameters are managed (activations stay resident)") +
                ("; Adam" if args.adam else "; plain SGD") + "; hooks drive tc_migrate_step one call at a time",
    }
    pc.close()
    print(json.dumps(out))
    return out


def cpu_adam_demo(args, torch, T):
    import os
    import tempfile

    import numpy as np

    from .opt_states import OptStateCache, adam_
    from .torch_hooks import ParamCache
    if args.threads:
        torch.set_num_threads(args.threads)
    dtype = torch.bfloat16
    tokens = torch.randint(0, args.vocab, (args.batch, args.seq), device="cuda:0",
                           generator=torch.Generator(device="cuda:0").manual_seed(1))
    target = torch.randint(0, args.vocab, (args.batch, args.seq), device="cuda:0",
                           generator=torch.Generator(device="cuda:0").manual_seed(2))
    loss_fn = torch.nn.CrossEntropyLoss()

    def iteration(model):
        loss_fn(model(tokens).float().view(-1, args.vocab), target.view(-1)).backward()

    def make_model():
        torch.manual_seed(0)
        return build_model(torch, args.d_model, args.layers, args.heads, args.vocab, dtype)

    model = make_model()
    params = list(model.parameters())
    elems = [p.numel() for p in params]
    g_host = torch.empty(max(elems), dtype=torch.float32).pin_memory()    # a gradient on its way to the CPU
    tmp = torch.empty(max(elems), dtype=torch.float32)
    n_steps = args.steps + 1                                              # one warm-up step, also checked

    def cpu_update(p, states, step):
        """Gradient to the host, Adam on the CPU, rounded master copy back into the parameter."""
        n = p.numel()
        master, m, v = states
        g_host[:n].copy_(p.grad.reshape(-1))                              # bf16 on the GPU -> fp32 pinned, synchronous
        adam_(torch, master, m, v, g_host[:n], tmp[:n], step, lr=args.lr)
        p.data.copy_(master.view(p.shape))

    # ---- everything resident: parameters in HBM, states in ordinary host memory
    states = [[p.detach().float().cpu().reshape(-1), torch.zeros(p.numel()), torch.zeros(p.numel())] for p in params]
    step_no = 0

    def resident_step():
        nonlocal step_no
        step_no += 1
        for p in params:
            p.grad = None
        iteration(model)
        with torch.no_grad():
            for p, st in zip(params, states):
                cpu_update(p, st, step_no)

    resident_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        resident_step()
    torch.cuda.synchronize()
    t_res = (time.perf_counter() - t0) / args.steps
    want = [p.detach().cpu().clone() for p in params]
    want_master = {j: states[j][0].clone() for j in (0, len(params) // 2, len(params) - 1)}
    param_bytes = sum(p.numel() * p.element_size() for p in params)
    del model, params, states
    torch.cuda.empty_cache()

    # ---- parameters through the HBM cache, states through the two-tier cache
    model = make_model()
    pc = ParamCache(model, hbm_bytes=int(param_bytes * args.cache), dma_threshold=(args.dma_kib << 10) or None)
    assert [p.numel() for p in pc.params] == elems         # the same parameter order in both runs
    tmpdir = tempfile.TemporaryDirectory(prefix="tc_states_")
    state_bytes = 12 * sum(elems)
    sc = OptStateCache(elems, int(state_bytes * args.state_cache), os.path.join(tmpdir.name, "states.bin"))
    for j, p in enumerate(pc.params):
        sc.load(j, p.detach().float().cpu().numpy())
    pc.profile(lambda: iteration(model))
    pc.install()
    pc.tc.set_oplog(False, True)
    step_no = 0

    def update(j, p):
        st = sc.begin(j)
        cpu_update(p, st, step_no)
        sc.end(j)

    def cached_step():
        nonlocal step_no
        step_no += 1
        iteration(model)
        pc.update_sweep(update)
        sc.end_iteration()
        pc.end_iteration()

    cached_step()
    torch.cuda.synchronize()
    s0, o0 = pc.tc.cache_stats(), sc.stats()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        cached_step()
    torch.cuda.synchronize()
    t_off = (time.perf_counter() - t0) / args.steps
    pc.tc.synchronize()
    sc.tc.synchronize()
    s1, o1 = pc.tc.cache_stats(), sc.stats()
    got = pc.gather()
    differing = [j for j, (a, b) in enumerate(zip(got, want)) if not torch.equal(a.view(torch.int16), b.view(torch.int16))]
    same = not differing
    max_diff = max((float((got[j].float() - want[j].float()).abs().max()) for j in differing), default=0.0)
    same_master = all(np.array_equal(sc.read(j), w.numpy()) for j, w in want_master.items())
    n = args.steps
    out = {
        "model": {"class": {"gpt2": "transformers.GPT2LMHeadModel", "llama": "transformers.LlamaForCausalLM",
                            None: "built-in GPT-shaped decoder"}[args.hf],
                  "layers": args.layers, "d_model": args.d_model, "params": int(sum(elems)),
                  "param_GiB": param_bytes / 2**30, "state_GiB": state_bytes / 2**30, "dtype": "bf16 + fp32 states",
                  "tokens_per_step": args.batch * args.seq},
        "hbm_cache_fraction": float(pc.tc.plan.hbm_total) / param_bytes,
        "state_cache_fraction": float(sc.tc.plan.hbm_total) / state_bytes,
        "cpu_threads": torch.get_num_threads(),
        "resident": {"ms_per_step": t_res * 1e3},
        "through_both_caches": {
            "ms_per_step": t_off * 1e3, "slowdown": t_off / t_res,
            "param_hit_rate": (s1["hits"] - s0["hits"]) / max(1, s1["hits"] - s0["hits"] + s1["misses"] - s0["misses"]),
            "state_miss_rate": (o1["misses"] - o0["misses"]) / max(1, o1["hits"] - o0["hits"] + o1["misses"] - o0["misses"]),
            "h2d_GiB_per_step": (s1["bytes_h2d"] - s0["bytes_h2d"]) / n / 2**30,
            "state_file_read_GiB_per_step": (o1["bytes_file_read"] - o0["bytes_file_read"]) / n / 2**30,
            "state_file_write_GiB_per_step": (o1["bytes_file_write"] - o0["bytes_file_write"]) / n / 2**30,
            "ms_blocked_for_states_per_step": (o1["stall_ns"] - o0["stall_ns"]) / n / 1e6,
        },
        "final_parameters_equal_resident_training": bool(same),
        "parameters_differing": len(differing), "first_differing": differing[:6], "max_abs_difference": max_diff,
        "sampled_master_copies_equal": bool(same_master),
        "steps_checked": n_steps,
    }
    sc.close()
    pc.close()
    tmpdir.cleanup()
    print(json.dumps(out))
    return out


if __name__ == "__main__":
    main()
