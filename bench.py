#!/usr/bin/env python3
"""Benchmark of the AGZO per-step hot path on one MI355X.

Workload: the seven projections of one Qwen3-8B-shaped decoder layer (bf16 weights and
activations, N = 16 x 1024 tokens, r = 16, K = 3 power steps, MSE loss), synthetic inputs with a
power-law activation spectrum plus outlier channels.  One *step* = one full AGZO step (base forward
with subspace extraction, two perturbed forwards, two-point scalar, in-place rank-r update) for each
of the seven projections; as in Alg. 2 the updates follow once every scalar is known, in one batched
call for the seven matrices.  Inputs are resident in HBM before the timed region starts.

Prints one JSON line: steps/s for the layer set, the roofline of the dominant kernel (the forward
GEMM, timed live with HIP events on the library's stream), the update kernel's HBM figure, and the
CPU oracle timed on this host as a baseline.
"""
import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2601_17261_amd import binding, synth  # noqa: E402

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E


def build_layer_set(n_tokens, shapes, seed):
    """One (W, X, Y*) triple per projection; projections that read the same activations share X."""
    groups = {"q": "attn", "k": "attn", "v": "attn", "gate": "mlp", "up": "mlp"}
    xs, out = {}, []
    for idx, (name, d_in, d_out) in enumerate(shapes):
        key = groups.get(name, name)
        if key not in xs:
            xs[key] = synth.device_powerlaw_x(seed + 100 + idx, n_tokens, d_in)
        X = xs[key]
        W, T = synth.device_weights_and_target(seed + idx, X, d_out)
        out.append((name, d_in, d_out, W, X, T))
    torch.cuda.synchronize()
    return out


def cpu_baseline(n_tokens, r, K, eps, lr, shapes, budget_s=25.0):
    """The oracle, as it stands, on this host: full steps of the layer set's projections at the benchmark's token
    count, smallest first, until about `budget_s` seconds of CPU work are spent; what was not reached is scaled in by
    forward-flop ratio."""
    from oracle import agzo as oagzo
    try:
        import threadpoolctl
        cores = max(i["num_threads"] for i in threadpoolctl.threadpool_info()) if threadpoolctl.threadpool_info() else 1
    except Exception:
        cores = os.cpu_count() or 1
    rng = np.random.default_rng(0)
    todo = sorted(shapes, key=lambda s: s[1] * s[2])
    total_flops = sum(2.0 * n_tokens * d_in * d_out for _, d_in, d_out in shapes)
    spent, done_flops, done = 0.0, 0.0, []
    for name, d_in, d_out in todo:
        flops = 2.0 * n_tokens * d_in * d_out
        if done and spent + spent / done_flops * flops > 1.3 * budget_s:
            break                                   # the next one would overrun the budget
        W = synth.weights(rng, d_out, d_in, storage="bf16")
        X = synth.to_bf16_values(rng.standard_normal((n_tokens, d_in)).astype(np.float32))
        T = (X @ W.T).astype(np.float32)
        t0 = time.perf_counter()
        oagzo.agzo_step(W, X, T, r, K, eps, lr, seed=1, storage="bf16")
        spent += time.perf_counter() - t0
        done_flops += flops
        done.append(name)
        del W, X, T
    scale = total_flops / done_flops
    return {"value": 1.0 / (spent * scale), "unit": "steps/s", "cores": int(cores), "kind": "oracle",
            "sample": "one oracle step each of the projections %s (N=%d, r=%d, K=%d) took %.1f s; %s; inputs of the CPU leg: "
                      "iid N(0,1) activations rounded to bf16, W ~ N(0, 0.02^2), target = X W^T (every loss is 0: the "
                      "oracle's time does not depend on the values, so the GPU leg's power-law activations are not "
                      "regenerated on the host)" % (
                ",".join(done), n_tokens, r, K, spent,
                "that is the whole layer set" if len(done) == len(shapes) else
                "scaled to the whole layer set by forward-flop ratio %.2f" % scale)}


class MlpStack:
    """Alg. 2 over a model: the residual stack of gated-MLP blocks with an LM head (hidden 2048, intermediate 6144,
    vocabulary 32000), all linear layers perturbed at once, one global g.  Every linear-layer operation is a library
    call; the glue between layers (embedding lookup, RMS normalisation, SiLU gate, residual sum: not steps of the
    method) is the library's single-pass kernels (agzo_glue_*: fp32 arithmetic, one rounding to bf16) and a torch
    gather for the embedding.  The base pass keeps every layer's input (a few GB), so that all 85 extractions run as
    one batched call."""

    def __init__(self, ctx, params, ids, r, K):
        self.ctx, self.r, self.K = ctx, r, K
        self.nb = params["n_blocks"]
        self.names = []
        for b in range(self.nb):
            self.names += [("gate", b), ("up", b), ("down", b)]
        self.names.append(("head", 0))
        self.W = {nm: params[nm] for nm in self.names}
        self.E = params["E"]
        self.ids = ids.reshape(-1)
        tgt = torch.full(ids.shape, -1, dtype=torch.int32, device=ids.device)
        tgt[:, :-1] = ids[:, 1:].to(torch.int32)
        self.tgt = tgt.reshape(-1).contiguous()
        self.loss = binding.make_loss(self.tgt, kind=binding.LOSS_CE)
        n = self.ids.numel()
        self.Y = {nm: torch.empty(n, self.W[nm].shape[0], dtype=torch.bfloat16, device="cuda") for nm in self.names if nm[0] != "head"}
        self.B = {nm: torch.empty(self.W[nm].shape[1], r, dtype=torch.float32, device="cuda") for nm in self.names}
        self.X = {}
        self.out = torch.zeros(4, dtype=torch.float64, device="cuda")
        self.flops_fwd = sum(2.0 * n * self.W[nm].shape[0] * self.W[nm].shape[1] for nm in self.names)
        self.flops_rank = sum(2.0 * n * r * (self.W[nm].shape[0] + self.W[nm].shape[1]) for nm in self.names)

    def rms(self, h):
        y = torch.empty_like(h)
        self.ctx.glue_rmsnorm(h, y)
        return y

    def linear(self, nm, x, sign, eps, seed0, loss_dev):
        W, Y = self.W[nm], self.Y.get(nm)
        L = binding.make_layer(W, x, self.r, Y=Y)
        loss = self.loss if nm[0] == "head" else None
        seed = seed0 + self.names.index(nm)
        if sign == 0:
            self.X[nm] = x
            self.ctx.layer_forward_sketch(L, W, x, Y, binding.SKETCH_NONE, None, seed, None, loss, loss_dev)
        else:
            self.ctx.perturbed_forward(L, W, x, self.B[nm], seed, sign * eps, Y, loss, loss_dev)
        return Y

    def run_pass(self, sign, eps, seed0, loss_dev):
        h = self.E[self.ids]
        for b in range(self.nb):
            n = self.rms(h)
            a = self.linear(("gate", b), n, sign, eps, seed0, None)
            u = self.linear(("up", b), n, sign, eps, seed0, None)
            m = torch.empty_like(a)
            self.ctx.glue_swiglu(a, u, m)
            d = self.linear(("down", b), m, sign, eps, seed0, None)
            self.ctx.glue_add(h, d)
        self.linear(("head", 0), self.rms(h), sign, eps, seed0, loss_dev)

    def step(self, step, eps, lr):
        seed0 = 100_000 * (step + 1)
        self.run_pass(0, eps, seed0, self.out[0:1])
        self.ctx.basis_many([(binding.make_layer(self.W[nm], self.X[nm], self.r), self.X[nm], seed0 + i, None, self.B[nm])
                             for i, nm in enumerate(self.names)], self.K)
        self.X.clear()
        self.run_pass(+1, eps, seed0, self.out[1:2])
        self.run_pass(-1, eps, seed0, self.out[2:3])
        self.ctx.two_point(self.out, eps)
        self.ctx.update_many([(self.W[nm], self.B[nm], seed0 + i, lr, self.out[3:4]) for i, nm in enumerate(self.names)])


class Decoder(MlpStack):
    """Alg. 2 over full decoder layers (grouped-query attention with 128-wide heads, per-head normalisation, rotary
    embedding, gated MLP) with an LM head: eight linear layers per decoder layer all perturbed at once, one global g.
    share_bases: layers that read the same activations (q / k / v, gate / up) carry one basis (the paper extracts per
    layer; their Gaussian factors stay their own)."""

    def __init__(self, ctx, params, ids, r, K, share_bases):
        self.ctx, self.r, self.K = ctx, r, K
        self.nl = params["n_layers"]
        self.n_seq, self.T = ids.shape
        self.names = []
        for l in range(self.nl):
            self.names += [(p, l) for p in synth.DECODER_PROJECTIONS]
        self.names.append(("head", 0))
        self.index = {nm: i for i, nm in enumerate(self.names)}
        self.W = {nm: params[nm] for nm in self.names}
        self.E = params["E"]
        self.ids = ids.reshape(-1)
        tgt = torch.full(ids.shape, -1, dtype=torch.int32, device=ids.device)
        tgt[:, :-1] = ids[:, 1:].to(torch.int32)
        self.tgt = tgt.reshape(-1).contiguous()
        self.loss = binding.make_loss(self.tgt, kind=binding.LOSS_CE)
        n = self.ids.numel()
        self.Y = {nm: torch.empty(n, self.W[nm].shape[0], dtype=torch.bfloat16, device="cuda") for nm in self.names if nm[0] != "head"}
        self.share = {}
        if share_bases:
            for l in range(self.nl):
                self.share.update({("k", l): ("q", l), ("v", l): ("q", l), ("up", l): ("gate", l)})
        self.B = {nm: torch.empty(self.W[nm].shape[1], r, dtype=torch.float32, device="cuda") for nm in self.names if nm not in self.share}
        for nm, src in self.share.items():
            self.B[nm] = self.B[src]
        self.X = {}
        self.out = torch.zeros(4, dtype=torch.float64, device="cuda")
        self.flops_fwd = sum(2.0 * n * self.W[nm].shape[0] * self.W[nm].shape[1] for nm in self.names)
        self.flops_rank = sum(2.0 * n * r * (self.W[nm].shape[0] + self.W[nm].shape[1]) for nm in self.names)

    def linear(self, nm, x, sign, eps, seed0, loss_dev):
        W, Y = self.W[nm], self.Y.get(nm)
        L = binding.make_layer(W, x, self.r, Y=Y)
        loss = self.loss if nm[0] == "head" else None
        seed = seed0 + self.index[nm]
        if sign == 0:
            self.X[nm] = x
            self.ctx.layer_forward_sketch(L, W, x, Y, binding.SKETCH_NONE, None, seed, None, loss, loss_dev)
        else:
            self.ctx.perturbed_forward(L, W, x, self.B[nm], seed, sign * eps, Y, loss, loss_dev)
        return Y

    def run_pass(self, sign, eps, seed0, loss_dev):
        h = self.E[self.ids]
        for l in range(self.nl):
            n = self.rms(h)
            q, k, v = (self.linear((p, l), n, sign, eps, seed0, None) for p in ("q", "k", "v"))
            a = torch.empty_like(q)
            self.ctx.glue_attention(q, k, v, a, self.n_seq, self.T)
            self.ctx.glue_add(h, self.linear(("o", l), a, sign, eps, seed0, None))
            n = self.rms(h)
            g, u = self.linear(("gate", l), n, sign, eps, seed0, None), self.linear(("up", l), n, sign, eps, seed0, None)
            m = torch.empty_like(g)
            self.ctx.glue_swiglu(g, u, m)
            self.ctx.glue_add(h, self.linear(("down", l), m, sign, eps, seed0, None))
        self.linear(("head", 0), self.rms(h), sign, eps, seed0, loss_dev)

    def step(self, step, eps, lr):
        seed0 = 100_000 * (step + 1)
        self.run_pass(0, eps, seed0, self.out[0:1])
        own = [nm for nm in self.names if nm not in self.share]
        self.ctx.basis_many([(binding.make_layer(self.W[nm], self.X[nm], self.r), self.X[nm], seed0 + self.index[nm], None, self.B[nm])
                             for nm in own], self.K)
        self.X.clear()
        self.run_pass(+1, eps, seed0, self.out[1:2])
        self.run_pass(-1, eps, seed0, self.out[2:3])
        self.ctx.two_point(self.out, eps)
        self.ctx.update_many([(self.W[nm], self.B[nm], seed0 + self.index[nm], lr, self.out[3:4]) for nm in self.names])


def run_model(ctx, model, steps, warmup, note):
    eps, lr = float(np.float32(1e-3)), float(np.float32(1e-4))
    for s in range(warmup):
        model.step(s, eps, lr)
    ctx.check()
    torch.cuda.synchronize()
    ctx.profile_enable(1 << binding.PROF_GEMM)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    t0 = time.perf_counter()
    for s in range(steps):
        ev[s].record()
        model.step(warmup + s, eps, lr)
    ev[steps].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    n_g, ms_g = ctx.profile_read(binding.PROF_GEMM)
    ctx.profile_enable(False)
    ctx.check()
    losses = model.out.cpu().numpy()
    if not np.isfinite(losses).all():
        raise RuntimeError("non-finite loss in the model workload")
    per_step = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(steps))
    med = per_step[len(per_step) // 2]
    flops = 3.0 * model.flops_fwd + 2.0 * model.flops_rank
    return {"value": 1e3 / med, "unit": "steps/s", "ms_per_step": med, "ms_per_step_mean_wall": 1e3 * dt / steps, "steps": steps,
            "gemm_launches": n_g, "gemm_ms_per_step": ms_g / steps, "gemm_tflops": flops * steps / (ms_g * 1e-3) / 1e12,
            "forward_tflop": model.flops_fwd / 1e12, "linear_layers": len(model.names), "tokens": int(model.ids.numel()),
            "rank": model.r, "power_steps": model.K, "losses": {"L0": losses[0], "L+": losses[1], "L-": losses[2], "g": losses[3]},
            "note": note}


def run_decoder(ctx, steps, warmup, r=16, K=3, n_layers=28, n_seq=16, seq_len=512, share_bases=False):
    """Steps per second of Alg. 2 over a Qwen3-1.7B-shaped decoder (hidden 2048, 16 query heads on 8 kv heads of 128,
    intermediate 6144, 28 layers, vocabulary 32000), 16 x 512 tokens, token cross-entropy, global g."""
    params, ids = synth.device_decoder(13, n_layers, 2048, 16, 8, 6144, 32000, n_seq, seq_len)
    model = Decoder(ctx, params, ids, r, K, share_bases)
    return run_model(ctx, model, steps, warmup,
                     "Alg. 2 over %d decoder layers + LM head (%d linear layers): base pass keeping every layer's input, one batched "
                     "extraction (%s), two perturbed passes, global g, one batched update; attention, normalisations, gate and "
                     "residual sums are the library's glue kernels" % (n_layers, len(model.names),
                                                                       "one basis per distinct input" if share_bases else "one basis per layer"))


def run_mlp_stack(ctx, steps, warmup, r=16, K=3, n_blocks=28, n_seq=16, seq_len=512):
    """Steps per second of the MLP-stack workload (28 blocks + LM head, 16 x 512 tokens, token cross-entropy, global g)."""
    params, ids = synth.device_mlp_stack(11, n_blocks, 2048, 6144, 32000, n_seq, seq_len)
    model = MlpStack(ctx, params, ids, r, K)
    return run_model(ctx, model, steps, warmup,
                     "Alg. 2 over %d blocks + LM head: base pass keeping every layer's input, one batched extraction for the "
                     "%d layers, two perturbed passes (factored, fused cross-entropy on the head), global g, one batched "
                     "update" % (n_blocks, len(model.names)))


def gemm_shapes(args):
    """The forward GEMM alone on each distinct projection shape of the Qwen3-8B layer (for counter-collection runs: with
    --shape every GEMM dispatch of the process has that one shape).  Prints one JSON line per shape and variant."""
    ctx = binding.Context()
    N, r = args.tokens, args.rank
    eps = float(np.float32(1e-3))
    shapes = [("q", 4096, 4096), ("k", 4096, 1024), ("gate", 4096, 12288), ("down", 12288, 4096)]
    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)            # 1 GiB read + 1 GiB written by one elementwise kernel: scale for the traffic counters
        torch.cuda.synchronize()
        del src, dst
    xs = {}
    for name, d_in, d_out in shapes:
        if args.shape and name != args.shape:
            continue
        if d_in not in xs:
            xs[d_in] = synth.device_powerlaw_x(100 + d_in, N, d_in)
        X = xs[d_in]
        W, T = synth.device_weights_and_target(3 + d_out, X, d_out)
        L, loss = binding.make_layer(W, X, r), binding.make_loss(T)
        sc = torch.zeros(4, dtype=torch.float64, device="cuda")
        B = torch.empty(d_in, r, device="cuda")
        ctx.basis(L, X, 1, 5, None, 0, B)
        ctx.check()
        Ys = torch.empty(N, d_out, dtype=torch.bfloat16, device="cuda")
        Ls = binding.make_layer(W, X, r, Y=Ys)
        variants = {"base_forward_loss": lambda: ctx.layer_forward_sketch(L, W, X, None, 0, None, 1, None, loss, sc[0:1]),
                    "perturbed_forward_loss": lambda: ctx.perturbed_forward(L, W, X, B, 5, eps, None, loss, sc[1:2]),
                    # what the vendor's GEMM below does: bf16 output stored, no loss (the kernel a layer inside a model takes)
                    "base_forward_stores_output": lambda: ctx.layer_forward_sketch(Ls, W, X, Ys, 0, None, 1, None, None, None)}
        if not args.store_variant:
            del variants["base_forward_stores_output"]
        for vname, fn in variants.items():
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            ctx.profile_enable(1 << binding.PROF_GEMM)
            for _ in range(args.steps):
                fn()
            n, ms = ctx.profile_read(binding.PROF_GEMM)
            _, ghz = ctx.profile_clock()
            ctx.profile_enable(False)
            flops = 2.0 * N * d_in * d_out + (2.0 * N * r * (d_in + d_out) if vname.startswith("pert") else 0.0)
            print(json.dumps({"shape": "%s %d->%d" % (name, d_in, d_out), "tokens": N, "variant": vname, "launches": n,
                              "avg_us": 1e3 * ms / n, "tflops": flops / (ms / n * 1e-3) / 1e12, "shader_clock_ghz": ghz,
                              "algorithmic_bytes": 2.0 * N * d_in + 2.0 * d_in * d_out + 2.0 * N * d_out}), flush=True)
        # yardstick: the vendor library's plain bf16 GEMM (torch.matmul -> hipBLASLt / rocBLAS) on the same operands in the same
        # process: no loss, stores the N x d_out output; what this box's power budget lets a tuned kernel of that shape reach
        Yl = X @ W.t()
        for _ in range(3):
            torch.matmul(X, W.t(), out=Yl)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
        ev[0].record()
        for i in range(args.steps):
            torch.matmul(X, W.t(), out=Yl)
            ev[i + 1].record()
        torch.cuda.synchronize()
        us = sorted(1e3 * ev[i].elapsed_time(ev[i + 1]) for i in range(args.steps))
        print(json.dumps({"shape": "%s %d->%d" % (name, d_in, d_out), "tokens": N, "variant": "library_gemm_stores_output_no_loss", "launches": args.steps,
                          "avg_us": sum(us) / len(us), "median_us": us[len(us) // 2], "tflops": 2.0 * N * d_in * d_out / (sum(us) / len(us) * 1e-6) / 1e12}), flush=True)
        del W, T, Yl, Ys


def sketch_fusion(args):
    """Range sketch of Alg. 1 taken by a sweep of its own over X against the same sketch emitted by the forward GEMM
    (AGZO_SKETCH_RANGE_FUSED), on the projection shapes of the Qwen3-0.6B layer set (the shapes whose forward runs in
    the 128 x 128 tiling).  Per shape: torch-event time of the forward alone, forward + separate sketch, fused forward.
    One JSON line per shape and a summary line."""
    ctx = binding.Context()
    N, r = args.tokens, args.rank
    rows, tot = [], {"forward": 0.0, "separate": 0.0, "fused": 0.0}
    xs = {}
    for name, d_in, d_out in synth.QWEN3_0P6B_LAYER:
        if d_in not in xs:
            xs[d_in] = synth.device_powerlaw_x(100 + d_in, N, d_in)
        X = xs[d_in]
        W, T = synth.device_weights_and_target(3 + d_out, X, d_out)
        L, loss = binding.make_layer(W, X, r), binding.make_loss(T)
        sc = torch.zeros(1, dtype=torch.float64, device="cuda")
        S = torch.empty(d_in, r, dtype=torch.float32, device="cuda")
        variants = {"forward": lambda: ctx.layer_forward_sketch(L, W, X, None, binding.SKETCH_NONE, None, 1, None, loss, sc),
                    "separate": lambda: ctx.layer_forward_sketch(L, W, X, None, binding.SKETCH_RANGE, None, 1, S, loss, sc),
                    "fused": lambda: ctx.layer_forward_sketch(L, W, X, None, binding.SKETCH_RANGE_FUSED, None, 1, S, loss, sc)}
        res = {"shape": "%s %d->%d" % (name, d_in, d_out), "tokens": N, "rank": r}
        for vname, fn in variants.items():
            for _ in range(5):
                fn()
            ctx.check()
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
            ev[0].record()
            for i in range(args.steps):
                fn()
                ev[i + 1].record()
            torch.cuda.synchronize()
            us = sorted(1e3 * ev[i].elapsed_time(ev[i + 1]) for i in range(args.steps))
            res[vname + "_us"] = us[len(us) // 2]
            tot[vname] += us[len(us) // 2]
        res["sketch_bytes"] = 2.0 * N * d_in
        rows.append(res)
        print(json.dumps(res), flush=True)
        del W, T
    print(json.dumps({"summary": "sum over the seven projections, us", **tot,
                      "separate_minus_forward": tot["separate"] - tot["forward"], "fused_minus_forward": tot["fused"] - tot["forward"]}))


def sweep(args):
    """Qwen3-4B shapes, r in {1,4,16,64} x N in {512,4096,16384,65536}: per kernel the achieved rate, the
    algorithmic intensity and which roofline (HBM or MFMA) bounds it.  Prints one text table."""
    ctx = binding.Context()
    eps = float(np.float32(1e-3))
    projs = [p for p in synth.QWEN3_4B_LAYER if p[0] in ("q", "k", "gate", "down")]
    print("# kernel rates on Qwen3-4B-shaped projections, bf16; bound = larger of flops/2500 TFLOP/s and bytes/8000 GB/s")
    print("# %-5s %6s %3s | %-9s %9s %9s %8s %7s %6s" % ("proj", "N", "r", "kernel", "us", "TFLOP/s", "GB/s", "flop/B", "bound"))
    table = {}
    for N in (512, 4096, 16384, 65536):
        xs = {}
        for name, d_in, d_out in projs:
            if d_in not in xs:
                xs[d_in] = synth.device_powerlaw_x(7 + d_in, N, d_in)
            X = xs[d_in]
            W, T = synth.device_weights_and_target(3 + d_out, X, d_out)
            loss = binding.make_loss(T)
            sc = torch.zeros(4, dtype=torch.float64, device="cuda")
            for r in (1, 4, 16, 64):
                if r > min(N, d_in):
                    continue
                L = binding.make_layer(W, X, r)
                B = torch.empty(d_in, r, device="cuda")
                ctx.basis(L, X, 1, 5, None, 0, B)
                ctx.check()

                def timed(kind, fn, reps=5):
                    fn()
                    ctx.profile_enable(True)
                    for _ in range(reps):
                        fn()
                    n, ms = ctx.profile_read(kind)
                    ctx.profile_enable(False)
                    return 1e3 * ms / max(n, 1)       # us per launch of that kernel class

                rows = []
                us = timed(binding.PROF_GEMM, lambda: ctx.perturbed_forward(L, W, X, B, 5, eps, None, loss, sc[1:2]))
                rows.append(("pfwd+loss", us, 2.0 * N * d_in * d_out + 2.0 * N * r * (d_in + d_out),
                             2.0 * N * d_in + 2.0 * d_in * d_out + T.element_size() * float(N) * d_out))
                us = timed(binding.PROF_XQ, lambda: ctx.layer_forward_sketch(L, None, X, None, 2, B, 5, B.clone(), None, None))
                rows.append(("xq", us, 2.0 * N * d_in * r, 2.0 * N * d_in))
                us = timed(binding.PROF_XTT, lambda: ctx.layer_forward_sketch(L, None, X, None, 1, None, 5, B.clone(), None, None))
                rows.append(("xtt", us, 2.0 * N * d_in * r, 2.0 * N * d_in))
                us = timed(binding.PROF_UPDATE, lambda: ctx.update(L, W, B, 5, 1e-9, None))
                rows.append(("update", us, 2.0 * r * d_in * d_out, 4.0 * d_in * d_out))
                for kname, us, fl, by in rows:
                    bound = "mfma" if fl / 2.5e15 > by / 8e12 else "hbm"
                    print("  %-5s %6d %3d | %-9s %9.1f %9.1f %8.0f %7.1f %6s" %
                          (name, N, r, kname, us, fl / us / 1e6, by / us / 1e3, fl / by, bound), flush=True)
                    table.setdefault((name, kname, r), []).append((N, fl / us / 1e6, by / us / 1e3))
            del W, T
        del xs
        torch.cuda.empty_cache()
    # where the measured rates bend: a kernel is taken as bound by memory while its byte rate is the larger fraction of
    # its peak, and by the matrix cores once its flop rate is; the crossover is read from the measured rates, not
    # from the intensities
    print("# measured regime per kernel: fraction of 8000 GB/s / fraction of 2500 TFLOP/s at N = 512, 4096, 16384, 65536; "
          "crossover = first N where the flop fraction is the larger one")
    for (name, kname, r), rows in sorted(table.items()):
        cells, cross = [], None
        for N, tf, gb in rows:
            fb, ff = gb / PEAK_HBM_GBS, tf / PEAK_BF16_TFLOPS
            cells.append("%.2f/%.2f" % (fb, ff))
            if cross is None and ff > fb:
                cross = N
        print("#  %-5s %-9s r=%-2d  %s   crossover: %s" % (name, kname, r, "  ".join(cells),
              ("N = %d" % cross) if cross else "stays memory-bound up to N = 65536"))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--tokens", type=int, default=16384)
    ap.add_argument("--rank", type=int, default=16)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--naive", action="store_true", help="time the perturb-in-place / undo comparator instead")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (known traffic) so counter runs can be scaled")
    ap.add_argument("--sweep", action="store_true", help="rank x tokens sweep on Qwen3-4B shapes (text table)")
    ap.add_argument("--gemm-shapes", action="store_true",
                    help="time the forward GEMM alone on each distinct Qwen3-8B projection shape (one JSON line each)")
    ap.add_argument("--sketch-fusion", action="store_true",
                    help="time the range sketch as a sweep of its own against the one the forward GEMM emits, on the Qwen3-0.6B "
                         "projection shapes (use --tokens 2048)")
    ap.add_argument("--shape", choices=["q", "k", "gate", "down"], default=None, help="with --gemm-shapes: only this shape")
    ap.add_argument("--store-variant", action="store_true", help="with --gemm-shapes: also time the forward that stores a bf16 output and has no loss")
    ap.add_argument("--no-extras", action="store_true",
                    help="only the timed workload and its stage breakdown (for counter-collection runs of the profiler)")
    ap.add_argument("--workload", choices=["qwen3-8b", "qwen3-0.6b", "mlp-stack", "decoder"], default="qwen3-8b",
                    help="layer set: qwen3-8b is the benchmark configuration; qwen3-0.6b (use --tokens 2048 --rank 8) is the "
                         "small launch-bound one; mlp-stack is the 28-block residual stack with LM head and global g; decoder the "
                         "same with full decoder layers (attention)")
    ap.add_argument("--share-bases", action="store_true", help="decoder workload: one basis per distinct input")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives are part of it); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(2)

    if args.sweep:
        sweep(args)
        return
    if args.gemm_shapes:
        gemm_shapes(args)
        return
    if args.sketch_fusion:
        sketch_fusion(args)
        return
    if args.workload == "decoder":
        ctx = binding.Context()
        st = run_decoder(ctx, max(args.steps // 4, 3), max(args.warmup // 2, 1), r=args.rank, share_bases=args.share_bases)
        res = {"metric": "AGZO steps/sec (decoder stack with LM head)", "value": st["value"], "unit": "steps/s", "n_gpus": 1,
               "steps": st["steps"], "warmup": max(args.warmup // 2, 1), "ms_per_step": st["ms_per_step"],
               "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
               "config": {"workload": "28 Qwen3-1.7B-shaped decoder layers (hidden 2048, 16 heads on 8 kv heads, intermediate 6144) + "
                                      "2048x32000 LM head, 16x512 tokens, next-token cross-entropy, r=%d, K=3, global g, %s"
                                      % (args.rank, "shared bases" if args.share_bases else "per-layer bases")},
               "roofline": {"bound": "mfma", "kernel": "forward GEMMs of the step (gemm_bf16_aligned_kernel<1, false, 1>, gemm_bf16_small_kernel, LM head)",
                            "achieved": st["gemm_tflops"], "peak": PEAK_BF16_TFLOPS,
                            "unit": "TFLOP/s", "frac": st["gemm_tflops"] / PEAK_BF16_TFLOPS, "traffic": None},
               "detail": st}
        print(json.dumps(res))
        return
    if args.workload == "mlp-stack":
        ctx = binding.Context()
        st = run_mlp_stack(ctx, max(args.steps // 4, 3), max(args.warmup // 2, 1), r=args.rank)
        res = {"metric": "AGZO steps/sec (MLP stack with LM head)", "value": st["value"], "unit": "steps/s", "n_gpus": 1,
               "steps": st["steps"], "warmup": max(args.warmup // 2, 1), "ms_per_step": st["ms_per_step"],
               "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
               "config": {"workload": "28 SwiGLU-MLP blocks (hidden 2048, intermediate 6144, RMSNorm) + 2048x32000 LM head, "
                                      "16x512 tokens, next-token cross-entropy, r=%d, K=3, global g" % args.rank},
               "roofline": {"bound": "mfma", "kernel": "forward GEMMs of the step (gemm_bf16_aligned_kernel<1, false, 1>, gemm_bf16_small_kernel, LM head)",
                            "achieved": st["gemm_tflops"], "peak": PEAK_BF16_TFLOPS,
                            "unit": "TFLOP/s", "frac": st["gemm_tflops"] / PEAK_BF16_TFLOPS, "traffic": None},
               "detail": st}
        print(json.dumps(res))
        return
    N, r, K = args.tokens, args.rank, 3
    eps, lr = float(np.float32(1e-3)), float(np.float32(1e-4))
    shapes = synth.QWEN3_8B_LAYER if args.workload == "qwen3-8b" else synth.QWEN3_0P6B_LAYER
    layers = build_layer_set(N, shapes, seed=0)
    ctx = binding.Context()
    descs = []
    for name, d_in, d_out, W, X, T in layers:
        descs.append((binding.make_layer(W, X, r), W, X, binding.make_loss(T)))
    out = torch.zeros(len(layers), 4, dtype=torch.float64, device="cuda")
    flags = binding.NAIVE_INPLACE if args.naive else 0

    # Alg. 2 at the level of the layer set (agzo_step_many): every projection's base forward, all bases together (each
    # stage of Alg. 1 one launch for the seven layers), all projections X B in one launch, the perturbed forwards, the
    # scalars, and all updates in one batched sweep.  The in-place comparator runs layer by layer (agzo_step_no_update
    # + one batched update).
    def step_fn(descs_, out_, r_, c=ctx):
        bases = [torch.empty(W.shape[1], r_, dtype=torch.float32, device="cuda") for _, W, _, _ in descs_]
        arr = c.make_step_items([(L, W, X, loss, 0, out_[li], None) for li, (L, W, X, loss) in enumerate(descs_)])

        def run(step, fl):
            if fl & binding.NAIVE_INPLACE:
                for li, (L, W, X, loss) in enumerate(descs_):
                    c.step_no_update(L, W, X, loss, K, eps, 1000 * step + li, fl, out_[li], bases[li])
                c.update_many([(W, bases[li], 1000 * step + li, lr, out_[li, 3:4]) for li, (_, W, _, _) in enumerate(descs_)])
                return
            for li in range(len(descs_)):
                arr[li].seed = 1000 * step + li
            c.step_many_raw(arr, len(descs_), K, eps, lr, fl)
        return run

    run_step = step_fn(descs, out, r)

    def one_step(step, fl=None):
        run_step(step, flags if fl is None else fl)

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)            # 1 GiB read + 1 GiB written by one elementwise kernel
        torch.cuda.synchronize()
        del src, dst
    for s in range(args.warmup):
        one_step(s)
    ctx.check()
    torch.cuda.synchronize()
    # the timed region carries HIP events only around the two kernels whose rooflines are reported (forward GEMM,
    # update); every event costs stream time, so the other stages are timed in a pass of their own below
    ctx.profile_enable((1 << binding.PROF_GEMM) | (1 << binding.PROF_UPDATE))
    # per-step times from events on the library's stream (= torch's current stream), no host synchronisation inside
    step_ev = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    t0 = time.perf_counter()
    for s in range(args.steps):
        step_ev[s].record()
        one_step(args.warmup + s)
    step_ev[args.steps].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    per_step_ms = sorted(step_ev[i].elapsed_time(step_ev[i + 1]) for i in range(args.steps))
    median_ms = per_step_ms[len(per_step_ms) // 2]
    n_gemm, ms_gemm = ctx.profile_read(binding.PROF_GEMM)
    n_upd, ms_upd = ctx.profile_read(binding.PROF_UPDATE)
    try:
        n_clk, gemm_ghz = ctx.profile_clock()
    except binding.AgzoError:                    # telemetry only: never a reason to lose the measurement
        n_clk, gemm_ghz = 0, None
    ctx.profile_enable(False)
    # stage breakdown: two more steps with every kernel class timed (not part of `value`)
    nstage = 2
    ctx.profile_enable(True)
    for s in range(nstage):
        one_step(5_000 + s)
    torch.cuda.synchronize()
    st_gemm = ctx.profile_read(binding.PROF_GEMM)[1] / nstage
    st_upd = ctx.profile_read(binding.PROF_UPDATE)[1] / nstage
    ms_xq = ctx.profile_read(binding.PROF_XQ)[1] / nstage
    ms_xtt = ctx.profile_read(binding.PROF_XTT)[1] / nstage
    ms_qr = ctx.profile_read(binding.PROF_QR)[1] / nstage
    ctx.profile_enable(False)
    ctx.check()
    losses = out.cpu().numpy()
    if not np.isfinite(losses).all():
        print("bench.py: non-finite loss in the timed region", file=sys.stderr)
        sys.exit(1)

    # algorithmic work per launch, averaged over the launches of the timed region
    fwd_flops = sum(2.0 * N * d_in * d_out for _, d_in, d_out in shapes)        # one forward of the layer set
    rank_flops = sum(2.0 * N * r * (d_in + d_out) for _, d_in, d_out in shapes)   # rank-r term (perturbed only)
    gemm_per_step = 3 if not args.naive else 3
    algo_flops_per_launch = (gemm_per_step * fwd_flops + (0 if args.naive else 2 * rank_flops)) / (gemm_per_step * len(shapes))
    gemm_avg_ms = ms_gemm / max(n_gemm, 1)
    gemm_tflops = algo_flops_per_launch / (gemm_avg_ms * 1e-3) / 1e12
    # update: bytes of the timed region / its launches (one batched launch pair per step; the in-place comparator adds
    # three single-matrix sweeps per projection and step: perturb, to the other side, restore)
    upd_bytes_per_step = sum(2.0 * 2 * d_in * d_out + 4.0 * d_in * r for _, d_in, d_out in shapes) * (4 if args.naive else 1)
    upd_bytes_per_launch = upd_bytes_per_step * args.steps / max(n_upd, 1)
    upd_avg_ms = ms_upd / max(n_upd, 1)
    upd_gbs = upd_bytes_per_launch / (upd_avg_ms * 1e-3) / 1e9

    traffic = upd_traffic = None
    tfile = os.path.join(ROOT, "profiles", "gemm_bf16_qwen3_8b_traffic.txt")
    if os.path.exists(tfile) and args.workload == "qwen3-8b" and N == 16384 and r == 16:
        for line in open(tfile):
            if line.startswith("traffic_bytes_per_launch"):
                traffic = float(line.split()[1])
            if line.startswith("update_traffic_bytes_per_launch") and not args.naive:
                upd_traffic = float(line.split()[1])

    res = {
        "metric": "AGZO steps/sec per layer set (Qwen3-8B layer projections)",
        "value": 1e3 / median_ms, "unit": "steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": median_ms, "ms_per_step_mean_wall": 1e3 * dt / args.steps,
        "ms_per_step_min_max": [per_step_ms[0], per_step_ms[-1]], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": args.workload + " layer projections (q,k,v,o,gate,up,down), N=%d tokens, r=%d, K=%d, "
                               "bf16 weights/activations/targets, MSE loss, %s" % (N, r, K, "naive in-place comparator" if args.naive else "factored perturbed forward"),
                   "tokens": N, "rank": r, "power_steps": K, "eps": eps, "lr": lr},
        "roofline": {"bound": "mfma", "kernel": ("gemm_bf16_aligned_kernel<0, false, 1>" if args.workload == "qwen3-8b" and N % 256 == 0 and not args.naive
                                                  else "forward GEMM (gemm_bf16_aligned / gemm_bf16_small / gemm_bf16 kernels, by shape)"),
                     "achieved": gemm_tflops, "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": gemm_tflops / PEAK_BF16_TFLOPS, "traffic": traffic,
                     "traffic_source": "profiles/gemm_bf16_qwen3_8b_traffic.txt (two rocprofv3 --pmc runs of this command, scaled by a "
                                       "plain copy; counters cannot be read from inside this process)",
                     "launches": n_gemm, "avg_ms": gemm_avg_ms,
                     "shader_clock_ghz": gemm_ghz, "clock_note": "mean shader clock over the first workgroup of each of "
                     "these launches (in-kernel cycle counter / constant-rate counter); the peak assumes 2.4 GHz"},
        "roofline_update": {"bound": "hbm", "kernel": "update_prep_many_kernel + update_mfma_many_kernel (the layer set's matrices in one launch pair)", "achieved": upd_gbs, "peak": PEAK_HBM_GBS,
                            "unit": "GB/s", "frac": upd_gbs / PEAK_HBM_GBS, "traffic": upd_traffic,
                            "algorithmic_bytes": upd_bytes_per_launch, "launches": n_upd, "avg_ms": upd_avg_ms},
        "stage_ms_per_step": {"gemm": st_gemm, "update": st_upd, "xq": ms_xq, "xtt": ms_xtt, "qr": ms_qr,
                              "note": "from %d extra steps with every kernel class timed" % nstage},
    }
    if not args.no_extras:
        # the single-matrix update (agzo_update) per projection shape: prep + sweep, bytes = W read + written + the basis;
        # the small k/v matrices cannot fill launches of their own, which is what the batched call above avoids
        by_shape = {}
        Bu = {}
        for (name, d_in, d_out, W, X, T), (L, _, _, _) in zip(layers, descs):
            if d_in not in Bu:
                Bu[d_in] = torch.empty(d_in, r, dtype=torch.float32, device="cuda").normal_()
            ctx.update(L, W, Bu[d_in], 7, 1e-9, None)
            ctx.profile_enable(1 << binding.PROF_UPDATE)
            for _ in range(5):
                ctx.update(L, W, Bu[d_in], 7, 1e-9, None)
            n_u, ms_u = ctx.profile_read(binding.PROF_UPDATE)
            ctx.profile_enable(False)
            gbs = (4.0 * d_in * d_out + 4.0 * d_in * r) / (ms_u / max(n_u, 1) * 1e-3) / 1e9
            by_shape["%s %dx%d" % (name, d_out, d_in)] = {"us": 1e3 * ms_u / max(n_u, 1), "GB/s": gbs, "frac": gbs / PEAK_HBM_GBS}
        res["roofline_update"]["by_shape"] = by_shape
    if not args.naive and not args.no_extras:
        # the same steps with f0, f+ and f- evaluated from one pass over X and W (AGZO_SHARED_FORWARD):
        # identical results up to rounding, one GEMM main loop per projection instead of three
        for s in range(args.warmup):
            one_step(10_000 + s, binding.SHARED_FORWARD)
        torch.cuda.synchronize()
        ctx.profile_enable(1 << binding.PROF_GEMM)
        t1 = time.perf_counter()
        for s in range(args.steps):
            one_step(20_000 + s, binding.SHARED_FORWARD)
        torch.cuda.synchronize()
        dt1 = time.perf_counter() - t1
        n_g1, ms_g1 = ctx.profile_read(binding.PROF_GEMM)
        ctx.profile_enable(False)
        ctx.check()
        flops1 = (fwd_flops + 2 * rank_flops) / len(shapes)
        res["shared_forward"] = {"value": args.steps / dt1, "unit": "steps/s", "ms_per_step": 1e3 * dt1 / args.steps,
                                 "gemm_launches": n_g1, "gemm_avg_ms": ms_g1 / max(n_g1, 1),
                                 "gemm_tflops": flops1 / (ms_g1 / max(n_g1, 1) * 1e-3) / 1e12,
                                 "note": "f0, f+, f- from one pass over X and W per projection (single-layer problems only)"}
        # the forward GEMM storing a bf16 output instead of evaluating the loss: the kernel a layer inside a model takes,
        # and what the vendor library's GEMM does
        outs = [torch.empty(N, W.shape[0], dtype=torch.bfloat16, device="cuda") for (L, W, X, loss) in descs]
        lys = [binding.make_layer(W, X, r, Y=Y) for (L, W, X, loss), Y in zip(descs, outs)]
        for (L, W, X, loss), Ly, Y in zip(descs, lys, outs):
            ctx.layer_forward_sketch(Ly, W, X, Y, binding.SKETCH_NONE, None, 1, None, None, None)
        torch.cuda.synchronize()
        ctx.profile_enable(1 << binding.PROF_GEMM)
        for _ in range(3):
            for (L, W, X, loss), Ly, Y in zip(descs, lys, outs):
                ctx.layer_forward_sketch(Ly, W, X, Y, binding.SKETCH_NONE, None, 1, None, None, None)
        torch.cuda.synchronize()
        n_g2, ms_g2 = ctx.profile_read(binding.PROF_GEMM)
        ctx.profile_enable(False)
        del outs, lys
        res["forward_only"] = {"gemm_launches": n_g2, "gemm_avg_ms": ms_g2 / max(n_g2, 1),
                               "gemm_tflops": fwd_flops / len(shapes) / (ms_g2 / max(n_g2, 1) * 1e-3) / 1e12,
                               "note": "the same kernel storing a bf16 output instead of the fused loss (no target read)"}
        # the same step composed from the per-layer calls, with one basis per distinct input: q/k/v read the same
        # activations, so do gate/up, and Alg. 1 depends on the activations only (the paper extracts per layer; the
        # layers' Gaussian factors stay independent)
        Bs = {}

        def composed_step(step):
            Bs.clear()
            for li, (L, W, X, loss) in enumerate(descs):
                seed = 1000 * step + li
                ctx.layer_forward_sketch(L, W, X, None, binding.SKETCH_NONE, None, seed, None, loss, out[li, 0:1])
                key = X.data_ptr()
                if key not in Bs:
                    Bs[key] = torch.empty(X.shape[1], r, dtype=torch.float32, device="cuda")
                    ctx.basis(L, X, K, seed, None, 0, Bs[key])
                ctx.perturbed_forward(L, W, X, Bs[key], seed, eps, None, loss, out[li, 1:2])
                ctx.perturbed_forward(L, W, X, Bs[key], seed, -eps, None, loss, out[li, 2:3])
                ctx.two_point(out[li], eps)
            ctx.update_many([(W, Bs[X.data_ptr()], 1000 * step + li, lr, out[li, 3:4]) for li, (_, W, X, _) in enumerate(descs)])

        composed_step(40_000)
        torch.cuda.synchronize()
        t4 = time.perf_counter()
        for s in range(nsteps_c := max(2, args.steps // 2)):
            composed_step(40_001 + s)
        torch.cuda.synchronize()
        dt4 = time.perf_counter() - t4
        ctx.check()
        res["shared_basis"] = {"value": nsteps_c / dt4, "unit": "steps/s", "ms_per_step": 1e3 * dt4 / nsteps_c, "steps": nsteps_c,
                               "bases_per_step": len(Bs),
                               "note": "composed from the per-layer calls; layers that read the same activations share one "
                                       "extraction (4 instead of 7 per step)"}
        # the paper's literal schedule as a comparator: perturb W in place, plain forward, undo (Alg. 2)
        nsteps = max(2, args.steps // 2)
        one_step(30_000, binding.NAIVE_INPLACE)
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        for s in range(nsteps):
            one_step(30_001 + s, binding.NAIVE_INPLACE)
        torch.cuda.synchronize()
        dt2 = time.perf_counter() - t2
        ctx.check()
        res["naive_inplace"] = {"value": nsteps / dt2, "unit": "steps/s", "ms_per_step": 1e3 * dt2 / nsteps, "steps": nsteps,
                                "note": "perturb-in-place / undo comparator (4 extra sweeps of W per step; in bf16 a different "
                                        "computation: the perturbation is rounded into the weights)"}
        # the literal one-sided form of Eq. 10 / Alg. 2: the base forward and one perturbed forward per projection
        one_step(35_000, binding.ONE_SIDED)
        torch.cuda.synchronize()
        t7 = time.perf_counter()
        for s in range(nsteps):
            one_step(35_001 + s, binding.ONE_SIDED)
        torch.cuda.synchronize()
        dt7 = time.perf_counter() - t7
        ctx.check()
        res["one_sided"] = {"value": nsteps / dt7, "unit": "steps/s", "ms_per_step": 1e3 * dt7 / nsteps, "steps": nsteps,
                            "note": "g = (f+ - f0) / eps as printed in Eq. 10: two forwards per projection instead of three"}
        # the dense branch of Eq. 7 applied to the same matrices (the zeroth-order baseline the paper compares with): no
        # extraction, two plain forwards, four in-place sweeps that regenerate d_out x d_in normals each
        def dense_step(step):
            for li, (L, W, X, loss) in enumerate(descs):
                seed = 1000 * step + li
                ctx.dense_perturb(W, seed, eps)
                ctx.layer_forward_sketch(L, W, X, None, binding.SKETCH_NONE, None, seed, None, loss, out[li, 1:2])
                ctx.dense_perturb(W, seed, -2.0 * eps)
                ctx.layer_forward_sketch(L, W, X, None, binding.SKETCH_NONE, None, seed, None, loss, out[li, 2:3])
                ctx.dense_perturb(W, seed, eps)
                ctx.two_point(out[li], eps)
                ctx.dense_perturb(W, seed, -lr, out[li, 3:4])

        dense_step(50_000)
        torch.cuda.synchronize()
        t5 = time.perf_counter()
        for s in range(nsteps):
            dense_step(50_001 + s)
        torch.cuda.synchronize()
        dt5 = time.perf_counter() - t5
        ctx.check()
        res["dense_gaussian"] = {"value": nsteps / dt5, "unit": "steps/s", "ms_per_step": 1e3 * dt5 / nsteps, "steps": nsteps,
                                 "agzo_over_dense": (1e3 / median_ms) / (nsteps / dt5),
                                 "agzo_one_sided_over_dense": (nsteps / dt7) / (nsteps / dt5),
                                 "note": "Eq. 7's dense branch on the same matrices, composed from agzo_dense_perturb, the plain "
                                         "forward and agzo_two_point: two forwards and four generator-bound sweeps per projection"}
        # the data-independent low-rank estimator of the paper's Sec. 2 on the same kernels: a Gaussian V [d_in][r] in the
        # place of the activation basis (no extraction, no base forward), the estimate scaled by 1 / r
        Vs = [torch.empty(W.shape[1], r, dtype=torch.float32, device="cuda") for _, W, _, _ in descs]

        def lowrank_step(step):
            for li, (L, W, X, loss) in enumerate(descs):
                seed = 1000 * step + li
                ctx.fill_normal(Vs[li], seed, binding.TAG_Q0)
                ctx.perturbed_forward(L, W, X, Vs[li], seed, eps, None, loss, out[li, 1:2])
                ctx.perturbed_forward(L, W, X, Vs[li], seed, -eps, None, loss, out[li, 2:3])
                ctx.two_point(out[li], eps)
            ctx.update_many([(W, Vs[li], 1000 * step + li, lr / r, out[li, 3:4]) for li, (_, W, _, _) in enumerate(descs)])

        lowrank_step(60_000)
        torch.cuda.synchronize()
        t6 = time.perf_counter()
        for s in range(nsteps):
            lowrank_step(60_001 + s)
        torch.cuda.synchronize()
        dt6 = time.perf_counter() - t6
        ctx.check()
        res["lowrank_gaussian"] = {"value": nsteps / dt6, "unit": "steps/s", "ms_per_step": 1e3 * dt6 / nsteps, "steps": nsteps,
                                   "agzo_over_lowrank": (1e3 / median_ms) / (nsteps / dt6),
                                   "agzo_one_sided_over_lowrank": (nsteps / dt7) / (nsteps / dt6),
                                   "note": "perturbation U V^T with Gaussian factors (Sec. 2), two perturbed forwards and the batched "
                                           "rank-r update; composed from agzo_fill_normal, agzo_perturbed_forward, agzo_two_point, "
                                           "agzo_update_many"}
    # the standalone generator fill (the form in which the Gaussian factor is checked bit for bit): 2^28 normals
    gbuf = torch.empty(1 << 24, 16, dtype=torch.float32, device="cuda")
    ctx.fill_normal(gbuf, 1, binding.TAG_G)
    torch.cuda.synchronize()
    ctx.profile_enable(1 << binding.PROF_FILL)
    for i in range(5):
        ctx.fill_normal(gbuf, 2 + i, binding.TAG_G)
    n_fill, ms_fill = ctx.profile_read(binding.PROF_FILL)
    ctx.profile_enable(False)
    fill_gbs = gbuf.numel() * 4.0 / (ms_fill / max(n_fill, 1) * 1e-3) / 1e9
    res["roofline_generator"] = {"bound": "hbm", "kernel": "fill_normal_kernel", "achieved": fill_gbs, "peak": PEAK_HBM_GBS,
                                 "unit": "GB/s", "frac": fill_gbs / PEAK_HBM_GBS, "launches": n_fill,
                                 "normals_per_s": fill_gbs * 1e9 / 4.0,
                                 "note": "4 bytes written per value; 68 vector instructions per value (Philox4x32-10 + "
                                         "Box-Muller; profiles/generator_valu_instructions.txt): bound by its arithmetic"}
    # the dense Gaussian sweep of Eq. 7's other branch on a bf16 block of the same size (read + write 2 bytes each)
    theta = gbuf.view(torch.bfloat16)[:, :16]
    theta.zero_()
    ctx.dense_perturb(theta, 1, 1e-3)
    torch.cuda.synchronize()
    ctx.profile_enable(1 << binding.PROF_FILL)
    for i in range(5):
        ctx.dense_perturb(theta, 2 + i, 1e-3)
    n_dn, ms_dn = ctx.profile_read(binding.PROF_FILL)
    ctx.profile_enable(False)
    dn_rate = theta.numel() / (ms_dn / max(n_dn, 1) * 1e-3)
    res["roofline_generator"]["dense_sweep_bf16"] = {"kernel": "dense_axpy_kernel", "achieved": 4.0 * dn_rate / 1e9, "unit": "GB/s",
                                                     "frac": 4.0 * dn_rate / 1e9 / PEAK_HBM_GBS, "normals_per_s": dn_rate,
                                                     "launches": n_dn}
    del gbuf, theta
    if args.workload == "qwen3-8b" and not args.naive and not args.no_extras:
        # the small, launch-bound configuration next to the headline one: Qwen3-0.6B layer set, N = 2048, r = 8
        del layers, descs
        torch.cuda.empty_cache()
        s_layers = build_layer_set(2048, synth.QWEN3_0P6B_LAYER, seed=50)
        s_descs = [(binding.make_layer(W, X, 8), W, X, binding.make_loss(T)) for _, _, _, W, X, T in s_layers]
        s_out = torch.zeros(len(s_layers), 4, dtype=torch.float64, device="cuda")

        small_run = step_fn(s_descs, s_out, 8)

        def small_step(step):
            small_run(step, 0)

        for s_ in range(5):
            small_step(s_)
        torch.cuda.synchronize()
        n_small = 50
        t3 = time.perf_counter()
        for s_ in range(n_small):
            small_step(10 + s_)
        torch.cuda.synchronize()
        dt3 = time.perf_counter() - t3
        ctx.profile_enable(True)
        for s_ in range(2):
            small_step(100 + s_)
        torch.cuda.synchronize()
        st = {k: ctx.profile_read(v)[1] / 2 for k, v in (("gemm", binding.PROF_GEMM), ("update", binding.PROF_UPDATE),
                                                        ("xq", binding.PROF_XQ), ("xtt", binding.PROF_XTT), ("qr", binding.PROF_QR))}
        ctx.profile_enable(False)
        ctx.check()
        res["qwen3_0p6b_layer_set"] = {"value": n_small / dt3, "unit": "steps/s", "ms_per_step": 1e3 * dt3 / n_small,
                                       "tokens": 2048, "rank": 8, "steps": n_small, "stage_ms_per_step": st,
                                       "note": "launch- and latency-bound: 7 projections of 1-3 M parameters each"}
        # the same step recorded once in a HIP graph on a stream of its own and replayed (the calls enqueue kernels only);
        # the seeds are part of the recorded arguments, so every replay repeats one step's seeds: the work is the same
        try:
            side = torch.cuda.Stream()
            gctx = binding.Context(stream=side)
            torch.cuda.synchronize()
            graph_run = step_fn(s_descs, s_out, 8, gctx)
            with torch.cuda.stream(side):
                for s_ in range(3):
                    graph_run(200 + s_, 0)
                gctx.check()
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph, stream=side):
                    graph_run(300, 0)
            torch.cuda.synchronize()
            for s_ in range(5):
                graph.replay()
            torch.cuda.synchronize()
            t8 = time.perf_counter()
            for s_ in range(n_small):
                graph.replay()
            torch.cuda.synchronize()
            dt8 = time.perf_counter() - t8
            with torch.cuda.stream(side):
                gctx.check()
            res["qwen3_0p6b_layer_set"]["graph_replay"] = {"value": n_small / dt8, "unit": "steps/s",
                                                           "ms_per_step": 1e3 * dt8 / n_small, "steps": n_small}
            del graph
            gctx.close()
        except (binding.AgzoError, RuntimeError) as e:        # an extra: never a reason to lose the measurement
            res["qwen3_0p6b_layer_set"]["graph_replay"] = {"error": str(e)[:200]}
        del s_layers, s_descs
    # ceilings of this machine that the HBM figures can be read against: a plain device copy and a read-only sweep of 1 GiB
    # (torch's elementwise copy and reduction kernels, 10 launches each, HIP events on the current stream)
    try:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        def timed_ms(fn, reps=10):
            fn()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(reps):
                fn()
            b.record()
            torch.cuda.synchronize()
            return a.elapsed_time(b) / reps
        gib = float(1 << 30)
        res["box_ceilings"] = {"copy_GBps": 2.0 * gib / (timed_ms(lambda: dst.copy_(src)) * 1e-3) / 1e9,
                               "read_only_GBps": gib / (timed_ms(lambda: src.sum()) * 1e-3) / 1e9,
                               "note": "1 GiB fp32: copy counts bytes read + written, the read-only sweep is a sum reduction"}
        del src, dst
    except RuntimeError as e:
        res["box_ceilings"] = {"error": str(e)[:200]}
    if args.workload == "qwen3-8b" and not args.naive and not args.no_extras:
        # Alg. 2 over a model: the 28-block MLP stack with LM head at its full size (a workload of its own with
        # --workload mlp-stack)
        try:
            torch.cuda.empty_cache()
            res["mlp_stack"] = run_mlp_stack(ctx, 3, 1)
        except (binding.AgzoError, RuntimeError) as e:
            res["mlp_stack"] = {"error": str(e)[:300]}
        try:
            torch.cuda.empty_cache()
            res["decoder"] = run_decoder(ctx, 3, 1)
            torch.cuda.empty_cache()
            res["decoder_shared_bases"] = run_decoder(ctx, 3, 1, share_bases=True)
        except (binding.AgzoError, RuntimeError) as e:
            res["decoder"] = {"error": str(e)[:300]}
        torch.cuda.empty_cache()
    # yardstick for the MFMA fraction: a register-only MFMA loop (no LDS, no memory traffic) on this device, with
    # operand bits that never toggle (zeros) and with N(0,1) bf16 operands like the workload's
    gen = torch.Generator(device="cuda")
    gen.manual_seed(7)
    probes = {}
    try:
        for name, ops in (("zero_operands", torch.zeros(16384, dtype=torch.bfloat16, device="cuda")),
                          ("randn_operands", torch.randn(16384, device="cuda", generator=gen).to(torch.bfloat16))):
            for _ in range(6):                      # a few launches so that the clock settles (about 6 ms each)
                tf, ghz = ctx.probe_mfma(ops, 8, 3000)
            probes[name] = {"tflops": tf, "clock_ghz": ghz}
            if name == "randn_operands":            # the same flop count from 16x16x32 instructions
                for _ in range(6):
                    tf, ghz = ctx.probe_mfma(ops, 9, 3000)
                probes["randn_operands_16x16x32"] = {"tflops": tf, "clock_ghz": ghz}
        res["roofline"]["sustained_mfma"] = dict(probes, note="register-only matrix-instruction loop, 4 waves per CU, issued back to back: the rate this "
                                                 "device holds under its power limit (v_mfma_f32_32x32x16_bf16; _16x16x32: the instruction the GEMM uses)")
        res["roofline"]["frac_of_sustained"] = gemm_tflops / probes["randn_operands_16x16x32"]["tflops"]
    except binding.AgzoError as e:                  # a yardstick, not part of the measurement
        res["roofline"]["sustained_mfma"] = {"error": str(e)}
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(N, r, K, eps, lr, shapes)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
