"""GPU parity at the benchmark's full sizes (Qwen3-8B layer shapes, N = 16384, r = 16, K = 3), in the
launch configuration bench.py times (agzo_step through the C ABI, same input recipe).

k and q projections: the whole oracle step is affordable, so losses, g and every entry of the updated W
are compared.  down (d_in = 12288) and gate (d_out = 12288): the oracle's extraction is cheap (tall-skinny)
and is compared in full; outputs are compared on sampled rows, the updated W on sampled rows with the
GPU's own g (g itself is checked through the losses on the same sampled rows being consistent).
"""
import numpy as np
import pytest
import torch

from oracle import agzo as oagzo
from paper_2601_17261_amd import binding, synth

pytestmark = pytest.mark.gpu

N, R, K = 16384, 16, 3
EPS = float(np.float32(1e-3))
LR = float(np.float32(1e-4))


def rel(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


@pytest.fixture(scope="module")
def ctx():
    c = binding.Context()
    yield c
    c.close()


@pytest.fixture(scope="module")
def x4096():
    return synth.device_powerlaw_x(101, N, 4096)


# batched: the calls bench.py times (the step up to g, then the update through agzo_update_many); otherwise agzo_step
@pytest.mark.parametrize("name,d_out,target_dtype,R,batched", [("k", 1024, torch.bfloat16, 16, True),
                                                               ("k", 1024, torch.float32, 16, False),
                                                               ("q", 4096, torch.bfloat16, 16, True),
                                                               ("k", 1024, torch.bfloat16, 64, False)])   # the largest rank
def test_full_step_against_full_oracle(ctx, x4096, name, d_out, target_dtype, R, batched):
    X = x4096
    W, T = synth.device_weights_and_target(7 + d_out, X, d_out, target_dtype=target_dtype)
    W0 = host(W)
    Xh, Th = host(X), host(T)
    out = torch.zeros(4, dtype=torch.float64, device="cuda")
    seed = 4321
    if batched:
        B = torch.empty(X.shape[1], R, dtype=torch.float32, device="cuda")
        ctx.step_no_update(binding.make_layer(W, X, R), W, X, binding.make_loss(T), K, EPS, seed, 0, out, B)
        ctx.update_many([(W, B, seed, LR, out[3:4])])
    else:
        ctx.step(binding.make_layer(W, X, R), W, X, binding.make_loss(T), K, EPS, LR, seed, 0, out)
    ctx.check()
    o = oagzo.agzo_step(W0, Xh, Th, R, K, EPS, LR, seed, storage="bf16")
    got = out.cpu().numpy()
    assert abs(got[0] - o["L0"]) < 1e-5 * o["L0"]
    assert abs(got[1] - o["Lp"]) < 1e-5 * o["Lp"]
    assert abs(got[2] - o["Lm"]) < 1e-5 * o["Lm"]
    assert abs(got[3] - o["g"]) < 2e-2 * abs(o["g"]), (got[3], o["g"])
    Wn = host(W)
    assert rel(Wn, o["W_new"]) < 2e-2          # spec bar
    assert rel(Wn, o["W_new"]) < 3e-3          # what the arithmetic supports
    # entry by entry: equal, or one rounding step apart where the fp32 and fp64 evaluations of
    # W - lr g Z straddle a bf16 boundary (g itself differs in its last digits); more than one
    # step only for weights so small that the update term dominates them
    ulp = np.abs(o["W_new"]) * 2.0 ** -7
    diff = np.abs(Wn - o["W_new"])
    assert np.mean(diff > 0) < 2e-2
    assert np.mean(diff > ulp + 1e-30) < 1e-4


@pytest.mark.parametrize("name,d_in,d_out", [("down", 12288, 4096), ("gate", 4096, 12288)])
def test_wide_projections_sampled(ctx, x4096, name, d_in, d_out):
    X = x4096 if d_in == 4096 else synth.device_powerlaw_x(202, N, d_in)
    W, T = synth.device_weights_and_target(11 + d_out, X, d_out)
    W0 = host(W)
    Xh = host(X)
    seed = 777
    L = binding.make_layer(W, X, R)
    # extraction in full
    B = torch.empty(d_in, R, dtype=torch.float32, device="cuda")
    ctx.basis(L, X, K, seed, None, 0, B)
    ctx.check()
    ext = oagzo.subspace_extract(Xh, R, K, seed)
    Bg, Bo = host(B), ext["B"]
    assert np.linalg.norm(Bg.T @ Bg - np.eye(R)) < 1e-5
    assert np.linalg.norm(Bg @ (Bg.T @ Bo) - Bo) / np.sqrt(R) < 5e-3     # same subspace
    # outputs on sampled token rows
    rng = np.random.default_rng(5)
    rows = np.sort(rng.choice(N, size=24, replace=False))
    Y = torch.empty(N, d_out, dtype=torch.float32, device="cuda")
    Ly = binding.make_layer(W, X, R, Y=Y)
    Bo32 = torch.from_numpy(Bo.astype(np.float32)).cuda()
    Z, _G = oagzo.perturbation(Bo.astype(np.float32).astype(np.float64), seed, d_out)
    Y0 = Xh[rows] @ W0.T
    for sign in (0.0, +1.0, -1.0):
        if sign == 0.0:
            ctx.layer_forward_sketch(Ly, W, X, Y, binding.SKETCH_NONE, None, seed, None, None, None)
        else:
            ctx.perturbed_forward(Ly, W, X, Bo32, seed, sign * EPS, Y, None, None)
        want = Xh[rows] @ (W0 + sign * EPS * Z).T
        got = host(Y[torch.from_numpy(rows).cuda()])
        assert rel(got, want) < 3e-5
        if sign != 0.0:
            assert rel(got - Y0, want - Y0) < 5e-3
    # whole step: losses against the GPU's own stored outputs is circular, so check the update on sampled
    # rows of W with the step's g, and g's sign/size against the oracle's directional derivative
    out = torch.zeros(4, dtype=torch.float64, device="cuda")
    ctx.step(L, W, X, binding.make_loss(T), K, EPS, LR, seed, 0, out)
    ctx.check()
    got = out.cpu().numpy()
    Th = host(T)
    A = Xh @ W0.T - Th                                   # full residual (one fp64 forward)
    assert abs(got[0] - np.mean(A * A)) < 1e-5 * np.mean(A * A)
    Zg, _ = oagzo.perturbation(ext["B"], seed, d_out)
    dd = (2.0 / A.size) * np.sum((A.T @ Xh) * Zg)          # <grad, Z> = exact central difference on a quadratic
    assert abs(got[3] - dd) < 2e-2 * abs(dd), (got[3], dd)
    wrows = np.sort(rng.choice(d_out, size=64, replace=False))
    want = oagzo.round_bf16(W0[wrows] - LR * got[3] * Zg[wrows])
    assert rel(host(W)[wrows], want) < 3e-3


def test_layer_set_updated_in_one_call_at_full_size(ctx):
    """The seven matrices of the benchmark's layer set through agzo_update_many: every matrix bit-identical to its own
    agzo_update, and sampled rows against the oracle's W - lr g G B^T."""
    rng = np.random.default_rng(3)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(11)
    items, checks = [], []
    for li, (name, d_in, d_out) in enumerate(synth.QWEN3_8B_LAYER):
        W = (0.02 * torch.randn(d_out, d_in, device="cuda", generator=gen)).to(torch.bfloat16)
        Bh, _ = np.linalg.qr(rng.standard_normal((d_in, R)))
        B = torch.from_numpy(Bh.astype(np.float32)).cuda()
        g = torch.tensor([(-1.0) ** li * (0.3 + li)], dtype=torch.float64, device="cuda")
        items.append((W, B, 900 + li, 1e-2, g))
        checks.append((W.clone(), Bh.astype(np.float32).astype(np.float64), g.item()))
    ctx.update_many(items)
    ctx.check()
    for (W, B, seed, lr, g), (W0, Bh, gv) in zip(items, checks):
        d_out, d_in = W0.shape
        wrows = np.sort(rng.choice(d_out, size=48, replace=False))
        idx = torch.from_numpy(wrows).cuda()
        G = oagzo.gaussian_factor(seed, d_out, R)[wrows]
        want = oagzo.round_bf16(host(W0[idx]) - np.float64(np.float32(lr)) * gv * (G @ Bh.T))
        assert rel(host(W[idx]), want) < 3e-3
        assert rel(host(W[idx]) - host(W0[idx]), want - host(W0[idx])) < 5e-3
        single = W0                                     # update the untouched copy with the single-matrix call
        Ls = binding.AgzoLayer()
        Ls.n_tokens, Ls.d_in, Ls.d_out, Ls.r = 0, d_in, d_out, R
        Ls.dtype = Ls.y_dtype = binding.BF16
        Ls.tiling, Ls.ldw, Ls.ldx, Ls.ldy = 0, d_in, d_in, d_out
        ctx.update(Ls, single, B, seed, lr, g)
        assert torch.equal(single, W)
    ctx.check()


@pytest.mark.parametrize("d_out,d_in", [(16384 + 96, 8192), (32768 + 40, 16384)])
def test_very_large_matrix_update_walks_several_row_groups_per_workgroup(ctx, d_out, d_in):
    """Matrices large enough that a workgroup of the sweep takes two (first shape) or four (second) groups of 128 rows
    in turn, with a ragged last group: sampled rows against the oracle, and the batched call against the single one."""
    gen = torch.Generator(device="cuda")
    gen.manual_seed(d_out)
    W = (0.02 * torch.randn(d_out, d_in, device="cuda", generator=gen)).to(torch.bfloat16)
    W0 = W.clone()
    rng = np.random.default_rng(d_in)
    Bh, _ = np.linalg.qr(rng.standard_normal((d_in, R)))
    Bh = Bh.astype(np.float32)
    B = torch.from_numpy(Bh).cuda()
    g = torch.tensor([-1.3], dtype=torch.float64, device="cuda")
    seed, lr = 31, 1e-2
    L = binding.AgzoLayer()
    L.n_tokens, L.d_in, L.d_out, L.r = 0, d_in, d_out, R
    L.dtype = L.y_dtype = binding.BF16
    L.tiling, L.ldw, L.ldx, L.ldy = 0, d_in, d_in, d_out
    ctx.update(L, W, B, seed, lr, g)
    ctx.check()
    # the first and last rows, the rows around every 128-row group boundary of the first workgroups, and a random sample
    rows = np.unique(np.concatenate([np.arange(0, 4), np.arange(d_out - 4, d_out), np.arange(124, 132), np.arange(508, 516),
                                     np.arange(1020, 1028), rng.choice(d_out, size=48, replace=False)]))
    idx = torch.from_numpy(rows).cuda()
    G = oagzo.gaussian_factor(seed, d_out, R)[rows]
    w0 = host(W0[idx])
    want = oagzo.round_bf16(w0 - np.float64(np.float32(lr)) * (-1.3) * (G @ Bh.astype(np.float64).T))
    assert rel(host(W[idx]), want) < 3e-3
    assert rel(host(W[idx]) - w0, want - w0) < 5e-3
    changed = (W != W0).float().mean().item()
    assert changed > 0.5                                   # every part of the matrix was swept
    ctx.update_many([(W0, B, seed, lr, g)])                # the untouched copy through the batched call
    ctx.check()
    assert torch.equal(W0, W)


def test_bench_line_has_the_contract_fields():
    """bench.py in its default shape (fewer steps, no CPU baseline): one JSON line with the fields the harness reads,
    a roofline whose fraction is achieved / peak, and a finite positive throughput."""
    import json
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--steps", "2", "--warmup", "1", "--no-cpu-baseline"],
                         capture_output=True, text=True, timeout=600, cwd=root)
    assert res.returncode == 0, res.stderr[-2000:]
    lines = [l for l in res.stdout.splitlines() if l.startswith("{")]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
              "vs_baseline", "dtype", "data", "config", "roofline"):
        assert k in d, k
    assert d["n_gpus"] == 1 and d["steps"] == 2 and d["warmup"] == 1 and d["higher_is_better"] is True
    assert d["vs_baseline"] is None and d["data"] == "synthetic" and d["dtype"] == "bf16"
    assert "workload" in d["config"] and "model" not in d["config"]
    assert np.isfinite(d["value"]) and d["value"] > 0
    assert abs(d["value"] * d["ms_per_step"] - 1e3) < 1e-6 * 1e3
    rf = d["roofline"]
    for k in ("bound", "achieved", "peak", "unit", "frac", "traffic"):
        assert k in rf, k
    assert rf["bound"] == "mfma" and rf["unit"] == "TFLOP/s" and rf["peak"] == 2500.0
    assert abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-12
    res2 = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                          timeout=120, cwd=root)
    assert res2.returncode != 0 and "one GPU" in res2.stderr


@pytest.mark.parametrize("flags", [0, binding.SHARED_FORWARD])
def test_lm_head_cross_entropy_at_full_size(ctx, flags):
    """The output projection of the MLP-stack workload at its full size: 16 x 512 tokens, hidden 2048, vocabulary
    32000, token cross-entropy with the last position of every sequence ignored (32 x 125 GEMM tiles, the logits are
    never stored).  The oracle's three forwards are a teraflop each in fp64, which the host does in seconds."""
    n_seq, seq, hidden, vocab = 16, 512, 2048, 32000
    n = n_seq * seq
    rng = np.random.default_rng(77)
    X = synth.x_rmsnorm_gaussian(rng, n, hidden, storage="bf16")
    W = synth.weights(rng, vocab, hidden, storage="bf16")
    ids = rng.integers(0, vocab, size=(n_seq, seq))
    tgt = np.full((n_seq, seq), -1, dtype=np.int32)
    tgt[:, :-1] = ids[:, 1:]
    tgt = tgt.reshape(-1)
    Wd = torch.from_numpy(W).to("cuda", torch.bfloat16)
    Xd = torch.from_numpy(X).to("cuda", torch.bfloat16)
    Td = torch.from_numpy(tgt).cuda()
    out = torch.zeros(4, dtype=torch.float64, device="cuda")
    seed, lr = 2024, float(np.float32(1e-2))
    ctx.step(binding.make_layer(Wd, Xd, R), Wd, Xd, binding.make_loss(Td, kind=binding.LOSS_CE), K, EPS, lr, seed, flags, out)
    ctx.check()
    got = out.cpu().numpy()
    o = oagzo.agzo_step(W, X, tgt, R, K, EPS, lr, seed, loss="ce", storage="bf16")
    assert (tgt >= 0).sum() == n_seq * (seq - 1)
    assert abs(got[0] - o["L0"]) < 2e-6 * o["L0"]
    assert abs(got[1] - o["Lp"]) < 2e-6 * o["Lp"]
    assert abs(got[2] - o["Lm"]) < 2e-6 * o["Lm"]
    assert abs(got[3] - o["g"]) < 2e-2 * abs(o["g"]) + 1e-9, (got[3], o["g"])
    Wn = host(Wd)
    assert rel(Wn, o["W_new"]) < 3e-3
    assert np.mean(Wn != o["W_new"]) < 2e-2
    assert np.mean(Wn != W) > 0.01                       # the step moved the weights
