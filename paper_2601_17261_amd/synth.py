"""Seeded synthetic inputs shaped like the paper's workloads.

This module only *makes inputs* (weights, activations, targets) and holds none
of the method's arithmetic; both the CPU oracle's tests and the HIP path's
tests draw their inputs from here, so the two sides see identical numbers.

The paper fine-tunes Qwen3 / Pangu models on public NLP datasets
(App. B.1-B.2); neither weights nor data are used here.  What is kept is the
layer shapes and the spectral character the paper reports for activations
(Sec. 3.2, Fig. 1c: fast singular-value decay, a few dominant directions).

All functions return float32 numpy arrays whose values are exactly
representable in the stated storage type (fp32, or bf16 after rounding).
"""
import numpy as np
import torch

QWEN3_0P6B_LAYER = [("q", 1024, 2048), ("k", 1024, 1024), ("v", 1024, 1024), ("o", 2048, 1024),
                    ("gate", 1024, 3072), ("up", 1024, 3072), ("down", 3072, 1024)]
QWEN3_8B_LAYER = [("q", 4096, 4096), ("k", 4096, 1024), ("v", 4096, 1024), ("o", 4096, 4096),
                  ("gate", 4096, 12288), ("up", 4096, 12288), ("down", 12288, 4096)]
QWEN3_4B_LAYER = [("q", 2560, 4096), ("k", 2560, 1024), ("v", 2560, 1024), ("o", 4096, 2560),
                  ("gate", 2560, 9728), ("up", 2560, 9728), ("down", 9728, 2560)]


def to_bf16_values(a):
    """Round a float array to bfloat16 (nearest even) and return it as float32."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    return t.to(torch.bfloat16).to(torch.float32).numpy()


def _store(a, storage):
    a = np.asarray(a, dtype=np.float32)
    return to_bf16_values(a) if storage == "bf16" else a


def weights(rng, d_out, d_in, std=0.02, storage="f32"):
    return _store(rng.standard_normal((d_out, d_in)) * std, storage)


def shifted_target(rng, X, W, rank=4, std=0.05, storage="f32"):
    """MSE target Y* = X W*^T with W* = W + rank-`rank` shift whose entries have std `std`."""
    d_out, d_in = W.shape
    P = rng.standard_normal((d_out, rank))
    Q = rng.standard_normal((d_in, rank))
    Wstar = W.astype(np.float64) + (std / np.sqrt(rank)) * (P @ Q.T)
    Y = X.astype(np.float64) @ Wstar.T
    return _store(Y, storage)


def x_lowrank_plus_noise(rng, n, d, rank=16, s_hi=10.0, s_lo=0.1, noise=0.01, storage="f32"):
    """Planted spectrum: U diag(S) V^T + noise, S log-spaced s_hi..s_lo (the small fp32 config)."""
    U, _ = np.linalg.qr(rng.standard_normal((n, rank)))
    V, _ = np.linalg.qr(rng.standard_normal((d, rank)))
    S = np.logspace(np.log10(s_hi), np.log10(s_lo), rank)
    X = (U * S[None, :]) @ V.T + noise * rng.standard_normal((n, d))
    return _store(X, storage)


def x_rmsnorm_gaussian(rng, n, d, storage="bf16"):
    """iid N(0,1) rows scaled to unit RMS per token (input of a projection after RMSNorm)."""
    X = rng.standard_normal((n, d))
    X /= np.sqrt(np.mean(X * X, axis=1, keepdims=True))
    return _store(X, storage)


def x_powerlaw_outliers(rng, n, d, n_outliers=5, outlier_scale=20.0, storage="bf16"):
    """Power-law activation spectrum (singular values ~ 1/i) in a random rotation,
    a few outlier channels scaled up, global unit RMS.  Used for the Qwen3-8B/4B
    shaped layers."""
    Zm = rng.standard_normal((n, d)) / np.sqrt(n)
    Zm *= (1.0 / np.arange(1, d + 1))[None, :]
    V, _ = np.linalg.qr(rng.standard_normal((d, d)))
    X = Zm @ V.T
    ch = rng.choice(d, size=min(n_outliers, d), replace=False)
    X[:, ch] *= outlier_scale
    X /= np.sqrt(np.mean(X * X))
    return _store(X, storage)


def single_layer_problem(seed, n, d_in, d_out, kind="lowrank", storage="f32", target_storage="f32"):
    """(W, X, Y*) for one projection with an MSE loss to a shifted-weights target."""
    rng = np.random.default_rng(seed)
    W = weights(rng, d_out, d_in, storage=storage)
    if kind == "lowrank":
        X = x_lowrank_plus_noise(rng, n, d_in, rank=min(16, d_in, n), storage=storage)
    elif kind == "rmsnorm":
        X = x_rmsnorm_gaussian(rng, n, d_in, storage=storage)
    elif kind == "powerlaw":
        X = x_powerlaw_outliers(rng, n, d_in, storage=storage)
    else:
        raise ValueError(kind)
    Ystar = shifted_target(rng, X, W, storage=target_storage)
    return W, X, Ystar


# ----------------------------------------------------------------------------
# full-size inputs generated on the device (outside any timed region)
# ----------------------------------------------------------------------------
def device_powerlaw_x(seed, n, d_in, device="cuda", n_outliers=5, outlier_scale=20.0):
    """bf16 activations on the device, same recipe as x_powerlaw_outliers, drawn from torch's
    seeded generator."""
    gen = torch.Generator(device=device)
    gen.manual_seed(int(seed))
    f32 = dict(device=device, dtype=torch.float32, generator=gen)
    X = torch.randn(n, d_in, **f32) / float(np.sqrt(n))
    X *= (1.0 / torch.arange(1, d_in + 1, device=device, dtype=torch.float32))[None, :]
    # random rotation of feature space as a butterfly network: each stage permutes the channels at
    # random and rotates consecutive pairs by random angles (exactly orthogonal, O(n d) per stage,
    # plain elementwise kernels); 2 log2(d) stages mix every channel into every other.
    for _ in range(2 * int(np.ceil(np.log2(max(d_in, 2))))):
        perm = torch.randperm(d_in, device=device, generator=gen)
        X = X[:, perm]
        half = d_in // 2
        ang = torch.rand(half, **f32) * (2.0 * np.pi)
        c, s = torch.cos(ang)[None, :], torch.sin(ang)[None, :]
        a, b = X[:, 0:2 * half:2], X[:, 1:2 * half:2]
        ra, rb = c * a - s * b, s * a + c * b
        X[:, 0:2 * half:2] = ra
        X[:, 1:2 * half:2] = rb
        del a, b, ra, rb
    ch = torch.randperm(d_in, device=device, generator=gen)[:n_outliers]
    X[:, ch] *= outlier_scale
    X /= X.square().mean().sqrt()
    return X.to(torch.bfloat16)


def device_weights_and_target(seed, X, d_out, device="cuda", target_dtype=torch.bfloat16):
    """bf16 W ~ N(0, 0.02^2) and the MSE target Y* = X W*^T, W* = W + rank-4 shift (entry std 0.05), stored in
    `target_dtype` (bf16 like every other tensor of the bf16 configurations, or fp32)."""
    gen = torch.Generator(device=device)
    gen.manual_seed(int(seed))
    f32 = dict(device=device, dtype=torch.float32, generator=gen)
    d_in = X.shape[1]
    W = (torch.randn(d_out, d_in, **f32) * 0.02).to(torch.bfloat16)
    P = torch.randn(d_out, 4, **f32)
    Q = torch.randn(d_in, 4, **f32)
    Wstar = W.float() + (0.05 / 2.0) * (P @ Q.T)
    Ystar = X.float() @ Wstar.T
    return W, Ystar.to(target_dtype)


def mlp_stack_problem(seed, n_blocks, hidden, inter, vocab, n_seq, seq_len, emb_rank=16, gains=False):
    """Weights and token ids of a gated-MLP stack (the reduced form of the MLP-stack workload): bf16-exact values.

    params: "E" [vocab][hidden] (a rank-`emb_rank` part plus noise, so that activations have a few dominant
    directions), ("gate", b) / ("up", b) [inter][hidden], ("down", b) [hidden][inter], ("head", 0) [vocab][hidden],
    all ~ N(0, 0.02^2) except E (unit-RMS rows on average); ids uniform over the vocabulary.  gains=True adds
    the normalisation gains ("norm", b) and ("norm_f", 0), fp32 vectors of 1 + N(0, 0.1^2)."""
    rng = np.random.default_rng(seed)
    A = rng.standard_normal((vocab, emb_rank))
    C = rng.standard_normal((emb_rank, hidden))
    E = (A * np.logspace(0.0, -1.0, emb_rank)[None, :]) @ C + 0.3 * rng.standard_normal((vocab, hidden))
    E /= np.sqrt(np.mean(E * E))
    params = {"n_blocks": n_blocks, "E": to_bf16_values(E)}
    for b in range(n_blocks):
        params[("gate", b)] = weights(rng, inter, hidden, storage="bf16")
        params[("up", b)] = weights(rng, inter, hidden, storage="bf16")
        params[("down", b)] = weights(rng, hidden, inter, storage="bf16")
    params[("head", 0)] = weights(rng, vocab, hidden, storage="bf16")
    ids = rng.integers(0, vocab, size=(n_seq, seq_len), dtype=np.int64)
    if gains:       # drawn last, so that the other tensors do not depend on the flag
        for nm in [("norm", b) for b in range(n_blocks)] + [("norm_f", 0)]:
            params[nm] = (1.0 + 0.1 * rng.standard_normal(hidden)).astype(np.float32)
    return params, ids


def device_mlp_stack(seed, n_blocks, hidden, inter, vocab, n_seq, seq_len, emb_rank=16, device="cuda"):
    """The MLP-stack workload at any size, generated on the device (same recipe as mlp_stack_problem, without gains):
    bf16 tensors "E", ("gate", b), ("up", b), ("down", b), ("head", 0) and int64 ids [n_seq][seq_len]."""
    gen = torch.Generator(device=device)
    gen.manual_seed(int(seed))
    f32 = dict(device=device, dtype=torch.float32, generator=gen)
    A = torch.randn(vocab, emb_rank, **f32) * torch.logspace(0.0, -1.0, emb_rank, device=device)[None, :]
    E = A @ torch.randn(emb_rank, hidden, **f32) + 0.3 * torch.randn(vocab, hidden, **f32)
    E /= E.square().mean().sqrt()
    params = {"n_blocks": n_blocks, "E": E.to(torch.bfloat16)}
    for b in range(n_blocks):
        params[("gate", b)] = (torch.randn(inter, hidden, **f32) * 0.02).to(torch.bfloat16)
        params[("up", b)] = (torch.randn(inter, hidden, **f32) * 0.02).to(torch.bfloat16)
        params[("down", b)] = (torch.randn(hidden, inter, **f32) * 0.02).to(torch.bfloat16)
    params[("head", 0)] = (torch.randn(vocab, hidden, **f32) * 0.02).to(torch.bfloat16)
    ids = torch.randint(0, vocab, (n_seq, seq_len), device=device, generator=gen)
    return params, ids


DECODER_PROJECTIONS = ("q", "k", "v", "o", "gate", "up", "down")


def decoder_shapes(hidden, n_heads, n_kv_heads, inter, head_dim=128):
    """(d_out, d_in) of the seven projections of one decoder layer."""
    return {"q": (n_heads * head_dim, hidden), "k": (n_kv_heads * head_dim, hidden), "v": (n_kv_heads * head_dim, hidden),
            "o": (hidden, n_heads * head_dim), "gate": (inter, hidden), "up": (inter, hidden), "down": (hidden, inter)}


def decoder_problem(seed, n_layers, hidden, n_heads, n_kv_heads, inter, vocab, n_seq, seq_len, emb_rank=16):
    """Weights and token ids of a small decoder-style transformer (grouped-query attention with 128-wide heads, gated
    MLP, LM head): bf16-exact values, W ~ N(0, 0.02^2), embedding as in mlp_stack_problem."""
    rng = np.random.default_rng(seed)
    A = rng.standard_normal((vocab, emb_rank))
    C = rng.standard_normal((emb_rank, hidden))
    E = (A * np.logspace(0.0, -1.0, emb_rank)[None, :]) @ C + 0.3 * rng.standard_normal((vocab, hidden))
    E /= np.sqrt(np.mean(E * E))
    params = {"n_layers": n_layers, "n_heads": n_heads, "n_kv_heads": n_kv_heads, "E": to_bf16_values(E)}
    shapes = decoder_shapes(hidden, n_heads, n_kv_heads, inter)
    for l in range(n_layers):
        for p in DECODER_PROJECTIONS:
            params[(p, l)] = weights(rng, shapes[p][0], shapes[p][1], storage="bf16")
    params[("head", 0)] = weights(rng, vocab, hidden, storage="bf16")
    ids = rng.integers(0, vocab, size=(n_seq, seq_len), dtype=np.int64)
    return params, ids


def device_decoder(seed, n_layers, hidden, n_heads, n_kv_heads, inter, vocab, n_seq, seq_len, emb_rank=16, device="cuda"):
    """The decoder workload at any size, generated on the device (same recipe as decoder_problem)."""
    gen = torch.Generator(device=device)
    gen.manual_seed(int(seed))
    f32 = dict(device=device, dtype=torch.float32, generator=gen)
    A = torch.randn(vocab, emb_rank, **f32) * torch.logspace(0.0, -1.0, emb_rank, device=device)[None, :]
    E = A @ torch.randn(emb_rank, hidden, **f32) + 0.3 * torch.randn(vocab, hidden, **f32)
    E /= E.square().mean().sqrt()
    params = {"n_layers": n_layers, "n_heads": n_heads, "n_kv_heads": n_kv_heads, "E": E.to(torch.bfloat16)}
    shapes = decoder_shapes(hidden, n_heads, n_kv_heads, inter)
    for l in range(n_layers):
        for p in DECODER_PROJECTIONS:
            params[(p, l)] = (torch.randn(shapes[p][0], shapes[p][1], **f32) * 0.02).to(torch.bfloat16)
    params[("head", 0)] = (torch.randn(vocab, hidden, **f32) * 0.02).to(torch.bfloat16)
    ids = torch.randint(0, vocab, (n_seq, seq_len), device=device, generator=gen)
    return params, ids
