"""Oracle: one AGZO iteration over a small decoder-style transformer, in fp64 (test infrastructure only).

Alg. 2 for a model whose layers are full decoder layers (Sec. 3.1 treats every linear map of such a layer as a
layer W_l with input activations H_l): one unperturbed pass gives f0 and, at every linear layer, the activation
basis of that layer's own input (Alg. 1); then all linear layers are perturbed at once by +eps Z_l, Z_l = G_l B_l^T
(Eq. 7), for f+, and by -eps Z_l for f-; one global scalar g (Eq. 10) scales every layer's update.

Model (the structure of a Qwen3 decoder: grouped-query attention, per-head RMS normalisation of queries and keys,
rotary position embedding, gated MLP; gains fixed to 1, embedding frozen):
  h = E[ids]
  per layer:
    n = rmsnorm(h);  q = W_q n, k = W_k n, v = W_v n          (q: n_heads x 128, k and v: n_kv_heads x 128 per token)
    q, k <- rope(rmsnorm_per_head(q)), rope(rmsnorm_per_head(k))
    a = causal softmax(q k^T / sqrt(128)) v, every group of n_heads / n_kv_heads query heads reading one kv head
    h = h + W_o a
    n = rmsnorm(h);  h = h + W_down (silu(W_gate n) * (W_up n))
  logits = W_head rmsnorm(h);  loss = token cross-entropy with next-token targets inside each sequence
rope: the pair (x_i, x_{i+64}) of a head's 128 values is rotated by the angle t * theta^(-2i/128), t the token's position
inside its sequence, theta = 10^6 (the half-split pairing of the rotary embedding as these models use it).

Activation storage: every stored tensor is rounded to `act` ("bf16", "f32", or None): n, the projection outputs, the
rotated q and k, the attention output, the MLP's intermediate tensors, the residual sums.  The logits are never stored.
Nothing is blocked, fused or reordered.  Pins live in tests/test_oracle_decoder.py.
"""
import numpy as np

from . import agzo
from .stack import rmsnorm, shifted_targets, silu

HEAD_DIM = 128
ROPE_THETA = 1.0e6


def _store(a, act):
    return np.asarray(a, dtype=np.float64) if act is None else agzo.round_storage(a, act)


def layer_names(n_layers):
    """Order in which the linear layers are met (and seeds are assigned)."""
    names = []
    for l in range(n_layers):
        names += [(p, l) for p in ("q", "k", "v", "o", "gate", "up", "down")]
    return names + [("head", 0)]


def rope(x, positions):
    """x [tokens][heads][128]; rotates (x_i, x_{i+64}) by positions[t] * theta^(-2i/128)."""
    half = HEAD_DIM // 2
    inv = ROPE_THETA ** (-np.arange(half, dtype=np.float64) * 2.0 / HEAD_DIM)
    ang = np.asarray(positions, dtype=np.float64)[:, None] * inv[None, :]          # [tokens][64]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def head_norm(x):
    """RMS normalisation over each head's 128 values (gain 1)."""
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + 1e-6)


def attention(q, k, v, n_seq, seq_len, act):
    """q [N][H*128], k, v [N][Hkv*128] (token-major, sequences back to back) -> a [N][H*128]."""
    N = q.shape[0]
    H, Hkv = q.shape[1] // HEAD_DIM, k.shape[1] // HEAD_DIM
    pos = np.tile(np.arange(seq_len), n_seq)
    qh = _store(rope(head_norm(q.reshape(N, H, HEAD_DIM)), pos), act)
    kh = _store(rope(head_norm(k.reshape(N, Hkv, HEAD_DIM)), pos), act)
    vh = v.reshape(N, Hkv, HEAD_DIM)
    out = np.zeros((N, H, HEAD_DIM))
    group = H // Hkv
    mask = np.tril(np.ones((seq_len, seq_len), dtype=bool))
    for b in range(n_seq):
        sl = slice(b * seq_len, (b + 1) * seq_len)
        for h in range(H):
            s = qh[sl, h, :] @ kh[sl, h // group, :].T / np.sqrt(float(HEAD_DIM))
            s = np.where(mask, s, -np.inf)
            p = np.exp(s - s.max(axis=1, keepdims=True))
            p /= p.sum(axis=1, keepdims=True)
            out[sl, h, :] = p @ vh[sl, h // group, :]
    return out.reshape(N, H * HEAD_DIM)


def forward(params, ids, act="bf16", delta=None, record=None):
    """Loss of the model with weights W_l + delta[l] (delta: dict name -> matrix, or None).
    record, if a dict, receives the input activations of every linear layer."""
    def lin(name, x):
        W = np.asarray(params[name], dtype=np.float64)
        if delta is not None:
            W = W + delta[name]
        if record is not None:
            record[name] = x
        return x @ W.T

    ids = np.asarray(ids)
    n_seq, seq_len = ids.shape
    h = np.asarray(params["E"], dtype=np.float64)[ids.reshape(-1)]
    for l in range(params["n_layers"]):
        n = _store(rmsnorm(h), act)
        q, k, v = (_store(lin((p, l), n), act) for p in ("q", "k", "v"))
        a = _store(attention(q, k, v, n_seq, seq_len, act), act)
        h = _store(h + _store(lin(("o", l), a), act), act)
        n = _store(rmsnorm(h), act)
        g, u = _store(lin(("gate", l), n), act), _store(lin(("up", l), n), act)
        m = _store(silu(g) * u, act)
        h = _store(h + _store(lin(("down", l), m), act), act)
    logits = lin(("head", 0), _store(rmsnorm(h), act))
    return agzo.ce_loss(logits, shifted_targets(ids))


def agzo_decoder_step(params, ids, r, K, eps, lr, seeds, act="bf16", storage="bf16", one_sided=False, share=None):
    """One AGZO iteration (Alg. 2).  seeds: dict layer name -> 64-bit seed of that layer for this step.
    share: optional dict name -> name whose basis that layer reuses (layers that read the same activations: q / k / v,
    gate / up); the Gaussian factors stay per layer."""
    names = layer_names(params["n_layers"])
    inputs = {}
    L0 = forward(params, ids, act, None, inputs)
    B, G, Z = {}, {}, {}
    for nm in names:
        src = share.get(nm, nm) if share else nm
        B[nm] = B[src] if src != nm else agzo.subspace_extract(inputs[nm], r, K, seeds[nm])["B"]
        Z[nm], G[nm] = agzo.perturbation(B[nm], seeds[nm], np.asarray(params[nm]).shape[0])
    Lp = forward(params, ids, act, {nm: eps * Z[nm] for nm in names})
    Lm = 0.0 if one_sided else forward(params, ids, act, {nm: -eps * Z[nm] for nm in names})
    g = (Lp - L0) / eps if one_sided else (Lp - Lm) / (2.0 * eps)
    W_new = {nm: agzo.round_storage(np.asarray(params[nm], dtype=np.float64) - lr * g * Z[nm], storage) for nm in names}
    return {"L0": L0, "Lp": Lp, "Lm": Lm, "g": g, "B": B, "G": G, "Z": Z, "W_new": W_new, "inputs": inputs}
