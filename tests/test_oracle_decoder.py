"""Pins for the decoder oracle (oracle/decoder.py), against routines that share nothing with it:

* the unperturbed loss equals the same model written with torch's own functional ops in float64
  (rms_norm, scaled_dot_product_attention with a causal mask, silu, cross_entropy) with the rotary embedding written as a
  complex multiplication, when nothing is rounded;
* the attention is causal (a later token never changes an earlier token's output) and the rotary embedding makes the
  scores depend on positions only through their difference;
* g is the directional derivative of that loss along the joint perturbation (torch autograd);
* with basis sharing the layers that read the same activations carry one basis, and their Gaussian factors stay their own.
"""
import numpy as np
import torch
import torch.nn.functional as F

from oracle import agzo as oagzo
from oracle import decoder as odec
from oracle import stack as ostack
from paper_2601_17261_amd import synth

R, K = 4, 2


def small():
    return synth.decoder_problem(7, n_layers=2, hidden=64, n_heads=2, n_kv_heads=1, inter=96, vocab=61, n_seq=2, seq_len=13)


def seeds_for(params, step=0):
    return {nm: 1000 * step + i for i, nm in enumerate(odec.layer_names(params["n_layers"]))}


def torch_rope(x, pos):
    """x [N][H][128] float64: pairs (i, i + 64) as complex numbers times exp(i pos theta^(-2i/128))."""
    half = 64
    inv = torch.pow(torch.tensor(1.0e6, dtype=torch.float64), -torch.arange(half, dtype=torch.float64) * 2.0 / 128.0)
    z = torch.complex(x[..., :half], x[..., half:]) * torch.polar(torch.ones(len(pos), half, dtype=torch.float64),
                                                                  pos[:, None].double() * inv[None, :])[:, None, :]
    return torch.cat([z.real, z.imag], dim=-1)


def torch_loss(params, ids, weights):
    n_seq, seq_len = ids.shape
    H, Hkv = params["n_heads"], params["n_kv_heads"]
    N = n_seq * seq_len
    pos = torch.arange(seq_len).repeat(n_seq)
    h = torch.from_numpy(params["E"].astype(np.float64))[torch.from_numpy(ids.reshape(-1))]
    for l in range(params["n_layers"]):
        n = F.rms_norm(h, (h.shape[1],), eps=1e-6)
        q = F.linear(n, weights[("q", l)]).reshape(N, H, 128)
        k = F.linear(n, weights[("k", l)]).reshape(N, Hkv, 128)
        v = F.linear(n, weights[("v", l)]).reshape(N, Hkv, 128)
        q = torch_rope(F.rms_norm(q, (128,), eps=1e-6), pos)
        k = torch_rope(F.rms_norm(k, (128,), eps=1e-6), pos)
        # [batch][heads][time][128], kv heads repeated for their query groups
        def bh(t, heads):
            return t.reshape(n_seq, seq_len, heads, 128).permute(0, 2, 1, 3)
        kk = bh(k, Hkv).repeat_interleave(H // Hkv, dim=1)
        vv = bh(v, Hkv).repeat_interleave(H // Hkv, dim=1)
        a = F.scaled_dot_product_attention(bh(q, H), kk, vv, is_causal=True)
        a = a.permute(0, 2, 1, 3).reshape(N, H * 128)
        h = h + F.linear(a, weights[("o", l)])
        n = F.rms_norm(h, (h.shape[1],), eps=1e-6)
        h = h + F.linear(F.silu(F.linear(n, weights[("gate", l)])) * F.linear(n, weights[("up", l)]), weights[("down", l)])
    logits = F.linear(F.rms_norm(h, (h.shape[1],), eps=1e-6), weights[("head", 0)])
    return F.cross_entropy(logits, torch.from_numpy(ostack.shifted_targets(ids)), ignore_index=-1)


def test_unperturbed_loss_matches_torch_functional_model():
    params, ids = small()
    names = odec.layer_names(2)
    w = {nm: torch.from_numpy(params[nm].astype(np.float64)) for nm in names}
    want = torch_loss(params, ids, w).item()
    got = odec.forward(params, ids, act=None)
    assert abs(got - want) < 1e-12 * abs(want)
    # rounding the stored activations to bf16 moves the loss at bf16 level, not more
    assert abs(odec.forward(params, ids, act="bf16") - want) < 2e-3 * abs(want)


def test_attention_is_causal_and_rotary_scores_depend_on_position_differences():
    rng = np.random.default_rng(3)
    n_seq, T, H, Hkv = 2, 9, 4, 2
    q, k, v = rng.standard_normal((n_seq * T, H * 128)), rng.standard_normal((n_seq * T, Hkv * 128)), rng.standard_normal((n_seq * T, Hkv * 128))
    a = odec.attention(q, k, v, n_seq, T, None)
    k2, v2 = k.copy(), v.copy()
    k2[T - 1] += 5.0                      # the last token of the first sequence ...
    v2[T - 1] -= 3.0
    a2 = odec.attention(q, k2, v2, n_seq, T, None)
    np.testing.assert_array_equal(a[:T - 1], a2[:T - 1])          # ... is invisible to the earlier ones
    np.testing.assert_array_equal(a[T:], a2[T:])                  # and to the other sequence
    assert np.abs(a[T - 1] - a2[T - 1]).max() > 1e-3
    # the first token attends to itself only: its output is its own value vector (of its kv head)
    np.testing.assert_allclose(a[0].reshape(H, 128), v[0].reshape(Hkv, 128).repeat(H // Hkv, axis=0), atol=1e-12)
    # <rope(x, s), rope(y, t)> depends on s - t only, and rope is an isometry
    x, y = rng.standard_normal((1, 1, 128)), rng.standard_normal((1, 1, 128))
    d1 = float((odec.rope(x, [3]) * odec.rope(y, [7])).sum())
    d2 = float((odec.rope(x, [10]) * odec.rope(y, [14])).sum())
    assert abs(d1 - d2) < 1e-12
    assert abs(np.linalg.norm(odec.rope(x, [11])) - np.linalg.norm(x)) < 1e-12
    np.testing.assert_allclose(odec.rope(x, [0]), x, atol=0)


def test_g_is_the_directional_derivative_along_the_joint_perturbation():
    params, ids = small()
    names = odec.layer_names(2)
    seeds = seeds_for(params)
    o = odec.agzo_decoder_step(params, ids, R, K, 1e-4, 1e-2, seeds, act=None, storage="f32")
    w = {nm: torch.from_numpy(params[nm].astype(np.float64)).requires_grad_(True) for nm in names}
    torch_loss(params, ids, w).backward()
    dd = sum(float((w[nm].grad.numpy() * o["Z"][nm]).sum()) for nm in names)
    assert abs(o["g"] - dd) < 1e-5 * abs(dd), (o["g"], dd)
    o1 = odec.agzo_decoder_step(params, ids, R, K, 1e-4, 1e-2, seeds, act=None, storage="f32", one_sided=True)
    assert abs(o1["g"] - dd) < 2e-3 * abs(dd) and o1["Lm"] == 0.0
    # every layer moved along its own direction by the one scalar
    for nm in names:
        step = (params[nm].astype(np.float64) - o["W_new"][nm]) / (1e-2 * o["g"])
        np.testing.assert_allclose(step, o["Z"][nm], atol=2e-4 * np.abs(o["Z"][nm]).max())


def test_layers_reading_the_same_activations_and_basis_sharing():
    params, ids = small()
    seeds = seeds_for(params, step=2)
    o = odec.agzo_decoder_step(params, ids, R, K, 1e-3, 1e-2, seeds, act="bf16", storage="bf16")
    for l in range(2):
        np.testing.assert_array_equal(o["inputs"][("q", l)], o["inputs"][("k", l)])
        np.testing.assert_array_equal(o["inputs"][("q", l)], o["inputs"][("v", l)])
        np.testing.assert_array_equal(o["inputs"][("gate", l)], o["inputs"][("up", l)])
        assert o["inputs"][("o", l)].shape[1] == 2 * 128 and o["inputs"][("down", l)].shape[1] == 96
        assert not np.array_equal(o["B"][("q", l)], o["B"][("k", l)])          # own seeds, own bases
    for nm in odec.layer_names(2):
        np.testing.assert_array_equal(o["B"][nm], oagzo.subspace_extract(o["inputs"][nm], R, K, seeds[nm])["B"])
    share = {}
    for l in range(2):
        share.update({("k", l): ("q", l), ("v", l): ("q", l), ("up", l): ("gate", l)})
    s = odec.agzo_decoder_step(params, ids, R, K, 1e-3, 1e-2, seeds, act="bf16", storage="bf16", share=share)
    for l in range(2):
        np.testing.assert_array_equal(s["B"][("k", l)], s["B"][("q", l)])
        np.testing.assert_array_equal(s["B"][("up", l)], s["B"][("gate", l)])
        assert not np.array_equal(s["G"][("k", l)][: 64], s["G"][("q", l)][: 64])
        np.testing.assert_array_equal(s["B"][("q", l)], o["B"][("q", l)])
    assert s["L0"] == o["L0"] and s["g"] != o["g"]
