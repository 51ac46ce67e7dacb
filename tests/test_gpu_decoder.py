"""GPU parity for Alg. 2 over full decoder layers: the attention core on its own against the oracle's attention, and one
AGZO iteration over a reduced decoder (2 layers of grouped-query attention + gated MLP, LM head, token cross-entropy,
global g) composed from the library's calls: every linear layer (base forward, batched extraction, factored perturbed
forward, fused cross-entropy, rank-r update) and the model between the layers (agzo_glue_*) run in the library; torch
only gathers the embedding rows.
"""
import numpy as np
import pytest
import torch

from oracle import agzo as oagzo
from oracle import decoder as odec
from oracle import stack as ostack
from paper_2601_17261_amd import binding, synth

pytestmark = pytest.mark.gpu

R, K = 8, 2
LR = float(np.float32(1e-3))
BF = torch.bfloat16


def rel(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


@pytest.fixture(scope="module")
def ctx():
    c = binding.Context()
    yield c
    c.close()


def bf(a):
    return torch.from_numpy(synth.to_bf16_values(np.asarray(a, dtype=np.float32))).to("cuda", BF)


@pytest.mark.parametrize("n_seq,T,H,Hkv", [(2, 13, 2, 1), (3, 100, 4, 2), (1, 200, 8, 8), (2, 64, 2, 2), (1, 1, 2, 1),
                                           (2, 512, 16, 8),      # the decoder workload's sequence length and heads
                                           (1, 129, 4, 1)])      # one query past a workgroup's 128, four query heads per kv head
def test_attention_core_matches_oracle(ctx, n_seq, T, H, Hkv):
    rng = np.random.default_rng(100 * T + H)
    N = n_seq * T
    q, k, v = bf(rng.standard_normal((N, H * 128))), bf(2.0 * rng.standard_normal((N, Hkv * 128))), bf(rng.standard_normal((N, Hkv * 128)))
    out = torch.full((N, H * 128 + 8), 7.0, dtype=BF, device="cuda")          # rows inside a wider allocation
    ctx.glue_attention(q, k, v, out[:, :H * 128], n_seq, T)
    ctx.check()
    h64 = lambda t: t.double().cpu().numpy()
    want = odec.attention(h64(q), h64(k), h64(v), n_seq, T, "bf16")
    got = h64(out[:, :H * 128])
    # fp32 softmax with bf16 probabilities against fp64: one bf16 rounding of the result (2^-8 relative) plus the
    # probabilities' own rounding, which averages down over the keys
    assert rel(got, want) < 4e-3
    assert np.abs(got - want).max() < 2.0 ** -6 * max(np.abs(want).max(), 1.0)
    assert (out[:, H * 128:] == 7.0).all()
    # causal and per sequence: changing the last token of the first sequence leaves everything else bit-identical
    k2, v2 = k.clone(), v.clone()
    k2[T - 1] += 4.0
    v2[T - 1] -= 3.0
    out2 = torch.empty(N, H * 128, dtype=BF, device="cuda")
    ctx.glue_attention(q, k2, v2, out2, n_seq, T)
    keep = [i for i in range(N) if i != T - 1]
    assert torch.equal(out2[keep], out[:, :H * 128][keep])


def test_attention_rejects_bad_shapes(ctx):
    q = torch.zeros(8, 256, dtype=BF, device="cuda")
    kv = torch.zeros(8, 128, dtype=BF, device="cuda")
    out = torch.zeros(8, 256, dtype=BF, device="cuda")
    lib = ctx.lib
    import ctypes
    def call(n_seq, T, H, Hkv, theta=1.0e6):
        return lib.agzo_glue_attention(ctx.h, ctypes.c_void_p(q.data_ptr()), 256, ctypes.c_void_p(kv.data_ptr()), 128,
                                       ctypes.c_void_p(kv.data_ptr()), 128, ctypes.c_void_p(out.data_ptr()), 256, n_seq, T, H, Hkv, theta)
    assert call(1, 8, 2, 1) == 0
    assert call(1, 8, 3, 2) == binding.EINVAL          # heads not a multiple of kv heads
    assert call(1, 8, 2, 0) == binding.EINVAL
    assert call(-1, 8, 2, 1) == binding.EINVAL
    assert call(1, 8, 2, 1, 0.5) == binding.EINVAL
    assert call(0, 8, 2, 1) == 0                       # nothing to do
    ctx.check()


class GpuDecoder:
    def __init__(self, ctx, params, ids):
        self.ctx = ctx
        self.nl, self.H, self.Hkv = params["n_layers"], params["n_heads"], params["n_kv_heads"]
        self.names = odec.layer_names(self.nl)
        self.E = bf(params["E"])
        self.W = {nm: bf(params[nm]) for nm in self.names}
        self.n_seq, self.T = ids.shape
        self.ids = torch.from_numpy(ids.reshape(-1)).cuda()
        self.tgt = torch.from_numpy(ostack.shifted_targets(ids).astype(np.int32)).cuda()
        self.loss = binding.make_loss(self.tgt, kind=binding.LOSS_CE)
        self.B, self.X = {}, {}

    def linear(self, nm, x, sign, eps, seeds, loss_dev=None):
        W = self.W[nm]
        head = nm[0] == "head"
        Y = None if head else torch.empty(x.shape[0], W.shape[0], dtype=BF, device="cuda")
        L = binding.make_layer(W, x, R, Y=Y)
        loss = self.loss if head else None
        if sign == 0:
            self.X[nm] = x
            self.ctx.layer_forward_sketch(L, W, x, Y, binding.SKETCH_NONE, None, seeds[nm], None, loss, loss_dev)
        else:
            self.ctx.perturbed_forward(L, W, x, self.B[nm], seeds[nm], sign * eps, Y, loss, loss_dev)
        return Y

    def rms(self, h):
        y = torch.empty_like(h)
        self.ctx.glue_rmsnorm(h, y)
        return y

    def run_pass(self, sign, eps, seeds, loss_dev):
        h = self.E[self.ids].contiguous()
        for l in range(self.nl):
            n = self.rms(h)
            q, k, v = (self.linear((p, l), n, sign, eps, seeds) for p in ("q", "k", "v"))
            a = torch.empty_like(q)
            self.ctx.glue_attention(q, k, v, a, self.n_seq, self.T)
            self.ctx.glue_add(h, self.linear(("o", l), a, sign, eps, seeds))
            n = self.rms(h)
            g, u = self.linear(("gate", l), n, sign, eps, seeds), self.linear(("up", l), n, sign, eps, seeds)
            m = torch.empty_like(g)
            self.ctx.glue_swiglu(g, u, m)
            self.ctx.glue_add(h, self.linear(("down", l), m, sign, eps, seeds))
        self.linear(("head", 0), self.rms(h), sign, eps, seeds, loss_dev)

    def step(self, eps, lr, seeds, share=None):
        out = torch.zeros(4, dtype=torch.float64, device="cuda")
        self.run_pass(0, eps, seeds, out[0:1])
        own = [nm for nm in self.names if not share or nm not in share]
        for nm in own:
            self.B[nm] = torch.empty(self.W[nm].shape[1], R, dtype=torch.float32, device="cuda")
        self.ctx.basis_many([(binding.make_layer(self.W[nm], self.X[nm], R), self.X[nm], seeds[nm], None, self.B[nm]) for nm in own], K)
        for nm, src in (share or {}).items():
            self.B[nm] = self.B[src]
        self.run_pass(+1, eps, seeds, out[1:2])
        self.run_pass(-1, eps, seeds, out[2:3])
        self.ctx.two_point(out, eps)
        self.ctx.update_many([(self.W[nm], self.B[nm], seeds[nm], lr, out[3:4]) for nm in self.names])
        self.ctx.check()
        return out.cpu().numpy()


@pytest.mark.parametrize("shared", [False, True])
def test_reduced_decoder_step_matches_oracle(ctx, shared):
    """bf16 storage: every stored activation is a rounding point and the library's fp32 arithmetic can land one ulp from
    the oracle's fp64 there, which moves each loss by a few 1e-5 relative without cancelling between the passes; the
    perturbation is therefore large enough to stand clear of that floor (parity does not need the loss to be linear)."""
    eps = float(np.float32(3e-2))
    params, ids = synth.decoder_problem(17, n_layers=2, hidden=256, n_heads=2, n_kv_heads=1, inter=384, vocab=1000, n_seq=2, seq_len=72)
    names = odec.layer_names(2)
    seeds = {nm: 9000 + i for i, nm in enumerate(names)}
    share = None
    if shared:
        share = {}
        for l in range(2):
            share.update({("k", l): ("q", l), ("v", l): ("q", l), ("up", l): ("gate", l)})
    o = odec.agzo_decoder_step(params, ids, R, K, eps, LR, seeds, act="bf16", storage="bf16", share=share)
    model = GpuDecoder(ctx, params, ids)
    got = model.step(eps, LR, seeds, share)
    for nm in names:
        Bg = model.B[nm].double().cpu().numpy()
        # (the inputs of the later layers already differ from the oracle's at bf16 rounding level, and the last basis
        # directions, past the dominant ones, move with them)
        assert rel(Bg @ (Bg.T @ o["B"][nm]), o["B"][nm]) < 3e-2, nm
    tol_l, floor_l = 1e-4, 6e-5
    assert abs(got[0] - o["L0"]) < tol_l * o["L0"]
    assert abs(got[1] - o["Lp"]) < tol_l * o["Lp"]
    assert abs(got[2] - o["Lm"]) < tol_l * o["Lm"]
    floor_g = floor_l * o["L0"] / (2.0 * eps) * 2.0 ** 0.5
    assert abs(got[3] - o["g"]) < 2e-2 * abs(o["g"]) + floor_g, (got[3], o["g"], floor_g)
    for nm in names:
        Wg = model.W[nm].double().cpu().numpy()
        assert rel(Wg, o["W_new"][nm]) < 3e-3, nm
        assert (Wg != params[nm]).mean() > 0.01, nm                      # the update is not a no-op
        # elementwise with this side's scalar and basis: one rounding of the result plus the increment's own error
        Bg = model.B[nm].double().cpu().numpy()
        want = oagzo.round_bf16(params[nm].astype(np.float64) - LR * got[3] * (o["G"][nm] @ Bg.T))
        ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(want), 1e-30))) - 7)
        bound = ulp * 1.0001 + LR * 2.0 ** -14 * abs(got[3]) * (np.abs(o["G"][nm]) @ np.abs(Bg).T)
        diff = np.abs(Wg - want)
        assert (diff <= bound).all(), (nm, float((diff / bound).max()))
        assert (diff > 0).mean() < 0.05, nm
