"""GPU parity for the MLP-stack workload in its reduced form (2 blocks, 2 x 128 tokens, the full widths:
hidden 2048, intermediate 6144, vocabulary 32000; token cross-entropy; r = 16, K = 3): one AGZO iteration
over seven chained linear layers with one global g (Alg. 2), composed from the per-layer C-ABI calls.

Every linear-layer operation (base forward, subspace extraction, factored perturbed forward, fused
cross-entropy, the scalar g, the rank-r update) is a library call, and so are the in-place dense Gaussian sweeps of
the normalisation gains (the parameters that are not linear-layer weights); what sits between the layers
(embedding lookup, RMS normalisation, SiLU gate, residual sum: not steps of the method) is a few torch ops
here, fp32 arithmetic rounded to bf16 where the oracle rounds.  In the perturbed passes every layer reads
activations that already carry the perturbations of the layers before it, so the three passes share
nothing but the bases.
"""
import numpy as np
import pytest
import torch

from oracle import agzo as oagzo
from oracle import stack as ostack
from paper_2601_17261_amd import binding, synth

pytestmark = pytest.mark.gpu

R, K = 16, 3
LR = float(np.float32(1e-3))


def rel(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


class GpuStack:
    def __init__(self, ctx, params, ids, storage):
        self.ctx = ctx
        self.dt = torch.bfloat16 if storage == "bf16" else torch.float32
        self.nb = params["n_blocks"]
        self.names = ostack.layer_names(self.nb)
        self.E = torch.from_numpy(params["E"]).to("cuda", self.dt)
        self.W = {nm: torch.from_numpy(params[nm]).to("cuda", self.dt) for nm in self.names}
        self.ids = torch.from_numpy(ids.reshape(-1)).cuda()
        self.tgt = torch.from_numpy(ostack.shifted_targets(ids).astype(np.int32)).cuda()
        self.gains = {nm: torch.from_numpy(params[nm]).cuda() for nm in ostack.gain_names(params)}      # fp32
        self.B = {}
        self.L = {}

    def linear(self, nm, x, sign, eps, seeds, loss_dev=None):
        """One linear layer of one pass: sign 0 = unperturbed (and extract this layer's basis), +-1 = perturbed."""
        W = self.W[nm]
        head = nm[0] == "head"
        Y = None if head else torch.empty(x.shape[0], W.shape[0], dtype=self.dt, device="cuda")
        L = self.L[nm] = binding.make_layer(W, x, R, Y=Y)
        loss = binding.make_loss(self.tgt, kind=binding.LOSS_CE) if head else None
        if sign == 0:
            self.ctx.layer_forward_sketch(L, W, x, Y, binding.SKETCH_NONE, None, seeds[nm], None, loss, loss_dev)
            self.B[nm] = torch.empty(W.shape[1], R, dtype=torch.float32, device="cuda")
            self.ctx.basis(L, x, K, seeds[nm], None, 0, self.B[nm])
        else:
            self.ctx.perturbed_forward(L, W, x, self.B[nm], seeds[nm], sign * eps, Y, loss, loss_dev)
        return Y

    def rms(self, h, name):
        x = h.double()
        y = x * torch.rsqrt(x.pow(2).mean(dim=1, keepdim=True) + 1e-6)
        if name in self.gains:
            y = y * self.gains[name].double()[None, :]
        return y.to(self.dt)

    def run_pass(self, sign, eps, seeds, loss_dev):
        # the glue is evaluated in fp64 and rounded once to the storage type, like the oracle's, so that the
        # comparison is about the library's layers
        h = self.E[self.ids]
        for b in range(self.nb):
            n = self.rms(h, ("norm", b))
            a = self.linear(("gate", b), n, sign, eps, seeds)
            u = self.linear(("up", b), n, sign, eps, seeds)
            m = (torch.nn.functional.silu(a.double()) * u.double()).to(self.dt)
            d = self.linear(("down", b), m, sign, eps, seeds)
            h = (h.double() + d.double()).to(self.dt)
        self.linear(("head", 0), self.rms(h, ("norm_f", 0)), sign, eps, seeds, loss_dev)

    def step(self, eps, lr, seeds, flags=0):
        out = torch.zeros(4, dtype=torch.float64, device="cuda")
        def sweep_gains(scale, g_dev=None):
            # Alg. 2 for parameters that are not linear-layer weights: perturbed in place, restored, updated
            for nm, gv in self.gains.items():
                self.ctx.dense_perturb(gv, seeds[nm], scale, g_dev)

        self.run_pass(0, eps, seeds, out[0:1])
        sweep_gains(+eps)
        self.run_pass(+1, eps, seeds, out[1:2])
        if flags & binding.ONE_SIDED:
            sweep_gains(-eps)
        else:
            sweep_gains(-2.0 * eps)
            self.run_pass(-1, eps, seeds, out[2:3])
            sweep_gains(+eps)
        self.ctx.two_point(out, eps, flags)
        # every linear layer moves by the one global g: one batched call (the f32-storage stack: matrix by matrix inside it)
        self.ctx.update_many([(self.W[nm], self.B[nm], seeds[nm], lr, out[3:4]) for nm in self.names])
        sweep_gains(-lr, out[3:4])
        self.ctx.check()
        return out.cpu().numpy()


@pytest.fixture(scope="module")
def ctx():
    c = binding.Context()
    yield c
    c.close()


@pytest.fixture(scope="module")
def reduced_stack():
    return synth.mlp_stack_problem(31, n_blocks=2, hidden=2048, inter=6144, vocab=32000, n_seq=2, seq_len=128, gains=True)


# g is a difference of two ~10-sized losses.  With bf16 storage every stored activation is a rounding point, and where
# the library's fp32 accumulation and the oracle's fp64 fall on different sides of a bf16 boundary the two paths go on
# with activations one ulp apart: about 1e-3 of the ~1e7 stored values per pass, each moving the loss by ~1e-7 with a
# random sign, i.e. a few 1e-5 relative on each loss (measured 1.2e-5), which does not cancel between the passes.
# That floor is absolute in the losses, so the bf16 cases use a perturbation large enough to stand clear of it; parity
# does not need the loss to be linear in eps.  With fp32 storage the floor is ~1e-7 and eps = 1e-3 is checked tightly.
CASES = [
    # storage, eps, flags, tolerance on each loss (relative), on g (relative), floor of the loss difference (relative)
    ("f32", 1e-3, 0, 2e-6, 2e-3, 0.0),
    ("bf16", 1e-2, 0, 5e-5, 2e-2, 3e-5),
    ("bf16", 3e-2, binding.ONE_SIDED, 5e-5, 2e-2, 3e-5),
]


@pytest.mark.parametrize("storage,eps,flags,tol_l,tol_g,floor_l", CASES)
def test_reduced_mlp_stack_step_matches_oracle(ctx, reduced_stack, storage, eps, flags, tol_l, tol_g, floor_l):
    eps = float(np.float32(eps))
    params, ids = reduced_stack
    names = ostack.layer_names(2)
    seeds = {nm: 7000 + i for i, nm in enumerate(names + ostack.gain_names(params))}
    one_sided = bool(flags & binding.ONE_SIDED)
    o = ostack.agzo_stack_step(params, ids, R, K, eps, LR, seeds, act=storage, storage=storage, one_sided=one_sided)
    g_stack = GpuStack(ctx, params, ids, storage)
    got = g_stack.step(eps, LR, seeds, flags)
    # bases: compared through the projector (invariant to the conditioning of individual columns)
    for nm in names:
        Bg = g_stack.B[nm].double().cpu().numpy()
        assert rel(Bg @ (Bg.T @ o["B"][nm]), o["B"][nm]) < 2e-3, nm
    assert abs(got[0] - o["L0"]) < tol_l * o["L0"]
    assert abs(got[1] - o["Lp"]) < tol_l * o["Lp"]
    if one_sided:
        assert got[2] == 0.0
    else:
        assert abs(got[2] - o["Lm"]) < tol_l * o["Lm"]
    floor_g = floor_l * o["L0"] / (eps if one_sided else 2.0 * eps) * 2.0 ** 0.5
    assert abs(got[3] - o["g"]) < tol_g * abs(o["g"]) + floor_g, (got[3], o["g"], floor_g)
    # the gains moved along their dense directions by the same g (fp32, perturbed and restored in place)
    for nm in ostack.gain_names(params):
        got_gain = g_stack.gains[nm].double().cpu().numpy()
        want_gain = params[nm].astype(np.float64) - LR * got[3] * o["Z"][nm]
        assert np.abs(got_gain - want_gain).max() < 1e-6, nm
        assert np.abs(got_gain - params[nm]).max() > 1e-5, nm
        assert rel(got_gain - params[nm], o["W_new"][nm] - params[nm]) < tol_g + floor_g / abs(o["g"]), nm
    # the update: every layer moved along its own direction by the one global g
    for nm in names:
        Wg = g_stack.W[nm].double().cpu().numpy()
        want = o["W_new"][nm]
        assert rel(Wg, want) < (3e-3 if storage == "bf16" else 1e-5), nm
        assert (Wg != params[nm]).mean() > 0.01, nm                     # the update is not a no-op
        if storage == "bf16":
            # elementwise, with the scalar and basis this side computed (they differ from the oracle's within the
            # bounds above, and an increment of several ulps carries that difference): one rounding of the result
            # (an increment landing near a bf16 boundary may come out one ulp apart) plus the increment's own error
            # from the bf16 hi + lo split of its factors
            Bg = g_stack.B[nm].double().cpu().numpy()
            want = oagzo.round_bf16(params[nm].astype(np.float64) - LR * got[3] * (o["G"][nm] @ Bg.T))
            ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(want), 1e-30))) - 7)
            spread = np.abs(o["G"][nm]) @ np.abs(Bg).T
            bound = ulp * 1.0001 + LR * 2.0 ** -14 * abs(got[3]) * spread
            diff = np.abs(Wg - want)
            assert (diff <= bound).all(), (nm, float((diff / bound).max()))
            assert (diff > 0).mean() < 0.05, (nm, (diff > 0).mean())


def test_glue_kernels_match_the_oracle_model(ctx):
    """RMS normalisation, SiLU gate and residual sum between the linear layers: the library's single-pass kernels
    against the oracle's fp64 functions rounded once to bf16.  fp32 arithmetic can land on the other side of a bf16
    rounding boundary: isolated one-ulp differences only."""
    rng = np.random.default_rng(8)
    n, d = 70, 264

    def bf(a):
        return torch.from_numpy(synth.to_bf16_values(a)).to("cuda", torch.bfloat16)

    def check(got, want64):
        got = got.double().cpu().numpy()
        want = oagzo.round_bf16(want64)
        ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(want), 1e-30))) - 7)
        assert (np.abs(got - want) <= ulp * 1.0001).all()
        assert (got != want).mean() < 0.01

    x = 3.0 * rng.standard_normal((n, d))
    gain = (1.0 + 0.1 * rng.standard_normal(d)).astype(np.float32)
    xd = bf(x)
    x64 = xd.double().cpu().numpy()
    y = torch.empty_like(xd)
    ctx.glue_rmsnorm(xd, y)
    check(y, ostack.rmsnorm(x64))
    ctx.glue_rmsnorm(xd, y, torch.from_numpy(gain).cuda())
    check(y, ostack.rmsnorm(x64, gain))
    a, u = bf(2.0 * rng.standard_normal((n, d))), bf(rng.standard_normal((n, d)))
    m = torch.empty_like(a)
    ctx.glue_swiglu(a, u, m)
    check(m, ostack.silu(a.double().cpu().numpy()) * u.double().cpu().numpy())
    h = xd.clone()
    ctx.glue_add(h, a)
    check(h, x64 + a.double().cpu().numpy())
    # rows inside wider allocations, an empty tensor, and a row length that is not a multiple of 8
    wide = torch.zeros(n, d + 24, dtype=torch.bfloat16, device="cuda")
    ctx.glue_rmsnorm(xd, wide[:, 8:8 + d])
    check(wide[:, 8:8 + d], ostack.rmsnorm(x64))
    assert torch.count_nonzero(wide[:, :8]).item() == 0 and torch.count_nonzero(wide[:, 8 + d:]).item() == 0
    ctx.glue_add(torch.empty(0, 8, dtype=torch.bfloat16, device="cuda"), torch.empty(0, 8, dtype=torch.bfloat16, device="cuda"))
    with pytest.raises(binding.AgzoError) as e:
        ctx.glue_add(torch.zeros(4, 12, dtype=torch.bfloat16, device="cuda"), torch.zeros(4, 12, dtype=torch.bfloat16, device="cuda"))
    assert e.value.code == binding.EINVAL
    ctx.check()
