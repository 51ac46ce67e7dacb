"""Pins for the MLP-stack oracle (oracle/stack.py), against routines that share nothing with it:

* the unperturbed loss equals the same model written with torch's own functional ops in float64
  (rms_norm, silu, cross_entropy with ignore_index) when nothing is rounded;
* g is the directional derivative of that loss along the joint perturbation: it agrees with
  sum_l <dL/dW_l, Z_l> from torch autograd up to the O(eps^2) term of the central difference, and the
  one-sided form up to O(eps);
* with no blocks the stack is a single linear layer with a cross-entropy loss and the step reduces to
  oracle.agzo.agzo_step (itself pinned elsewhere);
* the update moves every layer along its own Z_l by the one global g; storage rounding only at the stated points.
"""
import numpy as np
import torch
import torch.nn.functional as F

from oracle import agzo as oagzo
from oracle import stack as ostack
from paper_2601_17261_amd import synth

R, K = 4, 2


def small(gains=False):
    return synth.mlp_stack_problem(11, n_blocks=2, hidden=48, inter=80, vocab=67, n_seq=3, seq_len=17, gains=gains)


def seeds_for(params, step=0):
    every = ostack.layer_names(params["n_blocks"]) + ostack.gain_names(params)
    return {nm: 1000 * step + i for i, nm in enumerate(every)}


def torch_loss(params, ids, weights):
    """The same model through torch.nn.functional, float64, nothing rounded."""
    ids_t = torch.from_numpy(ids.reshape(-1))
    h = torch.from_numpy(params["E"].astype(np.float64))[ids_t]
    for b in range(params["n_blocks"]):
        n = F.rms_norm(h, (h.shape[1],), weight=weights.get(("norm", b)), eps=1e-6)
        m = F.silu(F.linear(n, weights[("gate", b)])) * F.linear(n, weights[("up", b)])
        h = h + F.linear(m, weights[("down", b)])
    logits = F.linear(F.rms_norm(h, (h.shape[1],), weight=weights.get(("norm_f", 0)), eps=1e-6), weights[("head", 0)])
    tgt = torch.from_numpy(ostack.shifted_targets(ids))
    return F.cross_entropy(logits, tgt, ignore_index=-1)


def test_unperturbed_loss_matches_torch_functional_model():
    params, ids = small()
    w = {nm: torch.from_numpy(params[nm].astype(np.float64)) for nm in ostack.layer_names(2)}
    want = float(torch_loss(params, ids, w))
    got = ostack.forward(params, ids, act=None)
    assert abs(got - want) < 1e-12 * abs(want)
    # and the shifted targets: the last position of every sequence is ignored, the others look one ahead
    t = ostack.shifted_targets(ids).reshape(ids.shape)
    assert (t[:, -1] == -1).all() and (t[:, :-1] == ids[:, 1:]).all()


def test_g_is_the_directional_derivative_along_the_joint_perturbation():
    params, ids = small()
    names = ostack.layer_names(2)
    seeds = seeds_for(params)
    w = {nm: torch.from_numpy(params[nm].astype(np.float64)).requires_grad_(True) for nm in names}
    torch_loss(params, ids, w).backward()
    o = ostack.agzo_stack_step(params, ids, R, K, 1e-4, 0.0, seeds, act=None, storage="f32")
    want = sum(float((w[nm].grad.numpy() * o["Z"][nm]).sum()) for nm in names)
    assert abs(o["g"] - want) < 1e-5 * abs(want)
    # every layer contributes: leaving one layer's perturbation out changes the derivative
    for nm in names:
        assert abs(float((w[nm].grad.numpy() * o["Z"][nm]).sum())) > 1e-6 * abs(want)
    o1 = ostack.agzo_stack_step(params, ids, R, K, 1e-4, 0.0, seeds, act=None, storage="f32", one_sided=True)
    assert abs(o1["g"] - want) < 5e-2 * abs(want) and o1["Lm"] == 0.0
    assert abs(o1["g"] - want) > abs(o["g"] - want)          # the one-sided form carries the O(eps) term


def test_gains_take_the_dense_branch_with_the_same_global_g():
    params, ids = small(gains=True)
    every = ostack.layer_names(2) + ostack.gain_names(params)
    assert len(ostack.gain_names(params)) == 3
    seeds = seeds_for(params)
    w = {nm: torch.from_numpy(params[nm].astype(np.float64)).requires_grad_(True) for nm in every}
    loss = torch_loss(params, ids, w)
    assert abs(ostack.forward(params, ids, act=None) - loss.item()) < 1e-12 * loss.item()
    loss.backward()
    lr = 0.01
    o = ostack.agzo_stack_step(params, ids, R, K, 1e-4, lr, seeds, act=None, storage="f32")
    want = sum(float((w[nm].grad.numpy() * o["Z"][nm]).sum()) for nm in every)
    assert abs(o["g"] - want) < 1e-5 * abs(want)
    gain_part = sum(float((w[nm].grad.numpy() * o["Z"][nm]).sum()) for nm in ostack.gain_names(params))
    assert abs(gain_part) > 1e-3 * abs(want)                   # the gains' share of the derivative is not negligible
    for nm in ostack.gain_names(params):
        Rg = oagzo.dense_perturbation(seeds[nm], 1, 48)[0]     # a dense direction of the gain's own shape
        np.testing.assert_array_equal(o["Z"][nm], Rg)
        np.testing.assert_allclose(o["W_new"][nm], params[nm] - lr * o["g"] * Rg, rtol=0, atol=1e-7)
    # without gains in params the model is the gain-free one
    p0, _ = small(gains=False)
    for nm in ostack.layer_names(2):
        np.testing.assert_array_equal(p0[nm], params[nm])


def test_bases_come_from_each_layers_own_unperturbed_input():
    params, ids = small()
    seeds = seeds_for(params)
    o = ostack.agzo_stack_step(params, ids, R, K, 1e-3, 1e-2, seeds, act="bf16", storage="bf16")
    for nm in ostack.layer_names(2):
        X = o["inputs"][nm]
        assert X.shape == (ids.size, params[nm].shape[1])
        np.testing.assert_array_equal(X, oagzo.round_bf16(X))            # stored activations are bf16 values
        B = oagzo.subspace_extract(X, R, K, seeds[nm])["B"]
        np.testing.assert_array_equal(o["B"][nm], B)
        np.testing.assert_allclose(B.T @ B, np.eye(R), atol=1e-12)
    # gate and up of a block read the same tensor; down reads the gated product
    np.testing.assert_array_equal(o["inputs"][("gate", 1)], o["inputs"][("up", 1)])
    assert o["inputs"][("down", 0)].shape[1] == 80


def test_no_blocks_reduces_to_the_single_layer_step():
    params, ids = synth.mlp_stack_problem(5, n_blocks=0, hidden=40, inter=8, vocab=53, n_seq=2, seq_len=19)
    seeds = {("head", 0): 77}
    o = ostack.agzo_stack_step(params, ids, R, K, 1e-3, 1e-2, seeds, act="bf16", storage="bf16")
    X = oagzo.round_bf16(ostack.rmsnorm(params["E"].astype(np.float64)[ids.reshape(-1)]))
    s = oagzo.agzo_step(params[("head", 0)], X, ostack.shifted_targets(ids), R, K, 1e-3, 1e-2, 77, loss="ce", storage="bf16")
    for k in ("L0", "Lp", "Lm", "g"):
        assert o[k] == s[k]
    np.testing.assert_array_equal(o["W_new"][("head", 0)], s["W_new"])


def test_update_uses_one_global_g_and_each_layers_own_direction():
    params, ids = small()
    seeds = seeds_for(params, step=3)
    lr = 0.05
    o = ostack.agzo_stack_step(params, ids, R, K, 1e-3, lr, seeds, act="bf16", storage="f32")
    for nm in ostack.layer_names(2):
        step = (params[nm].astype(np.float64) - o["W_new"][nm]) / (lr * o["g"])
        np.testing.assert_allclose(step, o["Z"][nm], atol=2e-4 * np.abs(o["Z"][nm]).max())
        assert np.linalg.matrix_rank(o["Z"][nm]) == R
    # with a small enough step the loss goes down along -g Z (g Z correlates with the gradient, Eq. 10)
    new = dict(params)
    for nm in ostack.layer_names(2):
        new[nm] = o["W_new"][nm]
    assert ostack.forward(new, ids, act=None) < ostack.forward(params, ids, act=None)


def test_activation_guided_directions_align_with_the_true_gradient():
    """Thm 5.4 / Cor. 5.5 on every layer of the stack, against autograd's gradient: the mean of |cos(Z_l, grad_l)| over
    seeds is beta_{d_out r} times the mean captured energy |grad_l B_l| / |grad_l| (G is independent of the basis), it
    beats the dense direction's beta_{d_out d_in} on every layer, and the power steps raise the captured energy (the shape of
    the paper's ablation over K: most of the gain comes with the first step)."""
    import math
    params, ids = small()
    names = ostack.layer_names(2)
    w = {nm: torch.from_numpy(params[nm].astype(np.float64)).requires_grad_(True) for nm in names}
    torch_loss(params, ids, w).backward()
    inputs = {}
    ostack.forward(params, ids, act=None, record=inputs)
    beta = lambda D: math.exp(math.lgamma(D / 2.0) - math.lgamma((D + 1) / 2.0)) / math.sqrt(math.pi)
    n = 300
    for nm in names:
        grad = w[nm].grad.numpy()
        d_out, d_in = grad.shape
        gn = np.linalg.norm(grad)
        cs, ratio, ratio0 = np.empty(n), np.empty(n), np.empty(n)
        for s in range(n):
            B = oagzo.subspace_extract(inputs[nm], R, K, 7000 + s)["B"]
            Z, _ = oagzo.perturbation(B, 7000 + s, d_out)
            cs[s] = abs(float((Z * grad).sum())) / (np.linalg.norm(Z) * gn)
            ratio[s] = np.linalg.norm(grad @ B) / gn
            ratio0[s] = np.linalg.norm(grad @ oagzo.subspace_extract(inputs[nm], R, 0, 7000 + s)["B"]) / gn
        b = beta(d_out * R)
        sigma = math.sqrt(1.0 / (d_out * R) - b * b) * ratio.mean() + b * ratio.std()
        assert abs(cs.mean() - b * ratio.mean()) < 4.0 * sigma / math.sqrt(n), nm
        assert cs.mean() > 1.5 * beta(d_out * d_in), nm
        assert ratio.mean() > ratio0.mean() + 0.05, nm      # K = 2 power steps against none: 0.10 - 0.14 more of the energy here

