"""Pins for the oracle's AGZO step (CPU only).

Each test checks the oracle against something it does not define itself:
Eq. 5-6 (gradient lies in the activations' span) by brute-force finite
differences, uniqueness of the positive-diagonal QR, the library SVD as the
K -> infinity limit of Alg. 1, the exact Taylor expansion of a quadratic
loss for the two-point scalar, Prop. 5.1 (mean of the estimator is the
projected gradient), library cross-entropy and library bf16 rounding.
"""
import math

import numpy as np
import torch

from oracle import agzo, philox
from paper_2601_17261_amd import synth


def _tiny(seed=0, n=7, d_in=12, d_out=5):
    rng = np.random.default_rng(seed)
    W = rng.standard_normal((d_out, d_in)) * 0.3
    X = rng.standard_normal((n, d_in))
    T = rng.standard_normal((n, d_out))
    return W, X, T


# --- Eq. 5-6 -----------------------------------------------------------------
def test_gradient_identity_and_rowspace_brute_force():
    W, X, T = _tiny()           # N = 7 < d_in = 12: the activations span a strict subspace
    grad = agzo.mse_grad(X, W, T)
    fd = np.zeros_like(W)
    h = 1e-5
    for i in range(W.shape[0]):
        for j in range(W.shape[1]):
            Wp = W.copy(); Wp[i, j] += h
            Wm = W.copy(); Wm[i, j] -= h
            fd[i, j] = (agzo.mse_loss(agzo.forward(X, Wp), T) - agzo.mse_loss(agzo.forward(X, Wm), T)) / (2 * h)
    np.testing.assert_allclose(grad, fd, rtol=1e-7, atol=1e-9)
    # row(grad) inside the span of the tokens (rows of X = columns of H)
    _, s, Vt = np.linalg.svd(X, full_matrices=True)
    null = Vt[len(s):]                       # d_in - N directions orthogonal to every token
    assert np.linalg.norm(grad @ null.T) < 1e-12 * np.linalg.norm(grad)


def test_forward_layout_is_y_equals_W_h():
    W, X, _ = _tiny()
    Y = agzo.forward(X, W)
    for t in (0, 3, 6):
        np.testing.assert_allclose(Y[t], W @ X[t], rtol=1e-13)


# --- QR ------------------------------------------------------------------------
def test_qr_pos_is_the_unique_positive_diagonal_factorisation():
    rng = np.random.default_rng(1)
    Y = rng.standard_normal((40, 6)) @ np.diag([5, 1, 3, 0.1, 2, 0.01])
    Q, R = agzo.qr_pos(Y)
    assert Q.shape == (40, 6) and R.shape == (6, 6)
    assert np.linalg.norm(Q.T @ Q - np.eye(6)) < 1e-13
    assert np.allclose(R, np.triu(R)) and (np.diag(R) > 0).all()
    np.testing.assert_allclose(Q @ R, Y, atol=1e-12)
    # independent route to the same unique factor: Cholesky of the Gram matrix
    Rc = np.linalg.cholesky(Y.T @ Y).T
    np.testing.assert_allclose(R, Rc, rtol=1e-7)
    np.testing.assert_allclose(Q, Y @ np.linalg.inv(Rc), atol=1e-7)


# --- Alg. 1 --------------------------------------------------------------------
def _subspace_gap(B, U):
    return np.linalg.norm(B @ B.T - U @ U.T, 2)


def test_subspace_extract_orthonormal_and_inside_activation_span():
    W, X, _ = _tiny(2, n=9, d_in=20)
    for init in ("token", "feature"):
        ext = agzo.subspace_extract(X, r=3, K=3, seed=5, init=init)
        B = ext["B"]
        assert B.shape == (20, 3)
        assert np.linalg.norm(B.T @ B - np.eye(3)) < 1e-12
        for Q in ext["Q"]:
            assert np.linalg.norm(Q.T @ Q - np.eye(3)) < 1e-12
        assert len(ext["Q"]) == 3 and len(ext["S"]) == 4
        P = np.linalg.pinv(X) @ X               # projector on the tokens' span in feature space
        assert np.linalg.norm(B - P @ B) < 1e-10


def test_first_sketch_is_H_times_omega():
    W, X, _ = _tiny(3, n=6, d_in=10)
    S0 = agzo.range_sketch(X, 4, seed=11)
    om = philox.normal(11, philox.TAG_OMEGA, 6, 4).astype(np.float64)
    ref = np.zeros((10, 4))
    for d in range(10):
        for k in range(4):
            ref[d, k] = sum(X[t, d] * om[t, k] for t in range(6))
    np.testing.assert_allclose(S0, ref, rtol=1e-12, atol=1e-13)
    ext = agzo.subspace_extract(X, 4, K=0, seed=11)
    np.testing.assert_allclose(ext["S"][0], ref, rtol=1e-12, atol=1e-13)
    Q, _ = np.linalg.qr(ref)
    assert _subspace_gap(ext["B"], Q) < 1e-12    # K = 0: plain range finder


def test_exact_low_rank_activations_are_recovered_for_any_K():
    rng = np.random.default_rng(4)
    V, _ = np.linalg.qr(rng.standard_normal((30, 3)))
    X = rng.standard_normal((50, 3)) @ np.diag([3.0, 2.0, 1.0]) @ V.T      # rank exactly 3
    for K in (0, 1, 3):
        B = agzo.subspace_extract(X, 3, K, seed=9)["B"]
        assert _subspace_gap(B, V) < 1e-9


def test_power_iteration_converges_to_library_svd():
    """Planted spectrum with a gap (the small fp32 workload): the distance to the top-r
    right-singular subspace of X (= top-r left singular vectors of H) shrinks with K."""
    _, X, _ = synth.single_layer_problem(0, 512, 256, 256, kind="lowrank")
    X = X.astype(np.float64)
    _, _, Vt = np.linalg.svd(X, full_matrices=False)
    U = Vt[:4].T
    gaps = [_subspace_gap(agzo.subspace_extract(X, 4, K, seed=0)["B"], U) for K in (0, 1, 3, 6, 12)]
    assert all(b < a for a, b in zip(gaps, gaps[1:]))
    assert gaps[-1] < 5e-3 and gaps[2] < gaps[0] / 5
    # one power step multiplies each direction by its squared singular value
    Q = agzo.subspace_extract(X, 4, 1, seed=0)["Q"][0]
    np.testing.assert_allclose(agzo.power_sketch(X, Q), (X.T @ X) @ Q, rtol=1e-10, atol=1e-12)


# --- Eq. 7 -----------------------------------------------------------------------
def test_perturbation_lives_in_the_subspace():
    W, X, T = _tiny(5, n=20, d_in=16, d_out=6)
    out = agzo.agzo_step(W, X, T, r=3, K=3, eps=1e-3, lr=1e-2, seed=77)
    B, Z, G = out["B"], out["Z"], out["G"]
    np.testing.assert_array_equal(G, philox.normal(77, philox.TAG_G, 6, 3).astype(np.float64))
    I = np.eye(16)
    assert np.linalg.norm(Z @ (I - B @ B.T)) < 1e-12 * np.linalg.norm(Z)
    assert abs(np.linalg.norm(Z) - np.linalg.norm(G)) < 1e-12 * np.linalg.norm(G)
    assert np.linalg.matrix_rank(Z) <= 3
    # the update moves W only inside span(B), up to the one fp32 rounding of the stored result
    assert np.linalg.norm((out["W_new"] - W) @ (I - B @ B.T)) < 2.0 ** -23 * np.linalg.norm(W)
    assert np.linalg.norm(out["W_new"] - W) > 1e-4 * np.linalg.norm(W)
    for i in (0, 5):
        for j in (0, 15):
            assert abs(Z[i, j] - sum(G[i, k] * B[j, k] for k in range(3))) < 1e-14


def test_factored_forward_equals_materialised():
    W, X, T = _tiny(6, n=20, d_in=16, d_out=6)
    out = agzo.agzo_step(W, X, T, r=3, K=2, eps=0.05, lr=1e-2, seed=8)
    P = X @ out["B"]
    np.testing.assert_allclose(out["Yp"], out["Y0"] + 0.05 * P @ out["G"].T, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(out["Ym"], out["Y0"] - 0.05 * P @ out["G"].T, rtol=1e-12, atol=1e-13)


# --- Eq. 10 / Alg. 2 ---------------------------------------------------------------
def test_two_point_scalar_closed_form_on_quadratic():
    W, X, T = _tiny(7, n=20, d_in=16, d_out=6)
    grad = agzo.mse_grad(X, W, T)
    for eps in (1e-3, 0.1, 1.0):
        out = agzo.agzo_step(W, X, T, r=3, K=3, eps=eps, lr=1e-2, seed=21)
        dd = float(np.sum(grad * out["Z"]))                       # <grad, Z>_F
        assert abs(out["g"] - dd) < 1e-9 * max(1.0, abs(dd)) / min(1.0, eps)
        np.testing.assert_allclose(dd, np.sum((grad @ out["B"]) * out["G"]), rtol=1e-10)
        one = agzo.agzo_step(W, X, T, r=3, K=3, eps=eps, lr=1e-2, seed=21, one_sided=True)
        curv = (eps / T.size) * np.linalg.norm(X @ out["Z"].T) ** 2
        assert abs(one["g"] - (dd + curv)) < 1e-8 * max(1.0, abs(dd + curv)) / min(1.0, eps)
        assert one["L0"] == out["L0"]


def test_update_is_a_descent_step_with_slope_minus_g_squared():
    W, X, T = _tiny(8, n=20, d_in=16, d_out=6)
    lr = 1e-7
    out = agzo.agzo_step(W, X, T, r=3, K=3, eps=1e-3, lr=lr, seed=3, storage="f32")
    Wn = W - lr * out["g"] * out["Z"]        # un-rounded update
    slope = (agzo.mse_loss(agzo.forward(X, Wn), T) - out["L0"]) / lr
    assert abs(slope + out["g"] ** 2) < 1e-4 * out["g"] ** 2
    np.testing.assert_allclose(out["W_new"], Wn.astype(np.float32).astype(np.float64), rtol=0, atol=0)


def test_estimator_mean_is_projected_gradient():
    """Prop. 5.1 with a quadratic loss (no smoothing bias for the central difference):
    mean over seeds of g Z -> grad B B^T."""
    W, X, T = _tiny(9, n=10, d_in=8, d_out=3)
    B = agzo.subspace_extract(X, 2, 3, seed=1)["B"]
    grad = agzo.mse_grad(X, W, T)
    want = grad @ B @ B.T
    acc = np.zeros_like(W)
    n = 6000
    for s in range(n):
        out = agzo.agzo_step(W, X, T, r=2, K=3, eps=1e-2, lr=0.0, seed=10_000 + s, B=B)
        acc += out["g"] * out["Z"]
    err = np.linalg.norm(acc / n - want) / np.linalg.norm(want)
    assert err < 6.0 * math.sqrt((3 * 2 + 2) / n)      # ~ sqrt((D+2)/n) relative noise, D = d_out r


def _beta(D):
    return math.exp(math.lgamma(D / 2.0) - math.lgamma((D + 1) / 2.0)) / math.sqrt(math.pi)


def test_expected_cosine_is_beta_times_captured_gradient_energy():
    """Thm 5.4 (expected cosine of the noiseless estimator): for a fixed orthonormal basis A,
    E_R |cos(R A^T, grad)| = beta_{d_out r} |grad A|_F / |grad|_F, beta_D = Gamma(D/2) / (sqrt(pi) Gamma((D+1)/2));
    the paper prints beta_D's bounds sqrt(2/(pi D)) <= beta_D <= sqrt(2/(pi (D-1)))."""
    W, X, T = _tiny(4, n=10, d_in=8, d_out=3)
    r = 2
    B = agzo.subspace_extract(X, r, 3, seed=1)["B"]
    grad = agzo.mse_grad(X, W, T)
    D = 3 * r
    beta = _beta(D)
    assert math.sqrt(2 / (math.pi * D)) <= beta <= math.sqrt(2 / (math.pi * (D - 1)))
    ratio = np.linalg.norm(grad @ B) / np.linalg.norm(grad)
    assert 0.3 < ratio < 1.0                       # the basis captures part of the gradient, not all: the factor matters
    n = 8000
    cs = np.empty(n)
    for s in range(n):
        Z, _ = agzo.perturbation(B, 20_000 + s, 3)
        cs[s] = abs(float((Z * grad).sum())) / (np.linalg.norm(Z) * np.linalg.norm(grad))
    sigma = ratio * math.sqrt(1.0 / D - beta ** 2)
    assert abs(cs.mean() - beta * ratio) < 4.0 * sigma / math.sqrt(n)
    # the dense direction on the same layer (Cor. 5.5): beta_{d_out d_in}, smaller
    cd = np.empty(n)
    for s in range(n):
        Rd = agzo.dense_perturbation(20_000 + s, 3, 8)
        cd[s] = abs(float((Rd * grad).sum())) / (np.linalg.norm(Rd) * np.linalg.norm(grad))
    b24 = _beta(24)
    assert abs(cd.mean() - b24) < 4.0 * math.sqrt((1.0 / 24 - b24 ** 2) / n)
    assert cs.mean() > 1.3 * cd.mean()


# --- losses, rounding ---------------------------------------------------------------
def test_ce_matches_library_with_ignored_rows():
    rng = np.random.default_rng(10)
    z = rng.standard_normal((9, 13)) * 3
    t = np.array([0, 12, -1, 5, 5, -1, 7, 1, 2])
    ref = torch.nn.functional.cross_entropy(torch.from_numpy(z), torch.from_numpy(t), ignore_index=-1).item()
    assert abs(agzo.ce_loss(z, t) - ref) < 1e-12
    assert abs(agzo.mse_loss(z, z + 2.0) - 4.0) < 1e-12


def test_round_bf16_matches_library_and_ties_to_even():
    rng = np.random.default_rng(11)
    a = (rng.standard_normal(20000) * np.exp(rng.uniform(-8, 8, 20000))).astype(np.float32)
    ref = torch.from_numpy(a).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(agzo.round_bf16(a.astype(np.float64)), ref)
    # exact ties: 1 + 2^-8 is halfway between 1 and 1 + 2^-7 -> even mantissa (1.0)
    assert agzo.round_bf16(np.array([1.0 + 2.0 ** -8]))[0] == 1.0
    assert agzo.round_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6
    assert agzo.round_bf16(np.array([0.0]))[0] == 0.0


def test_bf16_storage_and_inplace_schedule():
    W, X, T = synth.single_layer_problem(3, 64, 32, 24, kind="rmsnorm", storage="bf16")
    W64, X64 = W.astype(np.float64), X.astype(np.float64)
    out = agzo.agzo_step(W64, X64, T, r=4, K=3, eps=1e-3, lr=1e-2, seed=5, storage="bf16")
    np.testing.assert_array_equal(out["W_new"], agzo.round_bf16(out["W_new"]))
    np.testing.assert_array_equal(out["W_new"], agzo.round_bf16(W64 - 1e-2 * out["g"] * out["Z"]))
    # in fp32 storage the in-place schedule agrees with the factored one up to fp32 rounding of W
    W32, X32, T32 = synth.single_layer_problem(3, 64, 32, 24, kind="rmsnorm", storage="f32")
    a = agzo.agzo_step(W32, X32, T32, r=4, K=3, eps=1e-3, lr=1e-2, seed=5, storage="f32")
    b = agzo.agzo_step_inplace(W32, X32, T32, a["B"], 1e-3, 1e-2, 5, storage="f32")
    assert abs(a["g"] - b["g"]) < 2e-3 * abs(a["g"])
    assert np.linalg.norm(a["W_new"] - b["W_new"]) < 1e-6 * np.linalg.norm(a["W_new"])
    # in bf16 storage most of an eps-sized perturbation is rounded away: the schedules differ
    c = agzo.agzo_step_inplace(W64, X64, T, out["B"], 1e-3, 1e-2, 5, storage="bf16")
    np.testing.assert_array_equal(c["Wp"], agzo.round_bf16(W64 + 1e-3 * out["Z"]))
    assert c["L0"] == out["L0"]
    # the printed, one-sided form of the same schedule agrees with the factored one-sided step in fp32 storage
    a1 = agzo.agzo_step(W32, X32, T32, r=4, K=3, eps=1e-3, lr=1e-2, seed=5, storage="f32", one_sided=True)
    b1 = agzo.agzo_step_inplace(W32, X32, T32, a1["B"], 1e-3, 1e-2, 5, storage="f32", one_sided=True)
    assert abs(a1["g"] - b1["g"]) < 2e-3 * abs(a1["g"]) and b1["Lm"] == 0.0 and b1["Lp"] == b["Lp"]
    assert np.linalg.norm(a1["W_new"] - b1["W_new"]) < 1e-6 * np.linalg.norm(a1["W_new"])
    assert abs(a1["g"] - a["g"]) > 1e-6 * abs(a["g"])          # and is not the central estimate


# --- Eq. 7, second branch: dense Gaussian perturbation of other parameters ---------------------
def test_dense_branch_moments_and_stream_separation():
    R = agzo.dense_perturbation(9, 512, 512)
    n = R.size
    assert abs(R.mean()) < 4.0 / math.sqrt(n)
    assert abs(R.var() - 1.0) < 4.0 * math.sqrt(2.0 / n)
    assert abs((R ** 4).mean() - 3.0) < 4.0 * math.sqrt(96.0 / n)
    G = agzo.gaussian_factor(9, 512, 512)             # same seed, the linear branch's stream
    assert abs((R * G).mean()) < 4.0 / math.sqrt(n)   # the two streams are uncorrelated
    assert not np.array_equal(R[:4, :4], agzo.dense_perturbation(10, 4, 4))
    # a block's values do not depend on how many rows or columns are asked for
    np.testing.assert_array_equal(R[:7, :9], agzo.dense_perturbation(9, 7, 9))


def test_dense_sweeps_compose_and_restore():
    rng = np.random.default_rng(3)
    th = rng.standard_normal((6, 10)).astype(np.float32).astype(np.float64)
    eps = 1e-3
    R = agzo.dense_perturbation(21, 6, 10)
    plus = agzo.dense_apply(th, 21, eps, "f32")
    np.testing.assert_allclose(plus, th + eps * R, rtol=0, atol=2.0 ** -23 * np.abs(th).max())
    back = agzo.dense_apply(agzo.dense_apply(plus, 21, -2 * eps, "f32"), 21, eps, "f32")
    assert np.abs(back - th).max() <= 2.0 ** -22 * np.abs(th).max()          # restored up to fp32 rounding
    # a 1-D block is one row of the same stream
    v = agzo.dense_apply(th[0], 21, 0.5, "f32")
    np.testing.assert_array_equal(v, agzo.dense_apply(th[:1], 21, 0.5, "f32")[0])
    # bf16 storage: a perturbation below half an ulp is swallowed, one well above it is not
    w = synth.to_bf16_values(np.full((4, 8), 0.02, dtype=np.float32)).astype(np.float64)
    np.testing.assert_array_equal(agzo.dense_apply(w, 5, 1e-7, "bf16"), w)
    assert (agzo.dense_apply(w, 5, 1e-2, "bf16") != w).mean() > 0.9


def test_dense_two_point_estimator_mean_is_the_gradient():
    # f(theta) = 0.5 |theta - a|^2: the central difference along R is exactly <grad, R>, and E[<grad, R> R] = grad
    rng = np.random.default_rng(8)
    th, a = rng.standard_normal((2, 5)), rng.standard_normal((2, 5))
    f = lambda t: 0.5 * float(((t - a) ** 2).sum())
    eps, n = 1e-3, 6000
    acc = np.zeros_like(th)
    for s in range(n):
        R = agzo.dense_perturbation(1000 + s, 2, 5)
        g = (f(th + eps * R) - f(th - eps * R)) / (2 * eps)
        assert abs(g - float(((th - a) * R).sum())) < 1e-9
        acc += g * R
    err = np.linalg.norm(acc / n - (th - a)) / np.linalg.norm(th - a)
    assert err < 4.0 * math.sqrt((th.size + 1.0) / n)


def test_dense_step_is_the_two_point_estimator_along_a_dense_direction():
    # squared error is quadratic in W, so the central difference along R is exactly <grad, R>
    rng = np.random.default_rng(12)
    X = rng.standard_normal((40, 12))
    W = (0.1 * rng.standard_normal((7, 12))).astype(np.float32).astype(np.float64)
    T = rng.standard_normal((40, 7))
    eps, lr, seed = 1e-3, 1e-2, 77
    R = agzo.dense_perturbation(seed, 7, 12)
    dd = float((agzo.mse_grad(X, W, T) * R).sum())
    o = agzo.dense_step(W, X, T, eps, lr, seed, storage="f32")
    assert abs(o["g"] - dd) < 2e-4 * abs(dd)                  # fp32 storage of the perturbed weights: 2^-24 |W| / eps
    assert np.abs(o["W_restored"] - W).max() <= 2.0 ** -22 * np.abs(W).max()
    np.testing.assert_allclose(o["W_new"] - o["W_restored"], -lr * o["g"] * R, rtol=0, atol=2.0 ** -23 * np.abs(W).max())
    # one-sided form: differs from the central one by the curvature term, eps/2 R^T H R
    o1 = agzo.dense_step(W, X, T, eps, lr, seed, storage="f32", one_sided=True)
    curv = (eps / 2.0) * 2.0 * float(((X @ R.T) ** 2).sum()) / (40 * 7)
    assert abs(o1["g"] - (dd + curv)) < 2e-3 * abs(dd)
    assert o1["Lm"] == 0.0 and o["L0"] == 0.0


def test_dense_direction_alignment_with_a_fixed_vector():
    # Cor. 5.5's baseline: for an isotropic Gaussian direction in n dimensions, E|cos(R, v)| = Gamma(n/2) / (sqrt(pi) Gamma((n+1)/2))
    v = np.arange(1.0, 17.0).reshape(4, 4)
    n_trials = 6000
    cs = np.empty(n_trials)
    for s in range(n_trials):
        R = agzo.dense_perturbation(5000 + s, 4, 4)
        cs[s] = abs(float((R * v).sum())) / (np.linalg.norm(R) * np.linalg.norm(v))
    beta16 = math.gamma(8.0) / (math.sqrt(math.pi) * math.gamma(8.5))
    assert abs(beta16 - 0.20261) < 1e-5
    # var |cos| = 1/n - beta^2
    assert abs(cs.mean() - beta16) < 4.0 * math.sqrt((1.0 / 16 - beta16 ** 2) / n_trials)

