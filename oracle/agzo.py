"""Oracle: one AGZO step for a linear layer, in fp64 (test infrastructure only).

Written from the paper: Sec. 3.1 (Eq. 5-6, gradient = upstream-gradient times
activations), Sec. 4.1 (Alg. 1 SubspaceExtract, Eq. 7 perturbation, Eq. 10
estimator) and Alg. 2 (perturb, evaluate, regenerate, update).  Nothing here
is blocked, fused or reordered: each function is the definition written out
with numpy fp64 primitives (matmul, LAPACK QR).

Notation (repo letters; the paper's are in brackets):
  W [W_l]    d_out x d_in weights, y = W h, batched Y = X W^T
  X [H_l^T]  N x d_in activations, one token per row
  B [A_l]    d_in x r orthonormal activation basis
  G [R_l]    d_out x r iid N(0,1) left factor, regenerated from the seed
  Z [Delta]  = G B^T, the rank-r perturbation (Eq. 7)
  eps [mu], lr [eta], g = projected-gradient scalar (Alg. 2)

Readings taken where the paper is silent (each is listed with its reason in
the design notes of this repository):
  * QR is the thin factorisation with positive diagonal of R (unique for a
    full-column-rank argument), applied at every QR of Alg. 1;
  * the default scalar is the central difference (L+ - L-)/(2 eps); the
    one-sided form of Eq. 10 / Alg. 2, (L+ - L0)/eps, is a mode;
  * MSE is the mean over all N*d_out entries; CE is the mean over rows whose
    target is >= 0 of -log softmax(logits)[target];
  * with bf16 storage the updated weights are rounded once, to nearest even.

Pins live in tests/test_oracle_*.py.
"""
import numpy as np

from . import philox


# ----------------------------------------------------------------------------
# storage rounding
# ----------------------------------------------------------------------------
def round_bf16(a):
    """Round fp64/fp32 values to the nearest bfloat16 (ties to even); returns fp64."""
    # Round straight from fp64 (no fp32 stop-over, so no double rounding):
    # keep 8 significant bits of the mantissa.  Values here are far from the
    # bf16 subnormal and overflow ranges.
    x = np.asarray(a, dtype=np.float64)
    m, e = np.frexp(x)                      # x = m * 2^e, 0.5 <= |m| < 1
    q = np.rint(m * 256.0) / 256.0          # rint = ties-to-even
    return np.ldexp(q, e)


def round_storage(a, storage):
    if storage == "f32":
        return np.asarray(a, dtype=np.float64).astype(np.float32).astype(np.float64)
    if storage == "bf16":
        return round_bf16(a)
    raise ValueError(storage)


# ----------------------------------------------------------------------------
# Alg. 1: SubspaceExtract
# ----------------------------------------------------------------------------
def qr_pos(Y):
    """Thin QR of a tall matrix with diag(R) > 0 (Alg. 1, the two 'qr' steps)."""
    Q, R = np.linalg.qr(np.asarray(Y, dtype=np.float64), mode="reduced")
    s = np.sign(np.diag(R))
    s[s == 0] = 1.0
    return Q * s[None, :], R * s[:, None]


def range_sketch(X, r, seed):
    """First two steps of Alg. 1: Omega ~ N(0,1)^{N x r} from the seed, Y = H Omega = X^T Omega."""
    X = np.asarray(X, dtype=np.float64)
    omega = philox.normal(seed, philox.TAG_OMEGA, X.shape[0], r).astype(np.float64)
    return X.T @ omega


def power_sketch(X, Q):
    """Power step of Alg. 1: Y = H (H^T Q) = X^T (X Q)."""
    X = np.asarray(X, dtype=np.float64)
    return X.T @ (X @ np.asarray(Q, dtype=np.float64))


def subspace_extract(X, r, K, seed, init="token"):
    """Alg. 1.  Returns dict with S0 (first sketch), every intermediate Q and S, and B.

    init="token"   : the paper's start, Omega in token space (N x r), Y = X^T Omega.
    init="feature" : flagged variant, Q0 = Gaussian d_in x r, Y = X^T (X Q0).
    """
    X = np.asarray(X, dtype=np.float64)
    if init == "token":
        Y = range_sketch(X, r, seed)
    elif init == "feature":
        Q0 = philox.normal(seed, philox.TAG_Q0, X.shape[1], r).astype(np.float64)
        Y = power_sketch(X, Q0)
    else:
        raise ValueError(init)
    out = {"S": [Y], "Q": []}
    for _ in range(K):
        Q, _R = qr_pos(Y)
        out["Q"].append(Q)
        Y = power_sketch(X, Q)
        out["S"].append(Y)
    B, _R = qr_pos(Y)
    out["B"] = B
    return out


# ----------------------------------------------------------------------------
# Eq. 7: perturbation;  forward;  losses
# ----------------------------------------------------------------------------
def gaussian_factor(seed, d_out, r):
    """G [R_l]: d_out x r iid N(0,1) regenerated from the seed (Alg. 2)."""
    return philox.normal(seed, philox.TAG_G, d_out, r).astype(np.float64)


def perturbation(B, seed, d_out):
    """Z = G B^T, materialised (Eq. 7, linear-layer branch)."""
    B = np.asarray(B, dtype=np.float64)
    G = gaussian_factor(seed, d_out, B.shape[1])
    return G @ B.T, G


def dense_perturbation(seed, rows, cols):
    """R for a parameter block that is not a linear-layer weight (Eq. 7, second branch):
    iid N(0,1) of the block's own shape, regenerated from the seed (stream TAG_DENSE)."""
    return philox.normal(seed, philox.TAG_DENSE, rows, cols).astype(np.float64)


def dense_apply(theta, seed, coef, storage):
    """theta + coef R rounded to the storage type: one in-place sweep of Alg. 2 (perturb with
    +eps, restore with -eps, update with -lr g) for such a block.  A 1-D block is one row."""
    t = np.asarray(theta, dtype=np.float64)
    t2 = t.reshape(1, -1) if t.ndim == 1 else t
    out = round_storage(t2 + coef * dense_perturbation(seed, t2.shape[0], t2.shape[1]), storage)
    return out.reshape(t.shape)


def forward(X, W):
    """Y = X W^T (y = W h per token)."""
    return np.asarray(X, dtype=np.float64) @ np.asarray(W, dtype=np.float64).T


def mse_loss(Y, target):
    d = np.asarray(Y, dtype=np.float64) - np.asarray(target, dtype=np.float64)
    return float(np.mean(d * d))


def ce_loss(logits, target):
    """Mean over rows with target >= 0 of -log softmax(logits)[target] (natural log)."""
    z = np.asarray(logits, dtype=np.float64)
    t = np.asarray(target).astype(np.int64)
    keep = t >= 0
    if not keep.any():
        return 0.0
    z = z[keep]
    t = t[keep]
    m = z.max(axis=1)
    lse = m + np.log(np.exp(z - m[:, None]).sum(axis=1))
    return float(np.mean(lse - z[np.arange(z.shape[0]), t]))


def loss_value(Y, kind, target):
    if kind == "mse":
        return mse_loss(Y, target)
    if kind == "ce":
        return ce_loss(Y, target)
    raise ValueError(kind)


def mse_grad(X, W, target):
    """Analytic dL/dW of the MSE loss: (2/(N d_out)) (Y - Y*)^T X  (Eq. 5 with Q = dL/dY^T)."""
    X = np.asarray(X, dtype=np.float64)
    Y = forward(X, W)
    return (2.0 / Y.size) * (Y - np.asarray(target, dtype=np.float64)).T @ X


# ----------------------------------------------------------------------------
# Alg. 2: one AGZO iteration for a single linear layer
# ----------------------------------------------------------------------------
def agzo_step(W, X, target, r, K, eps, lr, seed, loss="mse", storage="f32",
              one_sided=False, init="token", B=None):
    """One AGZO step.  W, X hold storage-exact values (fp32 or bf16 numbers).

    Order follows Alg. 2: base forward with subspace extraction, perturbation
    Z = G B^T from the seed, perturbed evaluation(s) with W +/- eps Z kept in
    fp64 (never rounded), scalar g, update W' = W - lr g Z rounded once to the
    storage type.
    """
    W = np.asarray(W, dtype=np.float64)
    X = np.asarray(X, dtype=np.float64)
    ext = None
    if B is None:
        ext = subspace_extract(X, r, K, seed, init=init)
        B = ext["B"]
    Z, G = perturbation(B, seed, W.shape[0])
    Y0 = forward(X, W)
    Yp = forward(X, W + eps * Z)
    Ym = forward(X, W - eps * Z)
    L0 = loss_value(Y0, loss, target)
    Lp = loss_value(Yp, loss, target)
    Lm = loss_value(Ym, loss, target)
    g = (Lp - L0) / eps if one_sided else (Lp - Lm) / (2.0 * eps)
    W_new = round_storage(W - lr * g * Z, storage)
    return {"ext": ext, "B": B, "G": G, "Z": Z, "Y0": Y0, "Yp": Yp, "Ym": Ym,
            "L0": L0, "Lp": Lp, "Lm": Lm, "g": g, "W_new": W_new}


def apply_rank_r(W, B, seed, coef, storage):
    """W + coef * G B^T, rounded to storage: one in-place sweep of Alg. 2 (perturb / restore / update)."""
    W = np.asarray(W, dtype=np.float64)
    Z, _ = perturbation(B, seed, W.shape[0])
    return round_storage(W + coef * Z, storage)


def agzo_step_inplace(W, X, target, B, eps, lr, seed, loss="mse", storage="f32", one_sided=False):
    """The paper's literal in-place schedule (Alg. 2: perturb in place, evaluate,
    restore and update), extended to the central difference: every sweep stores
    W in the storage type, so in bf16 this is a *different* computation from
    agzo_step (the perturbation is partly rounded away) and has its own parity.
    one_sided: exactly Alg. 2 as printed: one perturbed evaluation, g = (L+ - L0) / eps, and the
    last line as ONE sweep over the still-perturbed weights, W <- W - eps Z - lr g Z (one rounding
    to storage).  The central form has no printed last line; it restores (+eps from the minus
    side) and updates in two rounded sweeps."""
    W0 = np.asarray(W, dtype=np.float64)
    L0 = loss_value(forward(X, W0), loss, target)
    Wp = apply_rank_r(W0, B, seed, +eps, storage)
    Lp = loss_value(forward(X, Wp), loss, target)
    if one_sided:
        Wm, Lm = None, 0.0
        g = (Lp - L0) / eps
        W_new = apply_rank_r(Wp, B, seed, -(eps + lr * g), storage)   # restore and update, one sweep
    else:
        Wm = apply_rank_r(Wp, B, seed, -2.0 * eps, storage)
        Lm = loss_value(forward(X, Wm), loss, target)
        g = (Lp - Lm) / (2.0 * eps)
        Wr = apply_rank_r(Wm, B, seed, +eps, storage)      # restore
        W_new = apply_rank_r(Wr, B, seed, -lr * g, storage)    # update
    return {"L0": L0, "Lp": Lp, "Lm": Lm, "g": g, "W_new": W_new, "Wp": Wp, "Wm": Wm}


def dense_step(W, X, target, eps, lr, seed, loss="mse", storage="f32", one_sided=False):
    """Alg. 2 for a parameter block taken through the other branch of Eq. 7 (a dense Gaussian R of the block's
    own shape instead of G B^T), here the weight of one linear layer: the estimator the paper compares against.
    There is no factored form, so the schedule is the literal one: every sweep stores the block in its
    storage type (perturb +eps, evaluate, to the other side -2 eps, evaluate, restore +eps, update -lr g)."""
    W0 = np.asarray(W, dtype=np.float64)
    L0 = loss_value(forward(X, W0), loss, target) if one_sided else 0.0
    Wp = dense_apply(W0, seed, +eps, storage)
    Lp = loss_value(forward(X, Wp), loss, target)
    if one_sided:
        Lm, Wr = 0.0, dense_apply(Wp, seed, -eps, storage)
        g = (Lp - L0) / eps
    else:
        Wm = dense_apply(Wp, seed, -2.0 * eps, storage)
        Lm = loss_value(forward(X, Wm), loss, target)
        Wr = dense_apply(Wm, seed, +eps, storage)
        g = (Lp - Lm) / (2.0 * eps)
    W_new = dense_apply(Wr, seed, -lr * g, storage)
    return {"L0": L0, "Lp": Lp, "Lm": Lm, "g": g, "W_restored": Wr, "W_new": W_new}

