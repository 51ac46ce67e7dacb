"""Oracle: one AGZO iteration over a small decoder-style MLP stack, in fp64 (test infrastructure only).

Alg. 2 for a model with several linear layers: one unperturbed pass gives f0 and,
at every linear layer, the activation basis of that layer's own input (Alg. 1);
then every linear layer is perturbed at once by +eps Z_l, Z_l = G_l B_l^T (Eq. 7),
for f+, and by -eps Z_l for f-; one global scalar g (Eq. 10, central form by
default) scales every layer's update W_l <- W_l - lr g Z_l.  In the perturbed
passes a layer's input differs from the unperturbed one, which is why the three
passes cannot share their matrix products.

Model (a synthetic stand-in with the structure of a gated-MLP language model):
  h = E[ids]                                   embedding rows, frozen
  per block:  n = rmsnorm(h);  h = h + W_down (silu(W_gate n) * (W_up n))
  logits = W_head rmsnorm(h);  loss = token cross-entropy (oracle.agzo.ce_loss)
rmsnorm(x) = gain * x / sqrt(mean(x^2) + 1e-6).  The gains (one vector per block and
one before the head; fp32 values, all ones if params holds none) are the parameters
that are not linear-layer weights: they take Alg. 2's other branch, a dense Gaussian
perturbation R of their own shape (Eq. 7), with the same eps, the same global g and
the update gain <- gain - lr g R.  The embedding is frozen.

Activation storage: `act` names the type every stored tensor is rounded to
("bf16", "f32", or None for no rounding).  The rounding points are the stored
tensors: n, the three linear outputs, the gated product, the residual sum.
The logits are consumed from the accumulators and never stored.

Nothing here is blocked, fused or reordered.  Pins live in tests/test_oracle_stack.py.
"""
import numpy as np

from . import agzo


def _store(a, act):
    return np.asarray(a, dtype=np.float64) if act is None else agzo.round_storage(a, act)


def rmsnorm(x, gain=None):
    x = np.asarray(x, dtype=np.float64)
    y = x / np.sqrt(np.mean(x * x, axis=1, keepdims=True) + 1e-6)
    return y if gain is None else y * np.asarray(gain, dtype=np.float64)[None, :]


def silu(a):
    a = np.asarray(a, dtype=np.float64)
    return a / (1.0 + np.exp(-a))


def layer_names(n_blocks):
    """Order in which the linear layers are met (and seeds are assigned)."""
    names = []
    for b in range(n_blocks):
        names += [("gate", b), ("up", b), ("down", b)]
    return names + [("head", 0)]


def gain_names(params):
    """The gain vectors present in params, in the order they are met."""
    names = [("norm", b) for b in range(params["n_blocks"])] + [("norm_f", 0)]
    return [nm for nm in names if nm in params]


def shifted_targets(ids):
    """Next-token targets within each sequence; the last position of a sequence has none (-1)."""
    ids = np.asarray(ids)
    t = np.full(ids.shape, -1, dtype=np.int64)
    t[:, :-1] = ids[:, 1:]
    return t.reshape(-1)


def forward(params, ids, act="bf16", delta=None, record=None):
    """Loss of the stack with weights W_l + delta[l] (delta: dict name -> matrix, or None).

    record, if a dict, receives the input activations of every linear layer."""
    def lin(name, x):
        W = np.asarray(params[name], dtype=np.float64)
        if delta is not None:
            W = W + delta[name]
        if record is not None:
            record[name] = x
        return x @ W.T

    def gain(name):
        if name not in params:
            return None
        gv = np.asarray(params[name], dtype=np.float64)
        return gv + delta[name] if delta is not None and name in delta else gv

    ids = np.asarray(ids)
    h = np.asarray(params["E"], dtype=np.float64)[ids.reshape(-1)]
    for b in range(params["n_blocks"]):
        n = _store(rmsnorm(h, gain(("norm", b))), act)
        a = _store(lin(("gate", b), n), act)
        u = _store(lin(("up", b), n), act)
        m = _store(silu(a) * u, act)
        d = _store(lin(("down", b), m), act)
        h = _store(h + d, act)
    n = _store(rmsnorm(h, gain(("norm_f", 0))), act)
    logits = lin(("head", 0), n)
    return agzo.ce_loss(logits, shifted_targets(ids))


def agzo_stack_step(params, ids, r, K, eps, lr, seeds, act="bf16", storage="bf16", one_sided=False):
    """One AGZO iteration (Alg. 2).  seeds: dict layer name -> 64-bit seed of that layer for this step.

    Returns the three losses, g, per layer the basis B and factor G, and the updated weights."""
    names = layer_names(params["n_blocks"])
    inputs = {}
    L0 = forward(params, ids, act, None, inputs)
    B, G, Z = {}, {}, {}
    for nm in names:
        B[nm] = agzo.subspace_extract(inputs[nm], r, K, seeds[nm])["B"]
        Z[nm], G[nm] = agzo.perturbation(B[nm], seeds[nm], np.asarray(params[nm]).shape[0])
    # parameters that are not linear-layer weights: dense Gaussian of their own shape, kept in fp32
    gains = gain_names(params)
    for nm in gains:
        Z[nm] = agzo.dense_perturbation(seeds[nm], 1, np.asarray(params[nm]).shape[0])[0]
    every = names + gains
    Lp = forward(params, ids, act, {nm: eps * Z[nm] for nm in every})
    Lm = 0.0 if one_sided else forward(params, ids, act, {nm: -eps * Z[nm] for nm in every})
    g = (Lp - L0) / eps if one_sided else (Lp - Lm) / (2.0 * eps)
    W_new = {nm: agzo.round_storage(np.asarray(params[nm], dtype=np.float64) - lr * g * Z[nm], storage) for nm in names}
    for nm in gains:
        W_new[nm] = agzo.round_storage(np.asarray(params[nm], dtype=np.float64) - lr * g * Z[nm], "f32")
    return {"L0": L0, "Lp": Lp, "Lm": Lm, "g": g, "B": B, "G": G, "Z": Z, "W_new": W_new, "inputs": inputs}
