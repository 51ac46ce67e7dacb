"""GPU parity: every entry point of the C ABI against the fp64 CPU oracle, element by element,
on identical seeded inputs.  Sizes span several tiles plus ragged tails.

Bars (the benchmark spec): Philox words bit-exact; fp32-storage path <= 1e-4 relative (Frobenius);
bf16-storage path <= 2e-2 relative on outputs and updated W.  The kernels are in fact far
tighter than that, so each test also asserts a bound derived from the arithmetic:
  * fp32 path: products accumulate in fp64, results rounded once to fp32 -> ~1e-6;
  * bf16 path: bf16 x bf16 products are exact in fp32, fp32 accumulation over d_in terms
    -> ~sqrt(d_in) * 2^-24 ~ 1e-5 on Y; small fp32 factors enter as three bf16 planes (24 bits).
"""
import numpy as np
import pytest
import torch

from oracle import agzo as oagzo
from oracle import philox as ophilox
from paper_2601_17261_amd import binding, synth

pytestmark = pytest.mark.gpu

EPS = float(np.float32(1e-3))
LR = float(np.float32(1e-2))


@pytest.fixture(scope="module")
def ctx():
    c = binding.Context()
    yield c
    c.close()


def rel(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def dev(a, storage="f32"):
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16) if storage == "bf16" else t


def host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def assert_increment(W_gpu, W, W_oracle, storage, g_tol=2e-2):
    """The update itself, not the weights it rides on (a no-op update must fail): fp32 storage compares the increments;
    in bf16 storage most increments round away, so the entries the oracle moved must exist and move identically on the
    GPU (up to the few whose rounding boundary lies inside g's own tolerance), and the others must stay."""
    d_gpu, d_or = W_gpu - W, W_oracle - W
    assert np.count_nonzero(d_or) > 0, "the case has no power: the oracle's update rounds away everywhere"
    if storage == "f32":
        assert rel(d_gpu, d_or) < g_tol
        return
    moved = d_or != 0
    assert np.mean(W_gpu[moved] == W_oracle[moved]) > 0.9, np.mean(W_gpu[moved] == W_oracle[moved])
    assert np.mean(W_gpu[~moved] != W[~moved]) < 0.02


def problem(seed, n, d_in, d_out, kind, storage):
    W, X, T = synth.single_layer_problem(seed, n, d_in, d_out, kind=kind, storage=storage)
    return W, X, T, dev(W, storage), dev(X, storage), dev(T)


# ---------------------------------------------------------------------------------------------
# generator
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("rows,cols", [(1, 1), (7, 3), (300, 16), (1025, 5), (4096, 64)])
def test_philox_words_bit_exact(ctx, rows, cols):
    for seed, tag in ((0, 0), (0x0123456789ABCDEF, 1), (2 ** 64 - 1, 3)):
        dst = torch.empty(rows, cols, dtype=torch.int32, device="cuda")
        ctx.philox_words(dst, seed, tag)
        got = dst.cpu().numpy().view(np.uint32)
        np.testing.assert_array_equal(got, ophilox.philox_words(seed, tag, rows, cols))


@pytest.mark.parametrize("rows,cols", [(5, 1), (333, 7), (2048, 16), (12288, 64)])
def test_fill_normal_matches_oracle(ctx, rows, cols):
    dst = torch.empty(rows, cols, dtype=torch.float32, device="cuda")
    ctx.fill_normal(dst, 1234567, binding.TAG_G)
    got = host(dst)
    want = ophilox.normal(1234567, ophilox.TAG_G, rows, cols).astype(np.float64)
    assert np.abs(got - want).max() < 2e-6           # fp32 log / sincos vs fp64, |z| < 5.8
    assert rel(got, want) < 1e-6


def test_generator_empty_is_ok(ctx):
    dst = torch.empty(0, 4, dtype=torch.float32, device="cuda")
    ctx.fill_normal(dst, 1, 0)
    ctx.check()


# ---------------------------------------------------------------------------------------------
# QR
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("d,r,cond", [(64, 1, 1.0), (300, 4, 1e2), (1000, 16, 1e4), (4100, 33, 1e3), (777, 64, 1e2)])
def test_qr_matches_oracle(ctx, d, r, cond):
    rng = np.random.default_rng(d + r)
    Y = rng.standard_normal((d, r)) @ np.diag(np.logspace(0, -np.log10(cond), r)) @ rng.standard_normal((r, r))
    Y = Y.astype(np.float32)
    Q = torch.empty(d, r, dtype=torch.float32, device="cuda")
    ctx.qr(dev(Y), Q)
    ctx.check()
    want, _ = oagzo.qr_pos(Y.astype(np.float64))
    got = host(Q)
    assert np.linalg.norm(got.T @ got - np.eye(r)) < 1e-5
    assert rel(got, want) < 1e-5


def test_qr_rank_deficient_reports_numeric_error(ctx):
    Y = np.ones((128, 3), dtype=np.float32)
    Y[:, 1] = 0.0                      # an exactly zero column: pivot 0
    Q = torch.empty(128, 3, dtype=torch.float32, device="cuda")
    ctx.qr(dev(Y), Q)
    with pytest.raises(binding.AgzoError) as e:
        ctx.check()
    assert e.value.code == binding.ENUMERIC
    ctx.check()                        # flag is cleared by the failed check


# ---------------------------------------------------------------------------------------------
# per-entry-point parity, both storage types
# ---------------------------------------------------------------------------------------------
CASES = [
    # storage, n, d_in, d_out, r, kind, tolerance on Y / S / B
    ("f32", 300, 100, 70, 4, "lowrank", 2e-6),
    ("f32", 512, 256, 256, 4, "lowrank", 2e-6),
    ("f32", 130, 65, 33, 1, "lowrank", 2e-6),
    ("bf16", 300, 200, 264, 8, "lowrank", 2e-5),
    ("bf16", 600, 1024, 520, 16, "rmsnorm", 2e-5),
    ("bf16", 257, 72, 40, 1, "lowrank", 2e-5),
    ("bf16", 300, 1096, 1000, 1, "lowrank", 2e-5),      # r = 1 paths: normalisation, rank-1 sweep over three column blocks
    ("bf16", 515, 136, 300, 24, "powerlaw", 2e-5),
    ("bf16", 700, 320, 264, 40, "powerlaw", 2e-5),      # three 16-column blocks in every rank-r kernel
    ("bf16", 450, 192, 520, 64, "rmsnorm", 2e-5),       # the largest rank
    ("bf16", 200, 4136, 72, 16, "rmsnorm", 2e-5),       # few tokens, deep d_in with a ragged end: X Q splits d_in 8 ways
    ("bf16", 1100, 2048, 136, 40, "powerlaw", 2e-5),    # 18 token blocks x 4 splits, three 16-column blocks
]


# the bf16 forward GEMM has two tilings; these shapes would all take the small one, so each also runs with the large
TILINGS = [binding.TILING_AUTO, binding.TILING_LARGE]


@pytest.mark.parametrize("tiling", TILINGS)
@pytest.mark.parametrize("storage,n,d_in,d_out,r,kind,tol", CASES)
def test_forward_sketch_basis_perturbed_update(ctx, storage, n, d_in, d_out, r, kind, tol, tiling):
    if storage == "f32" and tiling != binding.TILING_AUTO:
        pytest.skip("the fp32-storage path has one tiling")
    seed = 4242 + n
    W, X, T, Wd, Xd, Td = problem(n + d_in, n, d_in, d_out, kind, storage)
    W64, X64 = W.astype(np.float64), X.astype(np.float64)
    L = binding.make_layer(Wd, Xd, r)
    L.tiling = tiling
    loss = binding.make_loss(Td)
    scal = torch.zeros(4, dtype=torch.float64, device="cuda")

    # base forward + range sketch
    Y = torch.empty(n, d_out, dtype=torch.float32, device="cuda")
    S = torch.empty(d_in, r, dtype=torch.float32, device="cuda")
    Ly = binding.make_layer(Wd, Xd, r, Y=Y)
    ctx.layer_forward_sketch(Ly, Wd, Xd, Y, binding.SKETCH_RANGE, None, seed, S, loss, scal[0:1])
    Y0 = oagzo.forward(X64, W64)
    S0 = oagzo.range_sketch(X64, r, seed)
    assert rel(host(Y), Y0) < tol
    assert rel(host(S), S0) < tol
    assert abs(scal[0].item() - oagzo.mse_loss(Y0, T)) < 1e-5 * oagzo.mse_loss(Y0, T)

    # power sketch from a given Q
    ext = oagzo.subspace_extract(X64, r, 3, seed)
    Q1 = ext["Q"][0].astype(np.float32)
    ctx.layer_forward_sketch(L, None, Xd, None, binding.SKETCH_POWER, dev(Q1), seed, S, None, None)
    assert rel(host(S), oagzo.power_sketch(X64, Q1.astype(np.float64))) < tol

    # power sketch without a Q: the Gaussian start matrix of the feature-space variant, from the seed
    ctx.layer_forward_sketch(L, None, Xd, None, binding.SKETCH_POWER, None, seed, S, None, None)
    Q0 = ophilox.normal(seed, ophilox.TAG_Q0, d_in, r).astype(np.float64)
    assert rel(host(S), oagzo.power_sketch(X64, Q0)) < tol

    # basis, with and without a precomputed first sketch
    B = torch.empty(d_in, r, dtype=torch.float32, device="cuda")
    ctx.basis(L, Xd, 3, seed, None, 0, B)
    ctx.check()
    Bg = host(B)
    Bo = ext["B"]
    assert np.linalg.norm(Bg.T @ Bg - np.eye(r)) < 1e-5
    gap = np.linalg.norm(Bg @ Bg.T - Bo @ Bo.T) / np.sqrt(r)
    assert gap < 2e-3, gap
    B2 = torch.empty_like(B)
    ctx.basis(L, Xd, 3, seed, dev(S0.astype(np.float32)), 0, B2)
    assert rel(host(B2), Bg) < 1e-4

    # perturbed forward with the oracle's basis (isolates this entry point)
    Bo32 = Bo.astype(np.float32)
    Z, G = oagzo.perturbation(Bo32.astype(np.float64), seed, d_out)
    for sign in (+1.0, -1.0):
        ctx.perturbed_forward(Ly, Wd, Xd, dev(Bo32), seed, sign * EPS, Y, loss, scal[1:2])
        Yp = oagzo.forward(X64, W64 + sign * EPS * Z)
        assert rel(host(Y), Yp) < tol
        # the perturbation itself, not just the output it rides on
        assert rel(host(Y) - Y0, Yp - Y0) < 5e-3
        Lp = oagzo.mse_loss(Yp, T)
        assert abs(scal[1].item() - Lp) < 1e-5 * Lp

    # update (g given on the device)
    g = -0.731
    gd = torch.tensor([g], dtype=torch.float64, device="cuda")
    Wu = Wd.clone()
    ctx.update(L, Wu, dev(Bo32), seed, LR, gd)
    want = oagzo.round_storage(W64 - LR * g * Z, storage)
    assert rel(host(Wu), want) < (1e-6 if storage == "f32" else 2e-3)
    assert rel(host(Wu) - W64, want - W64) < (1e-4 if storage == "f32" else 0.2)
    if storage == "bf16":
        # rounding decisions taken in fp32 instead of fp64: at most isolated one-ulp flips, plus the
        # increment's own error (bf16 hi/lo operands on the matrix cores: 2^-16 relative per product),
        # which shows where the increment nearly cancels the weight
        ulp = np.abs(want) * 2.0 ** -7
        inc_err = 2.0 ** -15 * LR * abs(g) * (np.abs(G) @ np.abs(Bo32.astype(np.float64)).T)
        assert (np.abs(host(Wu) - want) <= ulp + inc_err + 1e-30).all()
        assert np.mean(host(Wu) != want) < 2e-3
    ctx.check()


@pytest.mark.parametrize("tiling", TILINGS)
@pytest.mark.parametrize("n,d_in,d_out,r", [(515, 136, 300, 8), (512, 320, 768, 16)])
def test_outputs_stored_as_bf16(ctx, n, d_in, d_out, r, tiling):
    """Y kept in bf16 (the storage type of the bf16 configurations): the fp32 accumulators rounded once to nearest even,
    ragged and tile-aligned shapes, both tilings, base and perturbed forward."""
    seed = 77
    W, X, T, Wd, Xd, Td = problem(n + d_out, n, d_in, d_out, "powerlaw", "bf16")
    W64, X64 = W.astype(np.float64), X.astype(np.float64)
    Y = torch.empty(n, d_out, dtype=torch.bfloat16, device="cuda")
    L = binding.make_layer(Wd, Xd, r, Y=Y)
    L.tiling = tiling
    ctx.layer_forward_sketch(L, Wd, Xd, Y, binding.SKETCH_NONE, None, seed, None, None, None)
    B = oagzo.subspace_extract(X64, r, 2, seed)["B"].astype(np.float32)
    Z, _ = oagzo.perturbation(B.astype(np.float64), seed, d_out)
    for eps_signed, Wp in ((0.0, W64), (+EPS, W64 + EPS * Z)):
        if eps_signed != 0.0:
            ctx.perturbed_forward(L, Wd, Xd, dev(B), seed, eps_signed, Y, None, None)
        want = oagzo.round_bf16(oagzo.forward(X64, Wp))
        got = host(Y)
        assert rel(got, want) < 1e-3
        assert (got != want).mean() < 5e-3                    # accumulators a rounding boundary apart in fp32 and fp64
        # one rounding step apart at most; for outputs near zero the step is smaller than the fp32 accumulation error
        assert (np.abs(got - want) <= np.abs(want) * 2.0 ** -7 + 2e-5 * np.abs(want).max()).all()
    ctx.check()


@pytest.mark.parametrize("tiling", TILINGS)
@pytest.mark.parametrize("n,d_in,d_out,r,tdt", [(515, 136, 300, 8, "f32"), (512, 320, 768, 16, "f32"), (512, 320, 768, 16, "bf16")])
def test_operands_inside_wider_allocations(ctx, n, d_in, d_out, r, tdt, tiling):
    """W, X, Y and the target as column ranges of wider buffers (leading dimensions larger than the widths): a whole
    step, the stored outputs, and nothing written outside the ranges."""
    seed = 19
    W, X, T, _, _, _ = problem(n + 1, n, d_in, d_out, "powerlaw", "bf16")
    if tdt == "bf16":
        T = synth.to_bf16_values(T)

    def inside(a, storage, pad):
        big = torch.full((a.shape[0], a.shape[1] + pad), 7.0, dtype=torch.bfloat16 if storage == "bf16" else torch.float32,
                         device="cuda")
        big[:, :a.shape[1]] = dev(a, storage)
        return big, big[:, :a.shape[1]]

    Wb, Wd = inside(W, "bf16", 8)
    Xb, Xd = inside(X, "bf16", 16)
    Tb, Td = inside(T, tdt, 8)
    Yb, Y = inside(np.zeros((n, d_out), dtype=np.float32), "f32", 4)
    L = binding.make_layer(Wd, Xd, r, Y=Y)
    L.tiling = tiling
    assert L.ldw == d_in + 8 and L.ldx == d_in + 16 and L.ldy == d_out + 4
    sc = torch.zeros(1, dtype=torch.float64, device="cuda")
    ctx.layer_forward_sketch(L, Wd, Xd, Y, binding.SKETCH_NONE, None, seed, None, binding.make_loss(Td), sc)
    Y0 = oagzo.forward(X.astype(np.float64), W.astype(np.float64))
    assert rel(host(Y), Y0) < 2e-5
    assert abs(sc.item() - oagzo.mse_loss(Y0, T)) < 1e-5 * oagzo.mse_loss(Y0, T)
    assert (Yb[:, d_out:] == 7.0).all()
    out = torch.zeros(4, dtype=torch.float64, device="cuda")
    Ls = binding.make_layer(Wd, Xd, r)
    Ls.tiling = tiling
    ctx.step(Ls, Wd, Xd, binding.make_loss(Td), 2, EPS, LR, seed, 0, out)
    ctx.check()
    o = oagzo.agzo_step(W, X, T, r, 2, EPS, LR, seed, storage="bf16")
    got = out.cpu().numpy()
    for k, key in enumerate(("L0", "Lp", "Lm")):
        assert abs(got[k] - o[key]) < 1e-5 * o[key]
    assert abs(got[3] - o["g"]) < 2e-2 * abs(o["g"])
    assert rel(host(Wd), o["W_new"]) < 3e-3
    assert (Wb[:, d_in:] == 7.0).all() and (Xb[:, d_in:] == 7.0).all() and (Tb[:, d_out:] == 7.0).all()


# ---------------------------------------------------------------------------------------------
# several matrices updated in one call
# ---------------------------------------------------------------------------------------------
def _update_set(n_small):
    """(storage, d_out, d_in, r, row stride or None, g or None): mixed ranks (four padded widths), an fp32 matrix,
    a matrix inside a wider allocation, ragged row and column tails, and n_small equal small ones to overflow a batch."""
    base = [("bf16", 264, 200, 8, None, -0.731), ("bf16", 40, 72, 1, None, None), ("bf16", 520, 1024, 16, None, 0.4),
            ("bf16", 300, 136, 24, None, 1.7), ("bf16", 520, 192, 64, None, -0.2), ("f32", 70, 100, 4, None, 0.9),
            ("bf16", 130, 264, 40, 272, 0.55), ("bf16", 1, 8, 3, None, -1.0),
            ("bf16", 1000, 1096, 1, 1104, 0.3)]        # rank-1 sweeps share a launch of their own
    return base + [("bf16", 96 + 8 * i, 256 + 8 * i, 16, None, 0.1 * (i + 1)) for i in range(n_small)]


def test_update_many_matches_oracle_and_single_updates(ctx):
    rng = np.random.default_rng(77)
    items, singles, wants = [], [], []
    for idx, (storage, d_out, d_in, r, ld, g) in enumerate(_update_set(19)):
        W = (0.02 * rng.standard_normal((d_out, d_in))).astype(np.float32)
        if storage == "bf16":
            W = synth.to_bf16_values(W)
        B, _ = np.linalg.qr(rng.standard_normal((d_in, r)))
        B32 = B.astype(np.float32)
        seed = 1000 + idx
        if ld is None:
            Wa, Wb = dev(W, storage), dev(W, storage)
        else:       # a view with a row stride larger than d_in; the columns beyond d_in must stay as they are
            Wa = torch.full((d_out, ld), 3.0, dtype=torch.bfloat16, device="cuda")
            Wa[:, :d_in] = dev(W, storage)
            Wb = Wa.clone()
            Wa, Wb = Wa[:, :d_in], Wb[:, :d_in]
        gd = None if g is None else torch.tensor([g], dtype=torch.float64, device="cuda")
        Bd = dev(B32)
        items.append((Wa, Bd, seed, LR, gd))
        singles.append((Wb, Bd, seed, gd, r))
        Z, G = oagzo.perturbation(B32.astype(np.float64), seed, d_out)
        wants.append((storage, oagzo.round_storage(W.astype(np.float64) - LR * (1.0 if g is None else g) * Z, storage), W))
    ctx.update_many(items)
    ctx.check()
    for (Wa, _, _, _, _), (Wb, Bd, seed, gd, r), (storage, want, W) in zip(items, singles, wants):
        ctx.update(_layer_for(Wb, r), Wb, Bd, seed, LR, gd)
        assert torch.equal(Wa, Wb), (tuple(Wa.shape), r)                 # same arithmetic: the same bits
        assert rel(host(Wa), want) < (1e-6 if storage == "f32" else 2e-3)
        assert rel(host(Wa) - W, want - W) < (1e-4 if storage == "f32" else 0.2)
        if Wa.stride(0) != Wa.shape[1]:
            assert (Wa._base[:, Wa.shape[1]:] == 3.0).all()
    ctx.check()


def _layer_for(W, r):
    L = binding.AgzoLayer()
    L.n_tokens, L.d_in, L.d_out, L.r = 0, W.shape[1], W.shape[0], r
    L.dtype = L.y_dtype = binding.F32 if W.dtype == torch.float32 else binding.BF16
    L.tiling, L.ldw, L.ldx, L.ldy = 0, W.stride(0), W.shape[1], W.shape[0]
    return L


@pytest.mark.parametrize("r", [2, 3, 6, 8, 12, 16, 24, 33, 64])
def test_f32_update_at_every_rank_chunking(ctx, r):
    """fp32 storage keeps the vector-ALU sweep, compiled per chunk of the rank (1, 2, 4, 8, 16 and multiples of 16)."""
    rng = np.random.default_rng(r)
    d_out, d_in = 70 + r, 131
    W = (0.02 * rng.standard_normal((d_out, d_in))).astype(np.float32)
    B, _ = np.linalg.qr(rng.standard_normal((d_in, r)))
    B32 = B.astype(np.float32)
    Wd = dev(W)
    g = torch.tensor([0.77], dtype=torch.float64, device="cuda")
    ctx.update(_layer_for(Wd, r), Wd, dev(B32), 900 + r, LR, g)
    ctx.check()
    Z, _ = oagzo.perturbation(B32.astype(np.float64), 900 + r, d_out)
    want = oagzo.round_storage(W.astype(np.float64) - LR * 0.77 * Z, "f32")
    assert rel(host(Wd), want) < 1e-6
    assert rel(host(Wd) - W, want - W) < 1e-4


def test_update_many_rejects_bad_lists_and_accepts_an_empty_one(ctx):
    W = torch.zeros(16, 32, dtype=torch.bfloat16, device="cuda")
    B = torch.ones(32, 4, dtype=torch.float32, device="cuda")
    ctx.update_many([])
    arr = (binding.AgzoUpdateItem * 2)()
    for it in arr:
        it.W, it.B, it.g_dev, it.d_out, it.d_in, it.ldw = W.data_ptr(), B.data_ptr(), 0, 16, 32, 32
        it.r, it.dtype, it.seed, it.lr, it.reserved = 4, binding.BF16, 5, 1.0, 0
    for n, poke in ((-1, None), (2, ("reserved", 1)), (2, ("r", 65)), (2, ("ldw", 24)), (2, ("dtype", 7)), (2, ("W", 0)),
                    (2, ("d_in", 36))):
        saved = None
        if poke:
            saved = getattr(arr[1], poke[0])
            setattr(arr[1], poke[0], poke[1])
        with pytest.raises(binding.AgzoError) as e:
            ctx.update_many_raw(arr, n)
        assert e.value.code == binding.EINVAL
        if poke:
            setattr(arr[1], poke[0], saved)
    with pytest.raises(binding.AgzoError) as e:
        ctx.update_many_raw(None, 1)
    assert e.value.code == binding.EINVAL
    ctx.check()
    assert (W == 0).all()          # the first, valid item of a rejected list was not touched


@pytest.mark.parametrize("storage,n,d_in,d_out,r", [("f32", 512, 256, 256, 4), ("bf16", 600, 1024, 520, 16)])
@pytest.mark.parametrize("flags", [0, binding.ONE_SIDED, binding.SHARED_FORWARD])
def test_step_without_update_then_update_many_equals_step(ctx, storage, n, d_in, d_out, r, flags):
    W, X, T, Wd, Xd, Td = problem(7 + n, n, d_in, d_out, "rmsnorm" if storage == "bf16" else "lowrank", storage)
    L = binding.make_layer(Wd, Xd, r)
    loss = binding.make_loss(Td)
    W1, W2 = Wd.clone(), Wd.clone()
    out1 = torch.zeros(4, dtype=torch.float64, device="cuda")
    out2 = torch.zeros(4, dtype=torch.float64, device="cuda")
    ctx.step(L, W1, Xd, loss, 3, EPS, LR, 99, flags, out1)
    B = torch.empty(d_in, r, dtype=torch.float32, device="cuda")
    ctx.step_no_update(L, W2, Xd, loss, 3, EPS, 99, flags, out2, B)
    ctx.check()
    assert torch.equal(W2, Wd)                       # untouched so far
    assert torch.equal(out1, out2)
    ctx.update_many([(W2, B, 99, LR, out2[3:4])])
    ctx.check()
    assert torch.equal(W1, W2)
    with pytest.raises(binding.AgzoError) as e:
        ctx.step_no_update(L, W2, Xd, loss, 3, EPS, 99, flags, out2, None)
    assert e.value.code == binding.EINVAL


# ---------------------------------------------------------------------------------------------
# range sketch emitted by the forward GEMM itself (Sec. 4.1: the f0 pass also yields the subspace information)
# ---------------------------------------------------------------------------------------------
FUSED_SKETCH = [
    # n, d_in, d_out, r, kind
    (600, 1024, 520, 16, "rmsnorm"),         # 5 token tiles x 5 output tiles, 16 slices: every tile sketches 3-4 of them
    (300, 200, 264, 8, "lowrank"),           # ragged everywhere: last slice 8 wide, last token tile 44 rows
    (2048, 1024, 1024, 16, "rmsnorm"),       # a Qwen3-0.6B projection at that workload's token count
    (130, 72, 1100, 1, "lowrank"),           # more output tiles (9) than slices (2): most tiles sketch nothing
    (128, 64, 128, 3, "powerlaw"),           # a single tile, a single slice
    (1000, 3080, 136, 13, "powerlaw"),       # deep d_in against two output tiles: every tile sketches half the slices
]


@pytest.mark.parametrize("n,d_in,d_out,r,kind", FUSED_SKETCH)
@pytest.mark.parametrize("with_y,with_loss", [(True, True), (False, True), (True, False)])
def test_range_sketch_fused_into_the_forward(ctx, n, d_in, d_out, r, kind, with_y, with_loss):
    seed = 77 + n
    W, X, T, Wd, Xd, Td = problem(n + d_out, n, d_in, d_out, kind, "bf16")
    X64 = X.astype(np.float64)
    loss = binding.make_loss(Td) if with_loss else None
    scal = torch.zeros(2, dtype=torch.float64, device="cuda")
    Y1 = torch.full((n, d_out), 3.0, dtype=torch.bfloat16, device="cuda") if with_y else None
    Y2 = torch.full((n, d_out), 5.0, dtype=torch.bfloat16, device="cuda") if with_y else None
    S1 = torch.full((d_in, r), 9.0, dtype=torch.float32, device="cuda")
    S2 = torch.full((d_in, r), 8.0, dtype=torch.float32, device="cuda")
    L1 = binding.make_layer(Wd, Xd, r, Y=Y1)
    ctx.layer_forward_sketch(L1, Wd, Xd, Y1, binding.SKETCH_RANGE, None, seed, S1, loss, scal[0:1] if with_loss else None)
    L2 = binding.make_layer(Wd, Xd, r, Y=Y2)
    ctx.layer_forward_sketch(L2, Wd, Xd, Y2, binding.SKETCH_RANGE_FUSED, None, seed, S2, loss, scal[1:2] if with_loss else None)
    ctx.check()
    # the forward itself is the same arithmetic in the same order
    if with_y:
        assert torch.equal(Y1, Y2)
    if with_loss:
        assert scal[0].item() == scal[1].item()
    # the sketch against the definition (fp32 Omega is exact as three bf16 planes; fp32 sums)
    S0 = oagzo.range_sketch(X64, r, seed)
    assert rel(host(S2), S0) < 2e-5
    assert rel(host(S2), host(S1)) < 2e-5
    assert np.abs(host(S2) - S0).max() < 2e-5 * np.abs(S0).max() * np.sqrt(n)
    # and it is a sketch the extraction accepts as its first one: same basis as from the separate sweep
    B1 = torch.empty(d_in, r, dtype=torch.float32, device="cuda")
    B2 = torch.empty(d_in, r, dtype=torch.float32, device="cuda")
    ctx.basis(L1, Xd, 2, seed, S1, 0, B1)
    ctx.basis(L2, Xd, 2, seed, S2, 0, B2)
    ctx.check()
    Bg, Bh = host(B1), host(B2)
    assert np.linalg.norm(Bh @ Bh.T - Bg @ Bg.T) / np.sqrt(r) < 2e-3


def test_fused_range_sketch_is_refused_where_the_forward_cannot_emit_it(ctx):
    W, X, T, Wd, Xd, Td = problem(3, 300, 200, 264, "lowrank", "bf16")
    S = torch.zeros(200, 24, dtype=torch.float32, device="cuda")
    def call(L, W_, loss=None, out=None):
        with pytest.raises(binding.AgzoError) as e:
            ctx.layer_forward_sketch(L, W_, Xd, None, binding.SKETCH_RANGE_FUSED, None, 1, S, loss, out)
        assert e.value.code == binding.EINVAL
    call(binding.make_layer(Wd, Xd, 24), Wd)                      # r above 16
    call(binding.make_layer(Wd, Xd, 8), None)                     # no forward to ride on
    Ll = binding.make_layer(Wd, Xd, 8)
    Ll.tiling = binding.TILING_LARGE
    call(Ll, Wd)                                                   # the 256 x 256 tiling does not emit it
    ids = torch.zeros(300, dtype=torch.int32, device="cuda")
    call(binding.make_layer(Wd, Xd, 8), Wd, binding.make_loss(ids, kind=binding.LOSS_CE), torch.zeros(1, dtype=torch.float64, device="cuda"))
    # fp32 storage
    Wf, Xf = Wd.float(), Xd.float()
    with pytest.raises(binding.AgzoError) as e:
        ctx.layer_forward_sketch(binding.make_layer(Wf, Xf, 8), Wf, Xf, None, binding.SKETCH_RANGE_FUSED, None, 1, S, None, None)
    assert e.value.code == binding.EINVAL
    # a shape with many 256 x 256 tiles
    Wb = torch.zeros(4096, 64, dtype=torch.bfloat16, device="cuda")
    Xb = torch.zeros(4096, 64, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(binding.AgzoError) as e:
        ctx.layer_forward_sketch(binding.make_layer(Wb, Xb, 8), Wb, Xb, None, binding.SKETCH_RANGE_FUSED, None, 1, S, None, None)
    assert e.value.code == binding.EINVAL


# ---------------------------------------------------------------------------------------------
# several layers per call: every stage of Alg. 1 (and of the step around it) is one launch for all of them
# ---------------------------------------------------------------------------------------------
MANY_LAYERS = [
    # storage, n, d_in, d_out, r, kind
    ("bf16", 600, 1024, 520, 16, "rmsnorm"),
    ("bf16", 300, 200, 264, 8, "lowrank"),       # same padded rank as the first: shares its launches
    ("bf16", 700, 320, 264, 40, "powerlaw"),     # another padded rank: launches of its own
    ("bf16", 200, 4136, 72, 16, "rmsnorm"),      # X Q splits d_in here
    ("bf16", 512, 320, 768, 16, "powerlaw"),     # tile-aligned
    ("f32", 300, 100, 70, 4, "lowrank"),         # fp32 storage: runs layer by layer inside the call
    ("bf16", 300, 264, 136, 1, "lowrank"),       # a single column: normalised, not factored; rank-1 update sweep
    ("bf16", 400, 520, 264, 1, "rmsnorm"),
]


def test_basis_many_is_bit_identical_to_basis(ctx):
    items, want = [], []
    for li, (storage, n, d_in, d_out, r, kind) in enumerate(MANY_LAYERS):
        W, X, T, Wd, Xd, Td = problem(40 + li, n, d_in, d_out, kind, storage)
        L = binding.make_layer(Wd, Xd, r)
        S0 = None
        if li == 1:                                # one item brings its first sketch along
            S0 = torch.empty(d_in, r, dtype=torch.float32, device="cuda")
            ctx.layer_forward_sketch(L, None, Xd, None, binding.SKETCH_RANGE, None, 900 + li, S0, None, None)
        B1 = torch.empty(d_in, r, dtype=torch.float32, device="cuda")
        ctx.basis(L, Xd, 3, 900 + li, S0, 0, B1)
        want.append(B1)
        items.append((L, Xd, 900 + li, S0, torch.zeros(d_in, r, dtype=torch.float32, device="cuda")))
    ctx.basis_many(items, 3)
    ctx.check()
    for li, (it, B1) in enumerate(zip(items, want)):
        assert torch.equal(it[4], B1), li
    # the feature-space start, and K = 0
    for K, flags in ((2, binding.INIT_FEATURE), (0, 0)):
        for it in items:
            it[4].zero_()
        ctx.basis_many([(L, Xd, seed, None, B) for (L, Xd, seed, _, B) in items], K, flags)
        for li, (L, Xd, seed, _, B) in enumerate(items):
            B1 = torch.empty_like(B)
            ctx.basis(L, Xd, K, seed, None, flags, B1)
            assert torch.equal(B, B1), (K, flags, li)
    ctx.basis_many([], 3)
    ctx.check()


@pytest.mark.parametrize("n,d_in", [(700, 320), (2100, 1096), (64, 4136), (5000, 136)])
def test_basis_many_with_layers_that_read_the_same_activations(ctx, n, d_in):
    """q / k / v (and gate / up) of a layer read one tensor: several layers of a batched call point at the same activations,
    with their own seeds and ranks; bit-identical to the single calls."""
    rng = np.random.default_rng(n)
    Xa = dev(synth.to_bf16_values(rng.standard_normal((n, d_in)) * (1.0 / np.arange(1, d_in + 1)) ** 0.5), "bf16")
    Xb = dev(synth.to_bf16_values(rng.standard_normal((n, d_in))), "bf16")
    items, want = [], []
    for li, (X, r) in enumerate([(Xa, 16), (Xa, 9), (Xa, 16), (Xb, 16), (Xa, 12), (Xa, 16), (Xb, 3), (Xb, 3)]):
        L = binding.make_layer(None, X, r, d_out=8)
        B1 = torch.empty(d_in, r, dtype=torch.float32, device="cuda")
        ctx.basis(L, X, 3, 500 + li, None, 0, B1)
        want.append(B1)
        items.append((L, X, 500 + li, None, torch.zeros(d_in, r, dtype=torch.float32, device="cuda")))
    ctx.basis_many(items, 3)
    ctx.check()
    for li, (it, B1) in enumerate(zip(items, want)):
        assert torch.equal(it[4], B1), li
        Bh = host(B1)
        assert np.linalg.norm(Bh.T @ Bh - np.eye(Bh.shape[1])) < 1e-4


def test_basis_many_more_layers_than_one_launch_holds(ctx):
    rng = np.random.default_rng(5)
    items, want = [], []
    for li in range(19):
        n, d_in, r = int(rng.integers(40, 300)), 8 * int(rng.integers(4, 40)), int(rng.integers(1, 17))
        X = dev(synth.x_rmsnorm_gaussian(rng, n, d_in, storage="bf16"), "bf16")
        L = binding.make_layer(None, X, r, d_out=8)
        B1 = torch.empty(d_in, r, dtype=torch.float32, device="cuda")
        ctx.basis(L, X, 2, 70 + li, None, 0, B1)
        want.append(B1)
        items.append((L, X, 70 + li, None, torch.zeros_like(B1)))
    ctx.basis_many(items, 2)
    ctx.check()
    for li, (it, B1) in enumerate(zip(items, want)):
        assert torch.equal(it[4], B1), li


@pytest.mark.parametrize("r", [8, 24])
def test_basis_many_with_two_workgroups_per_cu(ctx, r):
    """Enough token blocks in one launch (>= 512) for the shallower load ring that lets two workgroups share a CU: the
    same slices in the same order, so still the per-layer call's bits."""
    rng = np.random.default_rng(9)
    X = dev(synth.x_rmsnorm_gaussian(rng, 2048, 264, storage="bf16"), "bf16")
    items, want = [], []
    for li in range(16):
        L = binding.make_layer(None, X, r, d_out=8)
        B1 = torch.empty(264, r, dtype=torch.float32, device="cuda")
        if li < 3:
            ctx.basis(L, X, 2, 500 + li, None, 0, B1)
            want.append(B1)
        items.append((L, X, 500 + li, None, torch.zeros_like(B1)))
    ctx.basis_many(items, 2)
    ctx.check()
    for li, B1 in enumerate(want):
        assert torch.equal(items[li][4], B1), li
    Bo = oagzo.subspace_extract(host(X), r, 2, 515)["B"]
    Bg = host(items[15][4])
    assert np.linalg.norm(Bg @ Bg.T - Bo @ Bo.T) / np.sqrt(r) < 2e-3


@pytest.mark.parametrize("flags", [0, binding.ONE_SIDED, binding.SHARED_FORWARD, binding.INIT_FEATURE])
def test_step_many_is_bit_identical_to_steps(ctx, flags):
    probs = []
    for li, (storage, n, d_in, d_out, r, kind) in enumerate(MANY_LAYERS):
        W, X, T, Wd, Xd, Td = problem(60 + li, n, d_in, d_out, kind, storage)
        if li == 4:
            Td = dev(synth.to_bf16_values(T), "bf16")      # bf16 target on the tile-aligned layer
        probs.append((binding.make_layer(Wd, Xd, r), Wd, Xd, Td))
    outs = torch.zeros(len(probs), 4, dtype=torch.float64, device="cuda")
    Wm = [Wd.clone() for _, Wd, _, _ in probs]
    losses = [binding.make_loss(Td) for _, _, _, Td in probs]
    ctx.step_many([(L, Wm[li], Xd, losses[li], 300 + li, outs[li], None) for li, (L, _, Xd, _) in enumerate(probs)],
                  3, EPS, LR, flags)
    ctx.check()
    for li, (L, Wd, Xd, Td) in enumerate(probs):
        W1 = Wd.clone()
        out1 = torch.zeros(4, dtype=torch.float64, device="cuda")
        ctx.step(L, W1, Xd, losses[li], 3, EPS, LR, 300 + li, flags, out1)
        ctx.check()
        assert torch.equal(out1, outs[li]), (li, out1, outs[li])
        assert torch.equal(W1.view(torch.int16 if W1.dtype == torch.bfloat16 else torch.int32),
                           Wm[li].view(torch.int16 if W1.dtype == torch.bfloat16 else torch.int32)), li
        assert not torch.equal(W1, Wd), li
    # with B_out the item's W stays as it was and its basis is handed out
    Bo = torch.zeros(probs[0][2].shape[1], probs[0][0].r, dtype=torch.float32, device="cuda")
    W0 = probs[0][1].clone()
    ctx.step_many([(probs[0][0], W0, probs[0][2], losses[0], 300, outs[0], Bo)], 3, EPS, LR, flags)
    B1 = torch.empty_like(Bo)
    ctx.basis(probs[0][0], probs[0][2], 3, 300, None, flags & binding.INIT_FEATURE, B1)
    assert torch.equal(W0, probs[0][1]) and torch.equal(Bo, B1)
    with pytest.raises(binding.AgzoError) as e:
        ctx.step_many([(probs[0][0], W0, probs[0][2], losses[0], 300, outs[0], None)], 3, EPS, LR, binding.NAIVE_INPLACE)
    assert e.value.code == binding.EINVAL
    ctx.check()


@pytest.mark.parametrize("storage,n,d_in,d_out,r,kind", [
    ("f32", 512, 256, 256, 4, "lowrank"),
    ("bf16", 515, 136, 300, 8, "lowrank"),
    ("bf16", 600, 1024, 520, 16, "rmsnorm"),
])
@pytest.mark.parametrize("flags", [0, binding.ONE_SIDED, binding.INIT_FEATURE, binding.SHARED_FORWARD,
                                   binding.SHARED_FORWARD | binding.ONE_SIDED])
@pytest.mark.parametrize("tiling", TILINGS)
def test_step_matches_oracle(ctx, storage, n, d_in, d_out, r, kind, flags, tiling):
    if tiling != binding.TILING_AUTO and (storage == "f32" or flags & binding.SHARED_FORWARD):
        pytest.skip("one tiling only")
    seed = 99
    W, X, T, Wd, Xd, Td = problem(7 + n, n, d_in, d_out, kind, storage)
    L = binding.make_layer(Wd, Xd, r)
    L.tiling = tiling
    out = torch.zeros(4, dtype=torch.float64, device="cuda")
    ctx.step(L, Wd, Xd, binding.make_loss(Td), 3, EPS, LR, seed, flags, out)
    ctx.check()
    o = oagzo.agzo_step(W, X, T, r, 3, EPS, LR, seed, storage=storage, one_sided=bool(flags & binding.ONE_SIDED),
                        init="feature" if flags & binding.INIT_FEATURE else "token")
    got = out.cpu().numpy()
    assert abs(got[0] - o["L0"]) < 1e-5 * o["L0"]
    assert abs(got[1] - o["Lp"]) < 1e-5 * o["Lp"]
    if not flags & binding.ONE_SIDED:
        assert abs(got[2] - o["Lm"]) < 1e-5 * o["Lm"]
    gtol = 2e-3 if storage == "f32" else 2e-2
    assert abs(got[3] - o["g"]) < gtol * abs(o["g"]) + 1e-9, (got[3], o["g"])
    assert rel(host(Wd), o["W_new"]) < (1e-4 if storage == "f32" else 2e-2)
    assert rel(host(Wd), o["W_new"]) < (1e-6 if storage == "f32" else 3e-3)
    assert_increment(host(Wd), W.astype(np.float64), o["W_new"], storage)


@pytest.mark.parametrize("storage,n,d_in,d_out,r", [("f32", 200, 96, 130, 4), ("bf16", 515, 136, 300, 8),
                                                      ("bf16", 512, 256, 1000, 16),
                                                      ("bf16", 512, 256, 768, 16),     # tile-aligned: six tiles of the persistent kernel
                                                      ("bf16", 2304, 128, 8192, 8)])   # 288 tiles: tile lists, the shortest pipeline
@pytest.mark.parametrize("flags", [0, binding.SHARED_FORWARD])
def test_cross_entropy_step_matches_oracle(ctx, storage, n, d_in, d_out, r, flags):
    """Token cross-entropy on the layer's outputs as logits (LM-head shape: d_out = vocabulary), with
    ignored rows (target -1)."""
    W, X, _ = synth.single_layer_problem(21 + n, n, d_in, d_out, kind="lowrank", storage=storage)
    W = (W * 5.0).astype(np.float32)                       # logits with some spread
    if storage == "bf16":
        W = synth.to_bf16_values(W)
    rng = np.random.default_rng(n)
    ids = rng.integers(0, d_out, size=n).astype(np.int32)
    ids[rng.choice(n, size=n // 7, replace=False)] = -1
    Wd, Xd, Td = dev(W, storage), dev(X, storage), torch.from_numpy(ids).cuda()
    L = binding.make_layer(Wd, Xd, r)
    loss = binding.make_loss(Td, kind=binding.LOSS_CE)
    # forward entry point on its own
    sc = torch.zeros(1, dtype=torch.float64, device="cuda")
    ctx.layer_forward_sketch(L, Wd, Xd, None, binding.SKETCH_NONE, None, 1, None, loss, sc)
    L0 = oagzo.ce_loss(oagzo.forward(X, W), ids)
    assert abs(sc.item() - L0) < 2e-6 * L0
    out = torch.zeros(4, dtype=torch.float64, device="cuda")
    ctx.step(L, Wd, Xd, loss, 3, EPS, LR, 17, flags, out)
    ctx.check()
    o = oagzo.agzo_step(W, X, ids, r, 3, EPS, LR, 17, loss="ce", storage=storage)
    got = out.cpu().numpy()
    assert abs(got[0] - o["L0"]) < 2e-6 * o["L0"]
    assert abs(got[1] - o["Lp"]) < 2e-6 * o["Lp"]
    assert abs(got[2] - o["Lm"]) < 2e-6 * o["Lm"]
    assert abs(got[3] - o["g"]) < 2e-2 * abs(o["g"]) + 1e-7, (got[3], o["g"])
    assert rel(host(Wd), o["W_new"]) < (1e-6 if storage == "f32" else 3e-3)


def test_config1_trajectory_20_steps(ctx):
    """The small fp32 workload in full: 256x256 layer, 512 tokens, r=4, K=3, 20 steps."""
    W, X, T, Wd, Xd, Td = problem(0, 512, 256, 256, "lowrank", "f32")
    L = binding.make_layer(Wd, Xd, 4)
    loss = binding.make_loss(Td)
    out = torch.zeros(20, 4, dtype=torch.float64, device="cuda")
    Wo = W.astype(np.float64)
    ref = []
    for step in range(20):
        ctx.step(L, Wd, Xd, loss, 3, EPS, LR, 1000 * step, 0, out[step])
        o = oagzo.agzo_step(Wo, X, T, 4, 3, EPS, LR, 1000 * step, storage="f32")
        Wo = o["W_new"]
        ref.append((o["L0"], o["Lp"], o["Lm"], o["g"]))
    ctx.check()
    got = out.cpu().numpy()
    ref = np.array(ref)
    assert np.abs(got[:, :3] / ref[:, :3] - 1).max() < 1e-5
    assert np.abs(got[:, 3] - ref[:, 3]).max() < 2e-3 * np.abs(ref[:, 3]).max()
    assert rel(host(Wd), Wo) < 1e-4
    assert rel(host(Wd) - W, Wo - W) < 1e-2          # the accumulated update itself
    assert ref[-1, 0] < ref[0, 0]                       # and the 20 steps did descend


@pytest.mark.parametrize("one_sided", [False, True])
def test_naive_inplace_comparator_has_its_own_oracle(ctx, one_sided):
    for storage, tolW in (("f32", 1e-6), ("bf16", 3e-3)):
        W, X, T, Wd, Xd, Td = problem(5, 300, 136, 264, "lowrank", storage)
        r, seed = 8, 31
        L = binding.make_layer(Wd, Xd, r)
        B = torch.empty(136, r, dtype=torch.float32, device="cuda")
        ctx.basis(L, Xd, 3, seed, None, 0, B)
        out = torch.zeros(4, dtype=torch.float64, device="cuda")
        flags = binding.NAIVE_INPLACE | (binding.ONE_SIDED if one_sided else 0)
        ctx.step(L, Wd, Xd, binding.make_loss(Td), 3, EPS, LR, seed, flags, out)
        ctx.check()
        o = oagzo.agzo_step_inplace(W, X, T, host(B), EPS, LR, seed, storage=storage, one_sided=one_sided)
        got = out.cpu().numpy()
        assert abs(got[0] - o["L0"]) < 1e-5 * o["L0"]
        assert abs(got[1] - o["Lp"]) < 1e-4 * o["Lp"]
        assert abs(got[2] - o["Lm"]) <= 1e-4 * o["Lm"]
        assert rel(host(Wd), o["W_new"]) < tolW
        assert_increment(host(Wd), W.astype(np.float64), o["W_new"], storage)


@pytest.mark.parametrize("storage,one_sided", [("f32", False), ("bf16", False), ("bf16", True)])
def test_dense_gaussian_step_composed_from_the_calls(ctx, storage, one_sided):
    """Alg. 2 with a linear layer's weight taken through the dense branch of Eq. 7 (the estimator the paper compares
    with), composed from the library's calls: in-place dense sweeps, plain forwards with the fused loss, the scalar,
    the update sweep with g read from the device."""
    W, X, T, Wd, Xd, Td = problem(9, 300, 136, 264, "lowrank", storage)
    eps, lr, seed = float(np.float32(1e-2)), LR, 57
    L = binding.make_layer(Wd, Xd, 1)
    loss = binding.make_loss(Td)
    out = torch.zeros(4, dtype=torch.float64, device="cuda")
    flags = binding.ONE_SIDED if one_sided else 0

    def f(slot):
        ctx.layer_forward_sketch(L, Wd, Xd, None, binding.SKETCH_NONE, None, seed, None, loss, out[slot:slot + 1])

    if one_sided:
        f(0)
    ctx.dense_perturb(Wd, seed, +eps)
    f(1)
    if one_sided:
        ctx.dense_perturb(Wd, seed, -eps)
    else:
        ctx.dense_perturb(Wd, seed, -2.0 * eps)
        f(2)
        ctx.dense_perturb(Wd, seed, +eps)
    restored = host(Wd)
    ctx.two_point(out, eps, flags)
    ctx.dense_perturb(Wd, seed, -lr, out[3:4])
    ctx.check()
    o = oagzo.dense_step(W, X, T, eps, lr, seed, storage=storage, one_sided=one_sided)
    got = out.cpu().numpy()
    for k, key in ((0, "L0"), (1, "Lp"), (2, "Lm")):
        assert abs(got[k] - o[key]) <= 1e-4 * o[key], key
    assert abs(got[3] - o["g"]) < (2e-3 if storage == "f32" else 2e-2) * abs(o["g"]), (got[3], o["g"])
    ulp = 2.0 ** -(23 if storage == "f32" else 7)
    assert np.abs(restored - W).max() <= 4 * ulp * np.abs(W).max()
    assert rel(host(Wd), o["W_new"]) < (1e-5 if storage == "f32" else 3e-3)
    assert rel(host(Wd) - restored, o["W_new"] - o["W_restored"]) < (3e-3 if storage == "f32" else 0.2)


@pytest.mark.parametrize("storage", ["f32", "bf16"])
def test_low_rank_gaussian_step_composed_from_the_calls(ctx, storage):
    """The data-independent low-rank estimator of Sec. 2 (perturbation U V^T with Gaussian factors, estimate scaled by
    1 / r) on the rank-r kernels: V takes the place of the activation basis, U is the seeded Gaussian factor."""
    n, d_in, d_out, r, seed = 300, 136, 264, 8, 23
    W, X, T, Wd, Xd, Td = problem(13, n, d_in, d_out, "lowrank", storage)
    L = binding.make_layer(Wd, Xd, r)
    loss = binding.make_loss(Td)
    out = torch.zeros(4, dtype=torch.float64, device="cuda")
    V = torch.empty(d_in, r, dtype=torch.float32, device="cuda")
    ctx.fill_normal(V, seed, binding.TAG_Q0)
    ctx.perturbed_forward(L, Wd, Xd, V, seed, +EPS, None, loss, out[1:2])
    ctx.perturbed_forward(L, Wd, Xd, V, seed, -EPS, None, loss, out[2:3])
    ctx.two_point(out, EPS)
    ctx.update(L, Wd, V, seed, LR / r, out[3:4])
    ctx.check()
    Vo = ophilox.normal(seed, ophilox.TAG_Q0, d_in, r).astype(np.float64)
    assert np.abs(host(V) - Vo).max() < 2e-6
    o = oagzo.agzo_step(W, X, T, r, 0, EPS, float(np.float32(LR / r)), seed, storage=storage, B=host(V))
    got = out.cpu().numpy()
    assert abs(got[1] - o["Lp"]) < 1e-5 * o["Lp"] and abs(got[2] - o["Lm"]) < 1e-5 * o["Lm"]
    assert abs(got[3] - o["g"]) < (2e-3 if storage == "f32" else 2e-2) * abs(o["g"]), (got[3], o["g"])
    assert rel(host(Wd), o["W_new"]) < (1e-6 if storage == "f32" else 3e-3)
    assert rel(host(Wd) - W, o["W_new"] - W) < (3e-3 if storage == "f32" else 0.2)


@pytest.mark.parametrize("target_dtype", ["f32", "bf16"])
@pytest.mark.parametrize("flags", [0, binding.SHARED_FORWARD, binding.ONE_SIDED, binding.SHARED_FORWARD | binding.ONE_SIDED])
@pytest.mark.parametrize("n,d_in,d_out,r", [(512, 320, 768, 16),     # five d_in slices, one extension slice
                                            (256, 128, 512, 40),     # the shortest pipeline (two slices), two extension slices
                                            (512, 192, 256, 64),     # three extension slices
                                            (768, 1088, 256, 8),     # 17 slices: odd count, tiles_n = 1
                                            (512, 264, 768, 16)])    # d_in not a multiple of 64: the general kernel
def test_tile_aligned_shapes_take_the_specialised_loss_epilogues(ctx, target_dtype, flags, n, d_in, d_out, r):
    """Tokens and outputs multiples of the 256 x 256 tile: the squared-error kernel whose accumulators start at minus
    the target (one evaluation per launch, or f0, f+, f- from one pass in shared-forward mode), against an fp32 and a
    bf16 target."""
    W, X, T, Wd, Xd, Td = problem(61, n, d_in, d_out, "powerlaw", "bf16")
    if target_dtype == "bf16":
        T = synth.to_bf16_values(T)
        Td = dev(T, "bf16")
    L = binding.make_layer(Wd, Xd, r)
    L.tiling = binding.TILING_LARGE                # this shape alone would take the small tiling
    sc = torch.zeros(1, dtype=torch.float64, device="cuda")
    ctx.layer_forward_sketch(L, Wd, Xd, None, binding.SKETCH_NONE, None, 1, None, binding.make_loss(Td), sc)
    L0 = oagzo.mse_loss(oagzo.forward(X.astype(np.float64), W.astype(np.float64)), T)
    assert abs(sc.item() - L0) < 1e-5 * L0
    out = torch.zeros(4, dtype=torch.float64, device="cuda")
    ctx.step(L, Wd, Xd, binding.make_loss(Td), 2, EPS, LR, 17, flags, out)
    ctx.check()
    one_sided = bool(flags & binding.ONE_SIDED)
    o = oagzo.agzo_step(W, X, T, r, 2, EPS, LR, 17, storage="bf16", one_sided=one_sided)
    got = out.cpu().numpy()
    assert abs(got[0] - o["L0"]) < 1e-5 * o["L0"]
    assert abs(got[1] - o["Lp"]) < 1e-5 * o["Lp"]
    if not one_sided:
        assert abs(got[2] - o["Lm"]) < 1e-5 * o["Lm"]
    assert abs(got[3] - o["g"]) < 2e-2 * abs(o["g"]) + 1e-9, (got[3], o["g"])
    assert rel(host(Wd), o["W_new"]) < 3e-3
    assert_increment(host(Wd), W.astype(np.float64), o["W_new"], "bf16")


@pytest.mark.parametrize("n,d_in,d_out", [(4352, 128, 4352),    # 289 tiles: 36 per XCD, one left over; the shortest pipeline
                                          (4096, 192, 4352),    # 272 tiles: 34 per XCD, so two workgroups per XCD take two
                                          (2048, 320, 16640)])  # 520 tiles: every workgroup takes two, eight take three
def test_more_tiles_than_compute_units_walks_tile_lists(ctx, n, d_in, d_out):
    """The tile-aligned kernel runs one workgroup per compute unit, each walking a list of tiles with the next tile's first
    slices fetched under the last slices of the current one: losses (plain and perturbed, bf16 and fp32 targets) and the
    stored bf16 output against the oracle where some workgroups take one tile more than others."""
    r, seed = 16, 91
    W, X, T, Wd, Xd, Td = problem(7, n, d_in, d_out, "powerlaw", "bf16")
    X64, W64 = X.astype(np.float64), W.astype(np.float64)
    Y0 = oagzo.forward(X64, W64)
    L = binding.make_layer(Wd, Xd, r)
    B = torch.empty(d_in, r, dtype=torch.float32, device="cuda")
    ctx.basis(L, Xd, 1, seed, None, 0, B)
    Z, _ = oagzo.perturbation(host(B), seed, d_out)
    Yp = oagzo.forward(X64, W64 + EPS * Z)
    for tdt in ("bf16", "f32"):
        Tt = synth.to_bf16_values(T) if tdt == "bf16" else T
        Ttd = dev(Tt, tdt)
        sc = torch.zeros(2, dtype=torch.float64, device="cuda")
        ctx.layer_forward_sketch(L, Wd, Xd, None, binding.SKETCH_NONE, None, 1, None, binding.make_loss(Ttd), sc[0:1])
        ctx.perturbed_forward(L, Wd, Xd, B, seed, EPS, None, binding.make_loss(Ttd), sc[1:2])
        ctx.check()
        l0, lp = oagzo.mse_loss(Y0, Tt), oagzo.mse_loss(Yp, Tt)
        assert abs(sc[0].item() - l0) < 1e-5 * l0, tdt
        assert abs(sc[1].item() - lp) < 1e-5 * lp, tdt
    # stored output: every tile of every workgroup's list
    Y = torch.full((n, d_out), 7.0, dtype=torch.bfloat16, device="cuda")
    Ly = binding.make_layer(Wd, Xd, r, Y=Y)
    ctx.perturbed_forward(Ly, Wd, Xd, B, seed, EPS, Y, None, None)
    ctx.check()
    got = host(Y)
    assert np.abs(got - Yp).max() <= 2.0 ** -8 * np.abs(Yp).max() + 1e-6
    assert rel(got, Yp) < 3e-3
    tiles = np.abs(got - Yp).reshape(n // 256, 256, d_out // 256, 256).max(axis=(1, 3)) / np.abs(Yp).max()
    assert tiles.max() < 2.0 ** -8, np.unravel_index(tiles.argmax(), tiles.shape)


@pytest.mark.parametrize("storage", ["f32", "bf16"])
def test_all_zero_activations_raise_the_numeric_flag_and_leave_the_context_usable(ctx, storage):
    """X = 0: every sketch is zero, the first Cholesky pivot is 0, no basis exists.  The step reports AGZO_ENUMERIC at
    the next check instead of NaNs passing silently, and the context goes on working."""
    W, X, T, Wd, Xd, Td = problem(3, 300, 136, 264, "lowrank", storage)
    Xz = torch.zeros_like(Xd)
    out = torch.zeros(4, dtype=torch.float64, device="cuda")
    ctx.step(binding.make_layer(Wd, Xz, 4), Wd.clone(), Xz, binding.make_loss(Td), 2, EPS, LR, 5, 0, out)
    with pytest.raises(binding.AgzoError) as e:
        ctx.check()
    assert e.value.code == binding.ENUMERIC
    ctx.check()                                            # cleared
    W2 = Wd.clone()
    ctx.step(binding.make_layer(W2, Xd, 4), W2, Xd, binding.make_loss(Td), 2, EPS, LR, 5, 0, out)
    ctx.check()
    o = oagzo.agzo_step(W, X, T, 4, 2, EPS, LR, 5, storage=storage)
    assert abs(out[3].item() - o["g"]) < 2e-2 * abs(o["g"])
    assert rel(host(W2), o["W_new"]) < (1e-6 if storage == "f32" else 3e-3)


def test_step_is_deterministic(ctx):
    W, X, T, Wd, Xd, Td = problem(3, 600, 1024, 520, "rmsnorm", "bf16")
    L = binding.make_layer(Wd, Xd, 16)
    res = []
    for _ in range(2):
        Wc = Wd.clone()
        out = torch.zeros(4, dtype=torch.float64, device="cuda")
        ctx.step(L, Wc, Xd, binding.make_loss(Td), 3, EPS, LR, 5, 0, out)
        res.append((Wc.cpu(), out.cpu()))
    assert torch.equal(res[0][0], res[1][0]) and torch.equal(res[0][1], res[1][1])


@pytest.mark.parametrize("tiling", TILINGS)
def test_qwen3_0p6b_layer_set_one_step(ctx, tiling):
    """Config 2 at full size: the seven projections of a Qwen3-0.6B layer, N = 8 x 256, r = 8 (every shape here takes
    the small GEMM tiling by itself; the second run forces the large one)."""
    n, r = 2048, 8
    rng = np.random.default_rng(2)
    inputs = {}
    for name, d_in, d_out in synth.QWEN3_0P6B_LAYER:
        key = {"q": "attn", "k": "attn", "v": "attn", "gate": "mlp", "up": "mlp"}.get(name, name)
        if key not in inputs:
            inputs[key] = synth.x_rmsnorm_gaussian(rng, n, d_in, storage="bf16")
        X = inputs[key]
        W = synth.weights(rng, d_out, d_in, storage="bf16")
        T = synth.shifted_target(rng, X, W)
        Wd, Xd, Td = dev(W, "bf16"), dev(X, "bf16"), dev(T)
        L = binding.make_layer(Wd, Xd, r)
        L.tiling = tiling
        out = torch.zeros(4, dtype=torch.float64, device="cuda")
        seed = 1000 + len(name)
        ctx.step(L, Wd, Xd, binding.make_loss(Td), 3, EPS, LR, seed, 0, out)
        ctx.check()
        o = oagzo.agzo_step(W, X, T, r, 3, EPS, LR, seed, storage="bf16")
        got = out.cpu().numpy()
        assert abs(got[0] - o["L0"]) < 1e-5 * o["L0"], name
        assert abs(got[3] - o["g"]) < 2e-2 * abs(o["g"]) + 1e-9, (name, got[3], o["g"])
        assert rel(host(Wd), o["W_new"]) < 3e-3, name
        assert_increment(host(Wd), W.astype(np.float64), o["W_new"], "bf16")


# ---------------------------------------------------------------------------------------------
# argument checking
# ---------------------------------------------------------------------------------------------
def test_invalid_arguments_are_rejected(ctx):
    W, X, T, Wd, Xd, Td = problem(1, 64, 32, 16, "lowrank", "bf16")
    out = torch.zeros(4, dtype=torch.float64, device="cuda")
    loss = binding.make_loss(Td)
    for r in (0, 65, 33):
        with pytest.raises(binding.AgzoError) as e:
            ctx.step(binding.make_layer(Wd, Xd, r), Wd, Xd, loss, 3, EPS, LR, 1, 0, out)
        assert e.value.code == binding.EINVAL
    L = binding.make_layer(Wd, Xd, 4)
    with pytest.raises(binding.AgzoError):
        ctx.step(L, None, Xd, loss, 3, EPS, LR, 1, 0, out)
    with pytest.raises(binding.AgzoError):
        ctx.step(L, Wd, Xd, loss, 3, 0.0, LR, 1, 0, out)
    Lbad = binding.make_layer(Wd, Xd, 4)
    Lbad.ldx = 36                       # not a multiple of 8 for bf16
    with pytest.raises(binding.AgzoError):
        ctx.step(Lbad, Wd, Xd, loss, 3, EPS, LR, 1, 0, out)
    # empty layers and dimensions beyond the documented maximum are refused, not launched
    for field, value in (("n_tokens", 0), ("d_in", 0), ("d_out", 0), ("n_tokens", (1 << 24) + 1), ("d_out", (1 << 24) + 1)):
        Le = binding.make_layer(Wd, Xd, 4)
        setattr(Le, field, value)
        with pytest.raises(binding.AgzoError) as e:
            ctx.step(Le, Wd, Xd, loss, 3, EPS, LR, 1, 0, out)
        assert e.value.code == binding.EINVAL, field
    Lt = binding.make_layer(Wd, Xd, 4)
    Lt.tiling = 7
    with pytest.raises(binding.AgzoError):
        ctx.step(Lt, Wd, Xd, loss, 3, EPS, LR, 1, 0, out)
    # empty blocks are fine where the call has nothing to do
    ctx.dense_perturb(torch.empty(0, 8, dtype=torch.float32, device="cuda"), 1, 1.0)
    ctx.dense_perturb(torch.empty(0, dtype=torch.bfloat16, device="cuda"), 1, 1.0)
    ctx.check()
    np.testing.assert_array_equal(Wd.float().cpu().numpy(), W)     # nothing was touched


def test_misaligned_or_overlong_bf16_operands_are_rejected(ctx):
    """bf16 operands travel as 16-byte vectors: a pointer off by a few elements, or a leading dimension beyond what
    the kernels' 32-bit offsets cover, is refused by every entry point that reads X or W."""
    W, X, T, Wd, Xd, Td = problem(1, 64, 40, 16, "lowrank", "bf16")
    Xw = torch.zeros(64, 48, dtype=torch.bfloat16, device="cuda")
    Xoff = Xw[:, 4:44]                      # 8 bytes off a 16-byte boundary, ld = 48
    Ww = torch.zeros(16, 48, dtype=torch.bfloat16, device="cuda")
    Woff = Ww[:, 4:44]
    out = torch.zeros(4, dtype=torch.float64, device="cuda")
    B = torch.zeros(40, 4, dtype=torch.float32, device="cuda")
    S = torch.zeros(40, 4, dtype=torch.float32, device="cuda")
    loss = binding.make_loss(Td)
    calls = [
        lambda X_, W_: ctx.layer_forward_sketch(binding.make_layer(W_, X_, 4), W_, X_, None, binding.SKETCH_RANGE, None, 1, S, loss, out[0:1]),
        lambda X_, W_: ctx.basis(binding.make_layer(W_, X_, 4), X_, 3, 1, None, 0, B),
        lambda X_, W_: ctx.perturbed_forward(binding.make_layer(W_, X_, 4), W_, X_, B, 1, EPS, None, loss, out[1:2]),
        lambda X_, W_: ctx.step(binding.make_layer(W_, X_, 4), W_, X_, loss, 3, EPS, LR, 1, 0, out),
    ]
    for i, call in enumerate(calls):
        with pytest.raises(binding.AgzoError) as e:
            call(Xoff, Wd)
        assert e.value.code == binding.EINVAL, i
        if i != 1:                          # agzo_basis does not read W
            with pytest.raises(binding.AgzoError) as e:
                call(Xd, Woff)
            assert e.value.code == binding.EINVAL, i
    Lbig = binding.make_layer(Wd, Xd, 4)
    Lbig.ldx = 1 << 22
    with pytest.raises(binding.AgzoError) as e:
        ctx.step(Lbig, Wd, Xd, loss, 3, EPS, LR, 1, 0, out)
    assert e.value.code == binding.EINVAL
    ctx.check()
    assert torch.count_nonzero(Xw).item() == 0 and torch.count_nonzero(Ww).item() == 0


@pytest.mark.parametrize("storage,n,d_in,d_out", [("f32", 200, 96, 130), ("bf16", 515, 136, 300), ("bf16", 512, 128, 512)])
def test_cross_entropy_ids_beyond_the_outputs_are_skipped(ctx, storage, n, d_in, d_out):
    """An id >= d_out is a caller error; the kernels do not read a logit for it: the row counts as ignored."""
    W, X, _ = synth.single_layer_problem(5 + n, n, d_in, d_out, kind="lowrank", storage=storage)
    rng = np.random.default_rng(n)
    ids = rng.integers(0, d_out, size=n).astype(np.int32)
    bad = rng.choice(n, size=n // 9, replace=False)
    ids_bad = ids.copy()
    ids_bad[bad] = d_out + rng.integers(0, 1000, size=bad.size).astype(np.int32)
    ids_ref = ids.copy()
    ids_ref[bad] = -1
    Wd, Xd = dev(W, storage), dev(X, storage)
    L = binding.make_layer(Wd, Xd, 4)
    sc = torch.zeros(1, dtype=torch.float64, device="cuda")
    ids_dev = torch.from_numpy(ids_bad).cuda()
    ctx.layer_forward_sketch(L, Wd, Xd, None, binding.SKETCH_NONE, None, 1, None,
                             binding.make_loss(ids_dev, kind=binding.LOSS_CE), sc)
    ctx.check()
    want = oagzo.ce_loss(oagzo.forward(X, W), ids_ref)
    assert abs(sc.item() - want) < 2e-6 * want


# ---------------------------------------------------------------------------------------------
# measurement hooks: they report through the C ABI and leave the results untouched
# ---------------------------------------------------------------------------------------------
def test_clock_telemetry_and_mfma_probe(ctx):
    W, X, T, Wd, Xd, Td = problem(5, 300, 200, 136, "lowrank", "bf16")
    L = binding.make_layer(Wd, Xd, 4)
    loss = binding.make_loss(Td)
    out = torch.zeros(2, 4, dtype=torch.float64, device="cuda")
    W0, W1 = Wd.clone(), Wd.clone()
    ctx.step(L, W0, Xd, loss, 2, EPS, LR, 9, 0, out[0])
    ctx.profile_enable(1 << binding.PROF_GEMM)
    ctx.step(L, W1, Xd, loss, 2, EPS, LR, 9, 0, out[1])
    n_ev, _ = ctx.profile_read(binding.PROF_GEMM)
    n_clk, ghz = ctx.profile_clock()
    ctx.profile_enable(False)
    ctx.check()
    assert n_ev == 3 and n_clk == 3                  # f0, f+, f-
    assert 0.3 < ghz < 3.0
    assert torch.equal(out[0], out[1]) and torch.equal(W0, W1)      # telemetry changes no result
    assert ctx.profile_clock() == (0, 0.0)
    g = torch.Generator(device="cuda")
    g.manual_seed(3)
    ops = torch.randn(16384, device="cuda", generator=g).to(torch.bfloat16)
    tf, clk = ctx.probe_mfma(ops, 8, 200)
    # rate and clock are tied together: 4 SIMDs per CU, one 32x32x16 MFMA (32768 flop) per 32 cycles each
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    assert 0.3 < clk < 3.0
    assert tf == pytest.approx(cus * 4 * 1024 * clk * 1e-3, rel=0.05)
    tf4, clk4 = ctx.probe_mfma(ops, 4, 200)
    assert tf4 < 0.7 * tf * clk4 / clk
    # the same flop count from 16x16x32 instructions (16384 flop per 16 cycles)
    tf16, clk16 = ctx.probe_mfma(ops, 9, 200)
    assert tf16 == pytest.approx(cus * 4 * 1024 * clk16 * 1e-3, rel=0.05)
    for duty, iters in ((0, 10), (10, 10), (8, 0)):
        with pytest.raises(binding.AgzoError) as e:
            ctx.probe_mfma(ops, duty, iters)
        assert e.value.code == binding.EINVAL


# ---------------------------------------------------------------------------------------------
# dense Gaussian sweep (Eq. 7, parameters that are not linear-layer weights)
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("storage,shape", [("f32", (1, 2048)), ("f32", (33, 130)), ("f32", (5, 7)),
                                           ("bf16", (1, 4096)), ("bf16", (257, 72)), ("bf16", (64, 1023))])
def test_dense_perturb_matches_oracle(ctx, storage, shape):
    rng = np.random.default_rng(shape[1])
    th = synth.weights(rng, shape[0], shape[1], std=1.0, storage=storage)
    seed, eps, lr = 99 + shape[0], float(np.float32(1e-2)), float(np.float32(0.5))
    g = torch.tensor([-0.37], dtype=torch.float64, device="cuda")
    d = dev(th, storage)
    ulp_bits = 7 if storage == "bf16" else 23

    def check(got, want, incr):
        # one rounding to the storage type (fp32 arithmetic here, fp64 in the oracle: a value near a rounding
        # boundary may come out one ulp apart) plus the fp32 generator's own error (2e-6 absolute per normal)
        ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(want), 1e-30))) - ulp_bits)
        assert (np.abs(host(got) - want) <= ulp * 1.0001 + 3e-6 * abs(incr)).all()
        # (in fp32 the generator's own error is a sizeable part of an ulp, so only bf16 results are mostly identical)
        if storage == "bf16":
            assert (host(got) != want).mean() < 0.02

    def sweep(t, scale, g_dev=None, g_val=1.0):
        # compared sweep by sweep from this side's own state, so that a one-ulp difference is not carried along
        before = host(t)
        ctx.dense_perturb(t, seed, scale, g_dev)
        want = oagzo.dense_apply(before, seed, scale * g_val, storage)
        check(t, want, scale * g_val)
        return want

    p1 = sweep(d, eps)                     # perturb (Alg. 2)
    sweep(d, -2 * eps)                     # to the other side
    sweep(d, eps)                          # restore
    back = host(d)
    assert np.abs(back - th).max() <= 4 * 2.0 ** -ulp_bits * np.abs(th).max()
    sweep(d, -lr, g, -0.37)                # update with the device scalar
    assert np.abs(host(d) - back).max() > 0.1
    # a 1-D tensor is one row of the same stream
    if shape[0] == 1:
        d1 = dev(th, storage).reshape(-1)
        ctx.dense_perturb(d1, seed, eps)
        check(d1.reshape(1, -1), p1, eps)
    # strided rows: only the addressed columns change
    big = torch.zeros(shape[0], shape[1] + 5, dtype=d.dtype, device="cuda")
    view = big[:, :shape[1]]
    ctx.dense_perturb(view, seed, 1.0)
    assert (big[:, shape[1]:] == 0).all()
    check(view, oagzo.dense_apply(np.zeros(shape), seed, 1.0, storage), 1.0)
    with pytest.raises(binding.AgzoError) as e:
        ctx._rc(ctx.lib.agzo_dense_perturb(ctx.h, None, 0, 4, 4, 2, 1, 1.0, None))
    assert e.value.code == binding.EINVAL
    ctx.check()


# ---------------------------------------------------------------------------------------------
# degenerate shapes: a single token, rank equal to the token count or to d_in, no power steps
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("storage,n,d_in,d_out,r", [("bf16", 1, 8, 1, 1), ("bf16", 8, 8, 8, 8), ("bf16", 16, 64, 264, 16),
                                                     ("bf16", 40, 16, 3, 16), ("f32", 1, 1, 1, 1), ("f32", 2, 3, 1, 2),
                                                     ("f32", 5, 4, 7, 4)])
@pytest.mark.parametrize("tiling", TILINGS)
@pytest.mark.parametrize("K", [0, 2])
def test_degenerate_shapes_step(ctx, storage, n, d_in, d_out, r, K, tiling):
    if storage == "f32" and tiling != binding.TILING_AUTO:
        pytest.skip("the fp32-storage path has one tiling")
    seed = 17
    rng = np.random.default_rng(100 * n + d_in)
    X = synth.x_rmsnorm_gaussian(rng, n, d_in, storage=storage)
    W = synth.weights(rng, d_out, d_in, std=0.3, storage=storage)
    T = rng.standard_normal((n, d_out)).astype(np.float32)
    Wd, Xd, Td = dev(W, storage), dev(X, storage), dev(T)
    L = binding.make_layer(Wd, Xd, r)
    L.tiling = tiling
    out = torch.zeros(4, dtype=torch.float64, device="cuda")
    lr = float(np.float32(1e-2))
    ctx.step(L, Wd, Xd, binding.make_loss(Td), K, EPS, lr, seed, 0, out)
    ctx.check()
    o = oagzo.agzo_step(W, X, T, r, K, EPS, lr, seed, storage=storage)
    got = out.cpu().numpy()
    for i, k in enumerate(("L0", "Lp", "Lm")):
        assert abs(got[i] - o[k]) < 1e-5 * o[k] + 1e-12, (k, got[i], o[k])
    gtol = 2e-3 if storage == "f32" else 2e-2
    # g is a difference of losses: next to the relative bound stands the losses' own rounding, amplified by 1 / (2 eps)
    assert abs(got[3] - o["g"]) < gtol * abs(o["g"]) + (1e-7 if storage == "f32" else 2e-6) * o["L0"] / EPS, (got[3], o["g"])
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(o["W_new"]), 1e-30))) - (23 if storage == "f32" else 7))
    incr = lr * abs(o["g"]) * np.abs(o["Z"])
    assert (np.abs(host(Wd) - o["W_new"]) <= ulp * 1.0001 + (gtol + 1e-3) * incr + 1e-7).all()
    if r == d_in:
        # the basis spans the whole input space: the perturbation is then a full d_out x d_in Gaussian in disguise
        np.testing.assert_allclose(o["B"] @ o["B"].T, np.eye(d_in), atol=1e-10)
