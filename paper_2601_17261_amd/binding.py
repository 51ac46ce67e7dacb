"""Thin ctypes binding of libagzo.so: argument marshalling only.

Function names and argument order are those of include/agzo.h.  Tensors are
torch tensors on the GPU (torch is used for device memory and streams only);
nothing is computed here, and there is no fallback: if the HIP library is not
built, importing the entry points raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libagzo.so")

F32, BF16 = 0, 1
LOSS_NONE, LOSS_MSE, LOSS_CE = 0, 1, 2
SKETCH_NONE, SKETCH_RANGE, SKETCH_POWER, SKETCH_RANGE_FUSED = 0, 1, 2, 3
TAG_G, TAG_OMEGA, TAG_Q0, TAG_DENSE = 0, 1, 2, 3
ONE_SIDED, NAIVE_INPLACE, INIT_FEATURE, SHARED_FORWARD = 1, 2, 4, 8
OK, EINVAL, ENOMEM, ENUMERIC, EHIP = 0, -1, -2, -3, -4

TILING_AUTO, TILING_LARGE = 0, 1
PROF_GEMM, PROF_UPDATE, PROF_XQ, PROF_XTT, PROF_QR, PROF_FILL = range(6)
PROF_ALL = 63

EXPORTS = ["agzo_create", "agzo_destroy", "agzo_last_error", "agzo_check", "agzo_profile_enable",
           "agzo_profile_read", "agzo_profile_clock", "agzo_probe_mfma", "agzo_philox_words", "agzo_fill_normal",
           "agzo_layer_forward_sketch", "agzo_qr", "agzo_basis", "agzo_perturbed_forward", "agzo_two_point", "agzo_dense_perturb", "agzo_update", "agzo_update_noalloc",
           "agzo_update_many", "agzo_step", "agzo_step_no_update", "agzo_basis_many", "agzo_step_many",
           "agzo_glue_rmsnorm", "agzo_glue_swiglu", "agzo_glue_add", "agzo_glue_attention"]


class AgzoLayer(ctypes.Structure):
    _fields_ = [("n_tokens", ctypes.c_int64), ("d_in", ctypes.c_int64), ("d_out", ctypes.c_int64),
                ("r", ctypes.c_int32), ("dtype", ctypes.c_int32), ("y_dtype", ctypes.c_int32),
                ("tiling", ctypes.c_int32), ("ldw", ctypes.c_int64), ("ldx", ctypes.c_int64),
                ("ldy", ctypes.c_int64)]


class AgzoLossSpec(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("target_dtype", ctypes.c_int32), ("target", ctypes.c_void_p),
                ("ldt", ctypes.c_int64)]


class AgzoUpdateItem(ctypes.Structure):
    _fields_ = [("W", ctypes.c_void_p), ("B", ctypes.c_void_p), ("g_dev", ctypes.c_void_p),
                ("d_out", ctypes.c_int64), ("d_in", ctypes.c_int64), ("ldw", ctypes.c_int64),
                ("r", ctypes.c_int32), ("dtype", ctypes.c_int32), ("seed", ctypes.c_uint64),
                ("lr", ctypes.c_float), ("reserved", ctypes.c_int32)]


class AgzoBasisItem(ctypes.Structure):
    _fields_ = [("layer", AgzoLayer), ("X", ctypes.c_void_p), ("seed", ctypes.c_uint64), ("S0", ctypes.c_void_p),
                ("B", ctypes.c_void_p)]


class AgzoStepItem(ctypes.Structure):
    _fields_ = [("layer", AgzoLayer), ("W", ctypes.c_void_p), ("X", ctypes.c_void_p), ("loss", AgzoLossSpec),
                ("seed", ctypes.c_uint64), ("out_dev", ctypes.c_void_p), ("B_out", ctypes.c_void_p)]


class AgzoError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("agzo error %d: %s" % (code, msg))
        self.code = code


_lib = None


def load():
    """Load the built library (raises if it has not been built)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError("libagzo.so is not built: run `python -m paper_2601_17261_amd.build` "
                          "(there is no CPU fallback for the HIP path)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, u32, u64, f32 = (ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_uint32,
                                   ctypes.c_uint64, ctypes.c_float)
    lp, sp = ctypes.POINTER(AgzoLayer), ctypes.POINTER(AgzoLossSpec)
    lib.agzo_create.argtypes = [ctypes.POINTER(vp), vp]
    lib.agzo_destroy.argtypes = [vp]
    lib.agzo_destroy.restype = None
    lib.agzo_last_error.argtypes = [vp]
    lib.agzo_last_error.restype = ctypes.c_char_p
    lib.agzo_check.argtypes = [vp]
    lib.agzo_profile_enable.argtypes = [vp, i32]
    lib.agzo_profile_read.argtypes = [vp, i32, ctypes.POINTER(i64), ctypes.POINTER(ctypes.c_double)]
    lib.agzo_profile_clock.argtypes = [vp, ctypes.POINTER(i64), ctypes.POINTER(ctypes.c_double)]
    lib.agzo_probe_mfma.argtypes = [vp, vp, i32, i32, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
    lib.agzo_philox_words.argtypes = [vp, vp, i64, i32, u64, u32]
    lib.agzo_fill_normal.argtypes = [vp, vp, i64, i32, u64, u32]
    lib.agzo_layer_forward_sketch.argtypes = [vp, lp, vp, vp, vp, i32, vp, u64, vp, sp, vp]
    lib.agzo_qr.argtypes = [vp, vp, i64, i32, vp]
    lib.agzo_basis.argtypes = [vp, lp, vp, i32, u64, vp, i32, vp]
    lib.agzo_perturbed_forward.argtypes = [vp, lp, vp, vp, vp, u64, f32, vp, sp, vp]
    lib.agzo_two_point.argtypes = [vp, vp, f32, i32]
    lib.agzo_dense_perturb.argtypes = [vp, vp, i32, i64, i64, i64, u64, f32, vp]
    lib.agzo_update.argtypes = [vp, lp, vp, vp, u64, f32, vp]
    lib.agzo_update_noalloc.argtypes = [vp, lp, vp, vp, u64, f32, vp]
    lib.agzo_update_many.argtypes = [vp, ctypes.POINTER(AgzoUpdateItem), i32]
    lib.agzo_basis_many.argtypes = [vp, ctypes.POINTER(AgzoBasisItem), i32, i32, i32]
    lib.agzo_step_many.argtypes = [vp, ctypes.POINTER(AgzoStepItem), i32, i32, f32, f32, i32]
    lib.agzo_glue_rmsnorm.argtypes = [vp, vp, i64, vp, i64, vp, i64, i64, f32]
    lib.agzo_glue_swiglu.argtypes = [vp, vp, i64, vp, i64, vp, i64, i64, i64]
    lib.agzo_glue_add.argtypes = [vp, vp, i64, vp, i64, i64, i64]
    lib.agzo_glue_attention.argtypes = [vp, vp, i64, vp, i64, vp, i64, vp, i64, i32, i32, i32, i32, f32]
    lib.agzo_step.argtypes = [vp, lp, vp, vp, sp, i32, f32, f32, u64, i32, vp]
    lib.agzo_step_no_update.argtypes = [vp, lp, vp, vp, sp, i32, f32, u64, i32, vp, vp]
    for name in EXPORTS:
        if name not in ("agzo_destroy", "agzo_last_error"):
            getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _dt(t):
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError("unsupported dtype %s" % t.dtype)


def make_layer(W=None, X=None, r=1, Y=None, d_out=None):
    """Descriptor for row-major 2-D tensors W [d_out][d_in], X [n][d_in], optional Y [n][d_out]."""
    L = AgzoLayer()
    L.n_tokens, L.d_in = X.shape
    L.d_out = W.shape[0] if W is not None else (d_out or 0)
    L.r = r
    L.dtype = _dt(X)
    L.y_dtype = _dt(Y) if Y is not None else F32
    L.ldx = X.stride(0)
    L.ldw = W.stride(0) if W is not None else L.d_in
    L.ldy = Y.stride(0) if Y is not None else L.d_out
    return L


def make_loss(target=None, kind=LOSS_MSE):
    s = AgzoLossSpec()
    if target is None:
        s.kind = LOSS_NONE
        return s
    s.kind = kind
    s.target = target.data_ptr()
    if kind == LOSS_CE and target.dtype != torch.int32:
        raise TypeError("cross-entropy targets must be int32 ids")
    if kind == LOSS_MSE:
        s.target_dtype = _dt(target)
        s.ldt = target.stride(0)
    return s


class Context:
    """Owns an agzo_ctx bound to a torch stream (default: the current one)."""

    def __init__(self, stream=None):
        self.lib = load()
        if not torch.cuda.is_available():
            raise RuntimeError("the AGZO HIP path needs a GPU")
        self.stream = stream if stream is not None else torch.cuda.current_stream()
        h = ctypes.c_void_p()
        rc = self.lib.agzo_create(ctypes.byref(h), ctypes.c_void_p(self.stream.cuda_stream))
        if rc != 0:
            raise AgzoError(rc, "agzo_create failed")
        self.h = h

    def close(self):
        if getattr(self, "h", None):
            self.lib.agzo_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _rc(self, rc):
        if rc != 0:
            raise AgzoError(rc, self.lib.agzo_last_error(self.h).decode())

    # --- one method per C entry point, same name without the prefix -------------------------
    def check(self):
        self._rc(self.lib.agzo_check(self.h))

    def profile_enable(self, on):
        """on: False / True (all kernel classes) or a mask of (1 << PROF_x) bits."""
        mask = (PROF_ALL if on else 0) if isinstance(on, bool) else int(on)
        self._rc(self.lib.agzo_profile_enable(self.h, mask))

    def profile_read(self, kind):
        n, ms = ctypes.c_int64(0), ctypes.c_double(0.0)
        self._rc(self.lib.agzo_profile_read(self.h, kind, ctypes.byref(n), ctypes.byref(ms)))
        return n.value, ms.value

    def profile_clock(self):
        n, ghz = ctypes.c_int64(0), ctypes.c_double(0.0)
        self._rc(self.lib.agzo_profile_clock(self.h, ctypes.byref(n), ctypes.byref(ghz)))
        return n.value, ghz.value

    def probe_mfma(self, operands, duty, iters):
        """operands: 32 KiB device tensor of bf16 bit patterns; duty 1..8 of 8 groups of 32x32x16 instructions, or 9 for
        the flop count of all 8 from 16x16x32 instructions.  Returns (TFLOP/s, shader clock in GHz)."""
        if operands.numel() * operands.element_size() < 32768 or not operands.is_contiguous():
            raise ValueError("operands must be a contiguous device tensor of at least 32 KiB")
        tf, ghz = ctypes.c_double(0.0), ctypes.c_double(0.0)
        self._rc(self.lib.agzo_probe_mfma(self.h, _ptr(operands), duty, iters, ctypes.byref(tf), ctypes.byref(ghz)))
        return tf.value, ghz.value

    def philox_words(self, dst, seed, tag):
        rows, cols = dst.shape
        self._rc(self.lib.agzo_philox_words(self.h, _ptr(dst), rows, cols, seed, tag))

    def fill_normal(self, dst, seed, tag):
        rows, cols = dst.shape
        self._rc(self.lib.agzo_fill_normal(self.h, _ptr(dst), rows, cols, seed, tag))

    def layer_forward_sketch(self, L, W, X, Y, mode, Q, seed, S, loss, loss_dev):
        self._rc(self.lib.agzo_layer_forward_sketch(self.h, ctypes.byref(L), _ptr(W), _ptr(X), _ptr(Y), mode,
                                                    _ptr(Q), seed, _ptr(S),
                                                    ctypes.byref(loss) if loss is not None else None,
                                                    _ptr(loss_dev)))

    def qr(self, S, Q):
        d, r = S.shape
        self._rc(self.lib.agzo_qr(self.h, _ptr(S), d, r, _ptr(Q)))

    def basis(self, L, X, K, seed, S0, flags, B):
        self._rc(self.lib.agzo_basis(self.h, ctypes.byref(L), _ptr(X), K, seed, _ptr(S0), flags, _ptr(B)))

    def perturbed_forward(self, L, W, X, B, seed, eps_signed, Y, loss, loss_dev):
        self._rc(self.lib.agzo_perturbed_forward(self.h, ctypes.byref(L), _ptr(W), _ptr(X), _ptr(B), seed,
                                                 eps_signed, _ptr(Y),
                                                 ctypes.byref(loss) if loss is not None else None, _ptr(loss_dev)))

    def two_point(self, out4_dev, eps, flags=0):
        if out4_dev.dtype != torch.float64 or out4_dev.numel() < 4 or not out4_dev.is_contiguous():
            raise TypeError("out4_dev must be 4 contiguous float64 values on the device")
        self._rc(self.lib.agzo_two_point(self.h, _ptr(out4_dev), eps, flags))

    def dense_perturb(self, theta, seed, scale, g_dev=None):
        """theta: 1-D (taken as one row) or 2-D device tensor, fp32 or bf16, unit stride along the last axis."""
        if theta.dim() == 1:
            rows, cols, ld = 1, theta.shape[0], theta.shape[0]
        else:
            rows, cols = theta.shape
            ld = theta.stride(0)
        if theta.numel() and theta.stride(-1) != 1:
            raise ValueError("theta must have unit stride along its last axis")
        self._rc(self.lib.agzo_dense_perturb(self.h, _ptr(theta), _dt(theta), rows, cols, ld, seed, scale, _ptr(g_dev)))

    def update(self, L, W, B, seed, lr, g_dev):
        self._rc(self.lib.agzo_update(self.h, ctypes.byref(L), _ptr(W), _ptr(B), seed, lr, _ptr(g_dev)))

    def update_noalloc(self, L, W, B, seed, lr, g_dev):
        self._rc(self.lib.agzo_update_noalloc(self.h, ctypes.byref(L), _ptr(W), _ptr(B), seed, lr, _ptr(g_dev)))

    def update_many(self, items):
        """items: sequence of (W, B, seed, lr, g_dev) with W a 2-D device tensor (unit stride along d_in), B [d_in][r]."""
        arr = (AgzoUpdateItem * max(len(items), 1))()
        for it, (W, B, seed, lr, g_dev) in zip(arr, items):
            it.W, it.B, it.g_dev = W.data_ptr(), B.data_ptr(), (0 if g_dev is None else g_dev.data_ptr())
            it.d_out, it.d_in, it.ldw = W.shape[0], W.shape[1], W.stride(0)
            it.r, it.dtype, it.seed, it.lr, it.reserved = B.shape[1], _dt(W), seed, lr, 0
        self.update_many_raw(arr, len(items))

    def update_many_raw(self, arr, n):
        self._rc(self.lib.agzo_update_many(self.h, arr, n))

    def basis_many(self, items, K, flags=0):
        """items: sequence of (L, X, seed, S0 or None, B)."""
        arr = (AgzoBasisItem * max(len(items), 1))()
        for it, (L, X, seed, S0, B) in zip(arr, items):
            it.layer, it.X, it.seed = L, X.data_ptr(), seed
            it.S0, it.B = (0 if S0 is None else S0.data_ptr()), B.data_ptr()
        self._rc(self.lib.agzo_basis_many(self.h, arr, len(items), K, flags))

    def make_step_items(self, items):
        """items: sequence of (L, W, X, loss, seed, out_dev, B_out or None) -> ctypes array for step_many_raw (the seeds
        can be rewritten in place between steps)."""
        arr = (AgzoStepItem * max(len(items), 1))()
        for it, (L, W, X, loss, seed, out_dev, B_out) in zip(arr, items):
            it.layer, it.W, it.X, it.loss, it.seed = L, W.data_ptr(), X.data_ptr(), loss, seed
            it.out_dev, it.B_out = out_dev.data_ptr(), (0 if B_out is None else B_out.data_ptr())
        return arr

    def step_many_raw(self, arr, n, K, eps, lr, flags=0):
        self._rc(self.lib.agzo_step_many(self.h, arr, n, K, eps, lr, flags))

    def step_many(self, items, K, eps, lr, flags=0):
        self.step_many_raw(self.make_step_items(items), len(items), K, eps, lr, flags)

    def glue_rmsnorm(self, x, y, gain=None, eps=1e-6):
        n, d = x.shape
        self._rc(self.lib.agzo_glue_rmsnorm(self.h, _ptr(x), x.stride(0), _ptr(y), y.stride(0), _ptr(gain), n, d, eps))

    def glue_swiglu(self, a, u, m):
        n, d = a.shape
        self._rc(self.lib.agzo_glue_swiglu(self.h, _ptr(a), a.stride(0), _ptr(u), u.stride(0), _ptr(m), m.stride(0), n, d))

    def glue_add(self, h, delta):
        n, d = h.shape
        self._rc(self.lib.agzo_glue_add(self.h, _ptr(h), h.stride(0), _ptr(delta), delta.stride(0), n, d))

    def glue_attention(self, q, k, v, out, n_seq, seq_len, rope_theta=1.0e6):
        n_heads, n_kv = q.shape[1] // 128, k.shape[1] // 128
        self._rc(self.lib.agzo_glue_attention(self.h, _ptr(q), q.stride(0), _ptr(k), k.stride(0), _ptr(v), v.stride(0),
                                              _ptr(out), out.stride(0), n_seq, seq_len, n_heads, n_kv, rope_theta))

    def step_no_update(self, L, W, X, loss, K, eps, seed, flags, out_dev, B_out):
        self._rc(self.lib.agzo_step_no_update(self.h, ctypes.byref(L), _ptr(W), _ptr(X), ctypes.byref(loss), K, eps,
                                              seed, flags, _ptr(out_dev), _ptr(B_out)))

    def step(self, L, W, X, loss, K, eps, lr, seed, flags, out_dev):
        self._rc(self.lib.agzo_step(self.h, ctypes.byref(L), _ptr(W), _ptr(X), ctypes.byref(loss), K, eps, lr,
                                    seed, flags, _ptr(out_dev)))
