"""ctypes/numpy front end of the C oracle (oracle/f8_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
cpu_baseline leg of bench.py.  The product package never imports it, and this
module never imports the product package.

All arrays are numpy, host memory: bf16 as uint16 bit patterns, fp8 as uint8
codes, scales as float32.
"""
import ctypes as C
import os

import numpy as np

from . import build_oracle

E4M3, E5M2 = 0, 1
TENSORWISE, ROWWISE, COLWISE = 0, 1, 2
NT, NN, TN = 0, 1, 2

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = build_oracle.build(force=False)
        _lib = C.CDLL(path)
        _declare(_lib)
    return _lib


_i64, _int, _f32 = C.c_int64, C.c_int, C.c_float
_p = C.c_void_p


class QTensor(C.Structure):
    _fields_ = [("q", _p), ("amax", _p), ("scale", _p), ("inv_scale", _p),
                ("q_c", _p), ("amax_c", _p), ("scale_c", _p), ("inv_scale_c", _p)]


def _declare(l):
    l.f8o_fmax.restype = _f32
    l.f8o_fmax.argtypes = [_int]
    l.f8o_bf16_to_f32.restype = _f32
    l.f8o_bf16_to_f32.argtypes = [C.c_uint16]
    l.f8o_f32_to_bf16.restype = C.c_uint16
    l.f8o_f32_to_bf16.argtypes = [_f32]
    l.f8o_decode.restype = _f32
    l.f8o_decode.argtypes = [C.c_uint8, _int]
    l.f8o_encode.restype = C.c_uint8
    l.f8o_encode.argtypes = [_f32, _int]
    l.f8o_cast_one.restype = C.c_uint8
    l.f8o_cast_one.argtypes = [C.c_uint16, _f32, _int]
    l.f8o_amax.restype = None
    l.f8o_amax.argtypes = [_p, _i64, _i64, _i64, _int, _p]
    l.f8o_scale.restype = None
    l.f8o_scale.argtypes = [_p, _i64, _int, _p, _p]
    l.f8o_silu_mul.restype = None
    l.f8o_silu_mul.argtypes = [_p, _i64, _i64, _p, _p]
    l.f8o_silu_mul_bwd.restype = None
    l.f8o_silu_mul_bwd.argtypes = [_p, _p, _i64, _i64, _p, _p]
    l.f8o_rmsnorm.restype = None
    l.f8o_rmsnorm.argtypes = [_p, _p, _i64, _i64, C.c_double, _p, _p, _p]
    l.f8o_history_push.restype = None
    l.f8o_history_push.argtypes = [_p, _i64, _f32, _int, _p, _p]
    l.f8o_cast.restype = None
    l.f8o_cast.argtypes = [_p, _i64, _i64, _i64, _p, _int, _int, _p, _i64, _p, _i64]
    l.f8o_gemm.restype = None
    l.f8o_gemm.argtypes = [_int, _i64, _i64, _i64, _p, _int, _i64, _p, _int, _i64, _p, _p, _int, _p, _i64]
    l.f8o_gemm_f64.restype = None
    l.f8o_gemm_f64.argtypes = [_int, _i64, _i64, _i64, _p, _int, _i64, _p, _int, _i64, _p, _p, _int, _p, _p, _i64]
    l.f8o_gemm_points.restype = None
    l.f8o_gemm_points.argtypes = [_int, _i64, _p, _int, _i64, _p, _int, _i64, _p, _p, _int, _p, _p, _i64, _p]
    l.f8o_linear_fwd.restype = None
    l.f8o_linear_fwd.argtypes = [_i64, _i64, _i64, _int, _p, _p, _p, C.POINTER(QTensor), C.POINTER(QTensor)]
    l.f8o_linear_bwd.restype = None
    l.f8o_linear_bwd.argtypes = [_i64, _i64, _i64, _int, _int, _p, C.POINTER(QTensor), C.POINTER(QTensor),
                                 C.POINTER(QTensor), _p, _p]
    l.f8o_num_threads.restype = _int
    l.f8o_num_threads.argtypes = []


def _ptr(a):
    return None if a is None else a.ctypes.data_as(_p)


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


# ---- scalars ---------------------------------------------------------------

def fmax(fmt):
    return float(lib().f8o_fmax(fmt))


def bf16_to_f32(bits):
    """uint16 array of bf16 bit patterns -> float32 array (exact)."""
    bits = np.asarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << 16).view(np.float32)


def f32_to_bf16(x):
    """float32 array -> uint16 bf16 bits, RNE, element by element through C."""
    x = np.asarray(x, dtype=np.float32)
    f = lib().f8o_f32_to_bf16
    out = np.fromiter((f(float(v)) for v in x.ravel()), dtype=np.uint16, count=x.size)
    return out.reshape(x.shape)


def decode(codes, fmt):
    codes = np.asarray(codes, dtype=np.uint8)
    f = lib().f8o_decode
    table = np.array([f(c, fmt) for c in range(256)], dtype=np.float32)
    return table[codes]


def encode(y, fmt):
    """float32 array (finite, |y| <= FMAX, or NaN) -> uint8 codes."""
    y = np.asarray(y, dtype=np.float32)
    f = lib().f8o_encode
    out = np.fromiter((f(float(v), fmt) for v in y.ravel()), dtype=np.uint8, count=y.size)
    return out.reshape(y.shape)


# ---- steps -----------------------------------------------------------------

def _nscales(rows, cols, gran):
    return 1 if gran == TENSORWISE else (rows if gran == ROWWISE else cols)


def amax(x_bits, gran=TENSORWISE):
    x = _c(x_bits, np.uint16)
    rows, cols = x.shape
    out = np.empty(_nscales(rows, cols, gran), dtype=np.float32)
    lib().f8o_amax(_ptr(x), rows, cols, cols, gran, _ptr(out))
    return out


def scale(amax_arr, fmt):
    a = _c(np.atleast_1d(amax_arr), np.float32)
    s = np.empty_like(a)
    inv = np.empty_like(a)
    lib().f8o_scale(_ptr(a), a.size, fmt, _ptr(s), _ptr(inv))
    return s, inv


def cast(x_bits, scale_arr, gran=TENSORWISE, fmt=E4M3, transposed=False):
    x = _c(x_bits, np.uint16)
    rows, cols = x.shape
    s = _c(np.atleast_1d(scale_arr), np.float32)
    assert s.size == _nscales(rows, cols, gran)
    out = np.empty((rows, cols), dtype=np.uint8)
    out_t = np.empty((cols, rows), dtype=np.uint8) if transposed else None
    lib().f8o_cast(_ptr(x), rows, cols, cols, _ptr(s), gran, fmt, _ptr(out), cols,
                   _ptr(out_t), rows)
    return (out, out_t) if transposed else out


def amax_cast(x_bits, gran=TENSORWISE, fmt=E4M3):
    """The dynamic-scaling composition: amax -> scale -> cast."""
    a = amax(x_bits, gran)
    s, inv = scale(a, fmt)
    return a, s, inv, cast(x_bits, s, gran, fmt)


def _gemm_dims(layout, A, B):
    if layout == NT:
        (M, K), (N, K2) = A.shape, B.shape
    elif layout == NN:
        (M, K), (K2, N) = A.shape, B.shape
    else:
        (K, M), (K2, N) = A.shape, B.shape
    assert K == K2, (A.shape, B.shape, layout)
    return M, N, K


def gemm(layout, A, fa, B, fb, inv_sa, inv_sb, gran=TENSORWISE):
    """bf16 bits of D[M,N]; fp32 accumulation in ascending k."""
    A, B = _c(A, np.uint8), _c(B, np.uint8)
    M, N, K = _gemm_dims(layout, A, B)
    sa, sb = _c(np.atleast_1d(inv_sa), np.float32), _c(np.atleast_1d(inv_sb), np.float32)
    D = np.empty((M, N), dtype=np.uint16)
    lib().f8o_gemm(layout, M, N, K, _ptr(A), fa, A.shape[1], _ptr(B), fb, B.shape[1],
                   _ptr(sa), _ptr(sb), gran, _ptr(D), N)
    return D


def gemm_f64(layout, A, fa, B, fb, inv_sa, inv_sb, gran=TENSORWISE):
    """(D, Dabs): the unrounded fp64 result and sum_k |a||b| * |scales|."""
    A, B = _c(A, np.uint8), _c(B, np.uint8)
    M, N, K = _gemm_dims(layout, A, B)
    sa, sb = _c(np.atleast_1d(inv_sa), np.float32), _c(np.atleast_1d(inv_sb), np.float32)
    D = np.empty((M, N), dtype=np.float64)
    Dabs = np.empty((M, N), dtype=np.float64)
    lib().f8o_gemm_f64(layout, M, N, K, _ptr(A), fa, A.shape[1], _ptr(B), fb, B.shape[1],
                       _ptr(sa), _ptr(sb), gran, _ptr(D), _ptr(Dabs), N)
    return D, Dabs


def gemm_points(layout, A, fa, B, fb, inv_sa, inv_sb, ms, ns, gran=TENSORWISE):
    """bf16 bits of D[ms[i], ns[i]] for the listed output positions only."""
    A, B = _c(A, np.uint8), _c(B, np.uint8)
    M, N, K = _gemm_dims(layout, A, B)
    sa, sb = _c(np.atleast_1d(inv_sa), np.float32), _c(np.atleast_1d(inv_sb), np.float32)
    ms, ns = _c(ms, np.int64), _c(ns, np.int64)
    assert ms.shape == ns.shape and ms.max(initial=0) < M and ns.max(initial=0) < N
    out = np.empty(ms.size, dtype=np.uint16)
    lib().f8o_gemm_points(layout, K, _ptr(A), fa, A.shape[1], _ptr(B), fb, B.shape[1],
                          _ptr(sa), _ptr(sb), gran, _ptr(ms), _ptr(ns), ms.size, _ptr(out))
    return out.reshape(ms.shape)


# ---- the linear layer --------------------------------------------------------

class Quantised:
    """Host-side saved state of one tensor (numpy arrays kept alive here)."""

    def __init__(self, rows, cols, rowwise):
        n = rows if rowwise else 1
        self.q = np.zeros((rows, cols), np.uint8)
        self.amax = np.zeros(n, np.float32)
        self.scale = np.zeros(n, np.float32)
        self.inv_scale = np.zeros(n, np.float32)
        if rowwise:
            self.q_c = np.zeros((rows, cols), np.uint8)
            self.amax_c = np.zeros(cols, np.float32)
            self.scale_c = np.zeros(cols, np.float32)
            self.inv_scale_c = np.zeros(cols, np.float32)
        else:
            self.q_c = self.amax_c = self.scale_c = self.inv_scale_c = None

    def struct(self):
        return QTensor(_ptr(self.q), _ptr(self.amax), _ptr(self.scale), _ptr(self.inv_scale),
                       _ptr(self.q_c), _ptr(self.amax_c), _ptr(self.scale_c), _ptr(self.inv_scale_c))


def linear_fwd(X_bits, W_bits, rowwise=False):
    """Returns (Y bf16 bits [M,N], xq, wq)."""
    X, W = _c(X_bits, np.uint16), _c(W_bits, np.uint16)
    (M, K), (N, K2) = X.shape, W.shape
    assert K == K2
    xq, wq = Quantised(M, K, rowwise), Quantised(N, K, rowwise)
    Y = np.empty((M, N), np.uint16)
    xs, ws = xq.struct(), wq.struct()
    lib().f8o_linear_fwd(M, K, N, int(rowwise), _ptr(X), _ptr(W), _ptr(Y), C.byref(xs), C.byref(ws))
    return Y, xq, wq


def linear_bwd(dY_bits, xq, wq, rowwise=False, grad_fmt=E4M3):
    """Returns (dX bf16 bits [M,K], dW bf16 bits [N,K], dyq)."""
    dY = _c(dY_bits, np.uint16)
    M, N = dY.shape
    K = xq.q.shape[1]
    dyq = Quantised(M, N, rowwise)
    dX = np.empty((M, K), np.uint16)
    dW = np.empty((N, K), np.uint16)
    xs, ws, ds = xq.struct(), wq.struct(), dyq.struct()
    lib().f8o_linear_bwd(M, K, N, int(rowwise), grad_fmt, _ptr(dY), C.byref(xs), C.byref(ws),
                         C.byref(ds), _ptr(dX), _ptr(dW))
    return dX, dW, dyq


# ---- delayed / static scaling (tensorwise) ------------------------------------------

DYNAMIC, DELAYED, STATIC = 0, 1, 2


def history_push(history, amax_new, fmt):
    """In place: record amax_new in `history` (float32, newest first).  Returns the scale of
    the next step and its reciprocal, as float32 arrays of one element."""
    assert history.dtype == np.float32 and history.flags.c_contiguous
    s, inv = np.empty(1, np.float32), np.empty(1, np.float32)
    lib().f8o_history_push(_ptr(history), history.size, float(np.float32(amax_new)), fmt, _ptr(s), _ptr(inv))
    return s, inv


class ScalingState:
    """Per tensor (x, w, dy): the amax history (zeros at first) and the scale the next cast uses."""

    def __init__(self, mode, history_len=16):
        self.mode = mode
        self.hist = {k: np.zeros(history_len, np.float32) for k in ("x", "w", "dy")}
        self.scale = {k: np.ones(1, np.float32) for k in ("x", "w", "dy")}


def _quantise_scaled(bits, fmt, state, key):
    """One tensor under delayed or static scaling.  Returns a tensorwise Quantised whose scale
    is the one the codes were made with; amax is this step's (delayed) or None (static)."""
    rows, cols = bits.shape
    q = Quantised(rows, cols, False)
    s = state.scale[key].copy()
    q.scale[:] = s
    q.inv_scale[:] = np.float32(1.0) / s
    q.q[:] = cast(bits, s, TENSORWISE, fmt)
    if state.mode == DELAYED:
        q.amax[:] = amax(bits, TENSORWISE)
        state.scale[key], _ = history_push(state.hist[key], q.amax[0], fmt)
    else:
        q.amax = None
    return q


def linear_fwd_scaled(X_bits, W_bits, state):
    """Forward under delayed / static scaling.  Returns (Y bits, xq, wq); updates `state`."""
    X, W = _c(X_bits, np.uint16), _c(W_bits, np.uint16)
    xq = _quantise_scaled(X, E4M3, state, "x")
    wq = _quantise_scaled(W, E4M3, state, "w")
    Y = gemm(NT, xq.q, E4M3, wq.q, E4M3, xq.inv_scale, wq.inv_scale, TENSORWISE)
    return Y, xq, wq


def linear_bwd_scaled(dY_bits, xq, wq, state, grad_fmt=E4M3):
    """Backward under delayed / static scaling.  Returns (dX bits, dW bits, dyq)."""
    dY = _c(dY_bits, np.uint16)
    dyq = _quantise_scaled(dY, grad_fmt, state, "dy")
    dX = gemm(NN, dyq.q, grad_fmt, wq.q, E4M3, dyq.inv_scale, wq.inv_scale, TENSORWISE)
    dW = gemm(TN, dyq.q, grad_fmt, xq.q, E4M3, dyq.inv_scale, xq.inv_scale, TENSORWISE)
    return dX, dW, dyq


# ---- feed-forward glue ----------------------------------------------------------------

def silu_mul(ab_bits):
    """ab [M, 2H] = [a | b] bf16 bits -> (h [M, H] bits = bf16(silu(a) * b), amax of h)."""
    ab = _c(ab_bits, np.uint16)
    M, H2 = ab.shape
    h = np.empty((M, H2 // 2), np.uint16)
    am = np.empty(1, np.float32)
    lib().f8o_silu_mul(_ptr(ab), M, H2 // 2, _ptr(h), _ptr(am))
    return h, am


def silu_mul_bwd(ab_bits, dh_bits):
    """-> (dab [M, 2H] bits = [dh * b * silu'(a) | dh * silu(a)], amax of dab)."""
    ab, dh = _c(ab_bits, np.uint16), _c(dh_bits, np.uint16)
    M, H2 = ab.shape
    assert dh.shape == (M, H2 // 2)
    dab = np.empty((M, H2), np.uint16)
    am = np.empty(1, np.float32)
    lib().f8o_silu_mul_bwd(_ptr(ab), _ptr(dh), M, H2 // 2, _ptr(dab), _ptr(am))
    return dab, am


def rmsnorm(x_bits, g_bits, eps=1e-5):
    """-> (y [M, D] bf16 bits, rstd [M] fp32, amax of y)."""
    x, g = _c(x_bits, np.uint16), _c(g_bits, np.uint16)
    M, D = x.shape
    assert g.shape == (D,)
    y, rstd, am = np.empty((M, D), np.uint16), np.empty(M, np.float32), np.empty(1, np.float32)
    lib().f8o_rmsnorm(_ptr(x), _ptr(g), M, D, float(eps), _ptr(y), _ptr(rstd), _ptr(am))
    return y, rstd, am


def num_threads():
    return int(lib().f8o_num_threads())
