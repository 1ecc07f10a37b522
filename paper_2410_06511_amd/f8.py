"""ctypes binding of libf8.so: the same names as include/f8.h, argument
marshalling only.  Tensors are torch tensors on the GPU (used for memory and
streams); every step of the computation runs in the library's kernels.

The library is loaded on first use; if it has not been built this raises
(there is no fallback path).
"""
import ctypes as C
import os

import torch

E4M3, E5M2 = 0, 1
TENSORWISE, ROWWISE, COLWISE = 0, 1, 2
NT, NN, TN = 0, 1, 2
DYNAMIC, DELAYED, STATIC = 0, 1, 2
MAX_HISTORY = 1024

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libf8.so")
_lib = None

_i64, _int, _p = C.c_int64, C.c_int, C.c_void_p

EXPORTS = ["f8_workspace_bytes", "f8_status_string", "f8_amax", "f8_scale", "f8_cast", "f8_encode_f32",
           "f8_amax_cast", "f8_gemm", "f8_gemm_ws", "f8_linear_fwd", "f8_linear_bwd", "f8_cast_amax",
           "f8_amax_history_push", "f8_linear_fwd_scaled", "f8_linear_bwd_scaled",
           "f8_linear_fwd_chained", "f8_linear_bwd_chained", "f8_quantise",
           "f8_silu_mul", "f8_silu_mul_bwd", "f8_rmsnorm", "f8_silu_mul_quantise_delayed", "f8_linear_fwd_xq",
           "f8_silu_mul_bwd_quantise_delayed", "f8_linear_bwd_dyq",
           "f8_rope", "f8_transpose_bf16", "f8_add", "f8_rmsnorm_bwd", "f8_sdpa_fwd", "f8_sdpa_bwd", "f8_sdpa_bwd_workspace_bytes",
           "f8_rmsnorm_bwd_add", "f8_linear_fwd_wq", "f8_linear_fwd_noalloc", "f8_linear_fwd_quantise",
           "f8_probe_mfma", "f8_probe_copy", "f8_probe_read", "f8_probe_clock"]


class F8Error(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"f8 status {code}: {msg}")
        self.code = code


class QTensorStruct(C.Structure):
    _fields_ = [("q", _p), ("q_t", _p), ("amax", _p), ("scale", _p), ("inv_scale", _p),
                ("amax_t", _p), ("scale_t", _p), ("inv_scale_t", _p)]


class SavedStruct(C.Structure):
    _fields_ = [("x", QTensorStruct), ("w", QTensorStruct), ("dy", QTensorStruct)]


class LinearDesc(C.Structure):
    _fields_ = [("M", _i64), ("K", _i64), ("N", _i64), ("granularity", C.c_int32), ("grad_format", C.c_int32)]


class ScalingStateStruct(C.Structure):
    _fields_ = [("mode", C.c_int32), ("history_len", C.c_int32), ("hist_x", _p), ("hist_w", _p), ("hist_dy", _p),
                ("scale_x", _p), ("scale_w", _p), ("scale_dy", _p)]


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2410_06511_amd.build`")
        l = C.CDLL(LIB_PATH)
        l.f8_workspace_bytes.restype = C.c_size_t
        l.f8_workspace_bytes.argtypes = [_i64, _i64]
        l.f8_status_string.restype = C.c_char_p
        l.f8_status_string.argtypes = [_int]
        l.f8_amax.argtypes = [_p, _i64, _i64, _i64, _int, _p, _p, C.c_size_t, _p]
        l.f8_scale.argtypes = [_p, _i64, _int, _p, _p, _p]
        l.f8_cast.argtypes = [_p, _i64, _i64, _i64, _p, _int, _int, _p, _i64, _p, _i64, _p]
        l.f8_encode_f32.argtypes = [_p, _i64, _int, _int, _p, _p]
        l.f8_amax_cast.argtypes = [_p, _i64, _i64, _i64, _int, _int, _p, _p, _p, _p, _i64, _p, _i64, _p,
                                   C.c_size_t, _p]
        l.f8_gemm.argtypes = [_int, _i64, _i64, _i64, _p, _int, _i64, _p, _int, _i64, _p, _p, _int, _p, _i64, _p, _p]
        l.f8_gemm_ws.argtypes = [_int, _i64, _i64, _i64, _p, _int, _i64, _p, _int, _i64, _p, _p, _int, _p, _i64, _p, _p,
                                 C.c_size_t, _p]
        l.f8_linear_fwd.argtypes = [C.POINTER(LinearDesc), _p, _p, _p, C.POINTER(SavedStruct), _p, C.c_size_t, _p]
        l.f8_linear_bwd.argtypes = [C.POINTER(LinearDesc), _p, C.POINTER(SavedStruct), _p, _p, _p, C.c_size_t, _p]
        l.f8_linear_fwd_quantise.argtypes = [C.POINTER(LinearDesc), _p, _p, C.POINTER(SavedStruct), _p, C.c_size_t, _p]
        l.f8_cast_amax.argtypes = [_p, _i64, _i64, _i64, _p, _int, _p, _i64, _p, _i64, _p, _p, C.c_size_t, _p]
        l.f8_amax_history_push.argtypes = [_p, _i64, _p, _int, _p, _p, _p]
        l.f8_linear_fwd_scaled.argtypes = [C.POINTER(LinearDesc), C.POINTER(ScalingStateStruct), _p, _p, _p,
                                           C.POINTER(SavedStruct), _p, C.c_size_t, _p]
        l.f8_linear_bwd_scaled.argtypes = [C.POINTER(LinearDesc), C.POINTER(ScalingStateStruct), _p,
                                           C.POINTER(SavedStruct), _p, _p, _p, C.c_size_t, _p]
        l.f8_linear_fwd_chained.argtypes = [C.POINTER(LinearDesc), _p, _p, _p, _p, _p, C.POINTER(SavedStruct), _p,
                                            C.c_size_t, _p]
        l.f8_linear_bwd_chained.argtypes = [C.POINTER(LinearDesc), _p, _p, C.POINTER(SavedStruct), _p, _p, _p, _p,
                                            C.c_size_t, _p]
        l.f8_quantise.argtypes = [_p, _i64, _i64, _int, _int, C.POINTER(QTensorStruct), _p, C.c_size_t, _p]
        l.f8_silu_mul.argtypes = [_p, _i64, _i64, _p, _p, _p, C.c_size_t, _p]
        l.f8_silu_mul_bwd.argtypes = [_p, _p, _i64, _i64, _p, _p, _p, C.c_size_t, _p]
        l.f8_rmsnorm.argtypes = [_p, _p, _i64, _i64, C.c_float, _p, _p, _p, _p, C.c_size_t, _p]
        l.f8_silu_mul_quantise_delayed.argtypes = [_p, _i64, _i64, _int, _p, _i64, _p, C.POINTER(QTensorStruct), _p,
                                                   C.c_size_t, _p]
        l.f8_linear_fwd_xq.argtypes = [C.POINTER(LinearDesc), C.POINTER(ScalingStateStruct), _p, _p,
                                       C.POINTER(SavedStruct), _p, C.c_size_t, _p]
        l.f8_silu_mul_bwd_quantise_delayed.argtypes = [_p, _p, _i64, _i64, _int, _p, _i64, _p, C.POINTER(QTensorStruct),
                                                       _p, C.c_size_t, _p]
        l.f8_linear_bwd_dyq.argtypes = [C.POINTER(LinearDesc), C.POINTER(SavedStruct), _p, _p, _p]
        l.f8_rope.argtypes = [_p, _i64, _i64, _i64, _i64, _i64, C.c_double, _int, _p, _i64, _p, _p, _p]
        l.f8_transpose_bf16.argtypes = [_p, _i64, _i64, _i64, _p, _p]
        l.f8_add.argtypes = [_p, _p, _i64, _p, _p]
        l.f8_rmsnorm_bwd.argtypes = [_p, _p, _p, _p, _i64, _i64, _p, _p, _p, C.c_size_t, _p]
        l.f8_linear_fwd_wq.argtypes = [C.POINTER(LinearDesc), _p, _p, C.POINTER(SavedStruct), _p, C.c_size_t, _p]
        l.f8_linear_fwd_noalloc.argtypes = [C.POINTER(LinearDesc), _p, _p, _p, C.POINTER(SavedStruct), _p]
        l.f8_probe_mfma.argtypes = [_int, _p, _i64, _int, _p, _p, C.POINTER(_i64), _p]
        l.f8_probe_copy.argtypes = [_p, _p, _i64, _p]
        l.f8_probe_read.argtypes = [_p, _i64, _p, _p]
        l.f8_probe_clock.argtypes = [_p, _p]
        l.f8_rmsnorm_bwd_add.argtypes = [_p, _p, _p, _p, _p, _i64, _i64, _p, _p, _p, _p, C.c_size_t, _p]
        l.f8_sdpa_fwd.argtypes = [_p, _i64, _p, _i64, _p, _i64, _i64, _i64, _i64, _i64, _p, _i64, _p, _p, _p]
        l.f8_sdpa_bwd.argtypes = [_p, _i64, _p, _p, _i64, _p, _p, _i64, _p, _i64, _p, _i64, _p, _p, _i64, _i64, _i64, _i64,
                                  _i64, _p, _i64, _p, _i64, _p, _i64, _p, _p, _p, C.c_size_t, _p]
        l.f8_sdpa_bwd_workspace_bytes.argtypes = [_i64] * 5
        for name in EXPORTS[2:]:
            getattr(l, name).restype = _int
        l.f8_sdpa_bwd_workspace_bytes.restype = C.c_size_t
        _lib = l
    return _lib


def _check(code):
    if code != 0:
        raise F8Error(code, lib().f8_status_string(code).decode())


def _ptr(t):
    return None if t is None else t.data_ptr()


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream


def status_string(code):
    return lib().f8_status_string(code).decode()


def workspace_bytes(max_rows, max_cols):
    return int(lib().f8_workspace_bytes(max_rows, max_cols))


def new_workspace(max_rows, max_cols, device="cuda"):
    return torch.empty(workspace_bytes(max_rows, max_cols), dtype=torch.uint8, device=device)


def _ws(ws):
    return (None, 0) if ws is None else (ws.data_ptr(), ws.numel() * ws.element_size())


# ---- the entry points, one to one --------------------------------------------

def amax(x, g, amax_out, workspace=None, stream=None):
    rows, cols = x.shape
    wp, wb = _ws(workspace)
    _check(lib().f8_amax(_ptr(x), rows, cols, x.stride(0), g, _ptr(amax_out), wp, wb, _stream(stream)))


def scale(amax_t, fmt, scale_out, inv_scale_out=None, stream=None):
    _check(lib().f8_scale(_ptr(amax_t), amax_t.numel(), fmt, _ptr(scale_out), _ptr(inv_scale_out), _stream(stream)))


def cast(x, scale_t, g, fmt, out=None, out_t=None, stream=None):
    rows, cols = x.shape
    _check(lib().f8_cast(_ptr(x), rows, cols, x.stride(0), _ptr(scale_t), g, fmt,
                         _ptr(out), 0 if out is None else out.stride(0),
                         _ptr(out_t), 0 if out_t is None else out_t.stride(0), _stream(stream)))


def encode_f32(y, fmt, use_hw_convert, out, stream=None):
    _check(lib().f8_encode_f32(_ptr(y), y.numel(), fmt, int(use_hw_convert), _ptr(out), _stream(stream)))


def amax_cast(x, g, fmt, amax_out, scale_out, inv_scale_out, out=None, out_t=None, workspace=None, stream=None):
    rows, cols = x.shape
    wp, wb = _ws(workspace)
    _check(lib().f8_amax_cast(_ptr(x), rows, cols, x.stride(0), g, fmt, _ptr(amax_out), _ptr(scale_out),
                              _ptr(inv_scale_out), _ptr(out), 0 if out is None else out.stride(0),
                              _ptr(out_t), 0 if out_t is None else out_t.stride(0), wp, wb, _stream(stream)))


def gemm(layout, M, N, K, A, fa, B, fb, inv_scale_a, inv_scale_b, g, D, stream=None, amax_d=None, workspace=None):
    """f8_gemm, or f8_gemm_ws when a workspace is given."""
    if workspace is None:
        _check(lib().f8_gemm(layout, M, N, K, _ptr(A), fa, A.stride(0), _ptr(B), fb, B.stride(0),
                             _ptr(inv_scale_a), _ptr(inv_scale_b), g, _ptr(D), D.stride(0), _ptr(amax_d),
                             _stream(stream)))
        return
    wp, wb = _ws(workspace)
    _check(lib().f8_gemm_ws(layout, M, N, K, _ptr(A), fa, A.stride(0), _ptr(B), fb, B.stride(0),
                            _ptr(inv_scale_a), _ptr(inv_scale_b), g, _ptr(D), D.stride(0), _ptr(amax_d), wp, wb,
                            _stream(stream)))


class QTensor:
    """Device buffers of one quantised tensor T[rows, cols] (see f8_qtensor).  q_t (the codes
    transposed) exists under rowwise scaling, where it holds the per-column-scaled codes, and
    with transposed=True; otherwise it is None and the backward products read q in place."""

    def __init__(self, rows, cols, rowwise, device="cuda", transposed=False):
        u8 = dict(dtype=torch.uint8, device=device)
        f32 = dict(dtype=torch.float32, device=device)
        self.q = torch.empty((rows, cols), **u8)
        self.q_t = torch.empty((cols, rows), **u8) if (rowwise or transposed) else None
        n = rows if rowwise else 1
        self.amax, self.scale, self.inv_scale = (torch.empty(n, **f32) for _ in range(3))
        if rowwise:
            self.amax_t, self.scale_t, self.inv_scale_t = (torch.empty(cols, **f32) for _ in range(3))
        else:
            self.amax_t = self.scale_t = self.inv_scale_t = None

    def struct(self):
        return QTensorStruct(_ptr(self.q), _ptr(self.q_t), _ptr(self.amax), _ptr(self.scale), _ptr(self.inv_scale),
                             _ptr(self.amax_t), _ptr(self.scale_t), _ptr(self.inv_scale_t))


class Saved:
    """f8_saved for one linear: X [M,K], W [N,K], dY [M,N]."""

    def __init__(self, M, K, N, rowwise=False, device="cuda", transposed=False, x=None):
        """x: the QTensor of another linear that reads the same input (its codes are then shared, not copied)."""
        self.x = x if x is not None else QTensor(M, K, rowwise, device, transposed)
        self.w = QTensor(N, K, rowwise, device, transposed)
        self.dy = QTensor(M, N, rowwise, device, transposed)
        self._struct = SavedStruct(self.x.struct(), self.w.struct(), self.dy.struct())

    def struct(self):
        return self._struct


def quantise(t, g, fmt, q, workspace, stream=None):
    """q: QTensor.  Both orientations of t under dynamic scaling (see f8_quantise)."""
    rows, cols = t.shape
    wp, wb = _ws(workspace)
    st = q.struct()
    _check(lib().f8_quantise(_ptr(t), rows, cols, g, fmt, C.byref(st), wp, wb, _stream(stream)))


def linear_desc(M, K, N, rowwise=False, grad_format=E4M3):
    return LinearDesc(M, K, N, ROWWISE if rowwise else TENSORWISE, grad_format)


def linear_fwd(desc, X, W, Y, saved, workspace, stream=None):
    wp, wb = _ws(workspace)
    _check(lib().f8_linear_fwd(C.byref(desc), _ptr(X), _ptr(W), _ptr(Y), C.byref(saved.struct()), wp, wb,
                               _stream(stream)))


def linear_fwd_quantise(desc, X, W, saved, workspace, stream=None):
    """The quantisation half of linear_fwd: X and W into saved.x, saved.w, no product."""
    wp, wb = _ws(workspace)
    _check(lib().f8_linear_fwd_quantise(C.byref(desc), _ptr(X), _ptr(W), C.byref(saved.struct()), wp, wb, _stream(stream)))


def linear_fwd_noalloc(desc, X, W, Y, saved, stream=None):
    """linear_fwd on the library's built-in scratch: no workspace argument, nothing allocated."""
    _check(lib().f8_linear_fwd_noalloc(C.byref(desc), _ptr(X), _ptr(W), _ptr(Y), C.byref(saved.struct()), _stream(stream)))


def linear_fwd_wq(desc, X, Y, saved, workspace, stream=None):
    """Forward with the weight's codes kept in saved.w from an earlier linear_fwd."""
    wp, wb = _ws(workspace)
    _check(lib().f8_linear_fwd_wq(C.byref(desc), _ptr(X), _ptr(Y), C.byref(saved.struct()), wp, wb, _stream(stream)))


def linear_bwd(desc, dY, saved, dX, dW, workspace, stream=None):
    wp, wb = _ws(workspace)
    _check(lib().f8_linear_bwd(C.byref(desc), _ptr(dY), C.byref(saved.struct()), _ptr(dX), _ptr(dW), wp, wb,
                               _stream(stream)))


# ---- delayed / static scaling ----------------------------------------------------

def cast_amax(x, scale_t, fmt, amax_out, out=None, out_t=None, workspace=None, stream=None):
    rows, cols = x.shape
    wp, wb = _ws(workspace)
    _check(lib().f8_cast_amax(_ptr(x), rows, cols, x.stride(0), _ptr(scale_t), fmt,
                              _ptr(out), 0 if out is None else out.stride(0),
                              _ptr(out_t), 0 if out_t is None else out_t.stride(0), _ptr(amax_out), wp, wb,
                              _stream(stream)))


def amax_history_push(history, amax_new, fmt, scale_out, inv_scale_out=None, stream=None):
    _check(lib().f8_amax_history_push(_ptr(history), history.numel(), _ptr(amax_new), fmt, _ptr(scale_out),
                                      _ptr(inv_scale_out), _stream(stream)))


class ScalingState:
    """Device buffers of f8_scaling_state: per tensor (x, w, dy) an amax history (newest first,
    zero-initialised) and the scale the next cast uses."""

    def __init__(self, mode, history_len=16, device="cuda"):
        f32 = dict(dtype=torch.float32, device=device)
        self.mode, self.history_len = mode, history_len
        self.hist_x, self.hist_w, self.hist_dy = (torch.zeros(history_len, **f32) for _ in range(3))
        self.scale_x, self.scale_w, self.scale_dy = (torch.ones(1, **f32) for _ in range(3))
        self._struct = ScalingStateStruct(mode, history_len, _ptr(self.hist_x), _ptr(self.hist_w), _ptr(self.hist_dy),
                                          _ptr(self.scale_x), _ptr(self.scale_w), _ptr(self.scale_dy))

    def struct(self):
        return self._struct


class ReplayState:
    """f8_scaling_state in STATIC mode whose scales are the ones a Saved already holds, i.e. the
    scales its last forward (and backward) used.  Running a forward again with it reproduces that
    forward's codes bit for bit and records nothing in any amax history: what recomputation inside
    the backward (activation checkpointing) needs under delayed scaling."""

    def __init__(self, saved):
        self.mode, self.history_len, self.saved = STATIC, 1, saved
        self._struct = ScalingStateStruct(STATIC, 1, None, None, None, _ptr(saved.x.scale), _ptr(saved.w.scale),
                                          _ptr(saved.dy.scale))

    def struct(self):
        return self._struct


def linear_fwd_scaled(desc, state, X, W, Y, saved, workspace, stream=None):
    wp, wb = _ws(workspace)
    _check(lib().f8_linear_fwd_scaled(C.byref(desc), C.byref(state.struct()), _ptr(X), _ptr(W), _ptr(Y),
                                      C.byref(saved.struct()), wp, wb, _stream(stream)))


def linear_bwd_scaled(desc, state, dY, saved, dX, dW, workspace, stream=None):
    wp, wb = _ws(workspace)
    _check(lib().f8_linear_bwd_scaled(C.byref(desc), C.byref(state.struct()), _ptr(dY), C.byref(saved.struct()),
                                      _ptr(dX), _ptr(dW), wp, wb, _stream(stream)))


# ---- chained linears: amax handed from the producing GEMM to the consumer ----------

def linear_fwd_chained(desc, X, x_amax, W, Y, y_amax, saved, workspace, stream=None):
    wp, wb = _ws(workspace)
    _check(lib().f8_linear_fwd_chained(C.byref(desc), _ptr(X), _ptr(x_amax), _ptr(W), _ptr(Y), _ptr(y_amax),
                                       C.byref(saved.struct()), wp, wb, _stream(stream)))


def linear_bwd_chained(desc, dY, dy_amax, saved, dX, dx_amax, dW, workspace, stream=None):
    wp, wb = _ws(workspace)
    _check(lib().f8_linear_bwd_chained(C.byref(desc), _ptr(dY), _ptr(dy_amax), C.byref(saved.struct()), _ptr(dX),
                                       _ptr(dx_amax), _ptr(dW), wp, wb, _stream(stream)))


# ---- feed-forward glue ---------------------------------------------------------------

def silu_mul(ab, h, amax_h=None, workspace=None, stream=None):
    M, H2 = ab.shape
    wp, wb = _ws(workspace)
    _check(lib().f8_silu_mul(_ptr(ab), M, H2 // 2, _ptr(h), _ptr(amax_h), wp, wb, _stream(stream)))


def silu_mul_bwd(ab, dh, dab, amax_dab=None, workspace=None, stream=None):
    M, H2 = ab.shape
    wp, wb = _ws(workspace)
    _check(lib().f8_silu_mul_bwd(_ptr(ab), _ptr(dh), M, H2 // 2, _ptr(dab), _ptr(amax_dab), wp, wb, _stream(stream)))


def rmsnorm(x, g, eps, y, rstd=None, amax_y=None, workspace=None, stream=None):
    M, D = x.shape
    wp, wb = _ws(workspace)
    _check(lib().f8_rmsnorm(_ptr(x), _ptr(g), M, D, float(eps), _ptr(y), _ptr(rstd), _ptr(amax_y), wp, wb,
                            _stream(stream)))


def silu_mul_quantise_delayed(ab, fmt, history, scale_t, q, workspace, stream=None):
    M, H2 = ab.shape
    wp, wb = _ws(workspace)
    st = q.struct()
    _check(lib().f8_silu_mul_quantise_delayed(_ptr(ab), M, H2 // 2, fmt, _ptr(history), history.numel(), _ptr(scale_t),
                                              C.byref(st), wp, wb, _stream(stream)))


def linear_fwd_xq(desc, state, W, Y, saved, workspace, stream=None):
    wp, wb = _ws(workspace)
    _check(lib().f8_linear_fwd_xq(C.byref(desc), C.byref(state.struct()), _ptr(W), _ptr(Y), C.byref(saved.struct()),
                                  wp, wb, _stream(stream)))


def silu_mul_bwd_quantise_delayed(ab, dh, fmt, history, scale_t, q, workspace, stream=None):
    M, H2 = ab.shape
    wp, wb = _ws(workspace)
    st = q.struct()
    _check(lib().f8_silu_mul_bwd_quantise_delayed(_ptr(ab), _ptr(dh), M, H2 // 2, fmt, _ptr(history), history.numel(),
                                                  _ptr(scale_t), C.byref(st), wp, wb, _stream(stream)))


def linear_bwd_dyq(desc, saved, dX, dW, stream=None):
    _check(lib().f8_linear_bwd_dyq(C.byref(desc), C.byref(saved.struct()), _ptr(dX), _ptr(dW), _stream(stream)))


# ---- the bf16 operations between the Float8 linears of a transformer block -----------

def rope(x, S, n_heads, hd, out=None, out_t=None, theta=500000.0, inverse=False, stream=None, amax_inout=None):
    """x, out: 2-D (possibly column slices of wider tensors: the row pitch is taken from stride(0))."""
    M = x.shape[0]
    _check(lib().f8_rope(_ptr(x), x.stride(0), M, S, n_heads, hd, float(theta), int(bool(inverse)), _ptr(out),
                         out.stride(0) if out is not None else 0, _ptr(out_t), _ptr(amax_inout), _stream(stream)))


def transpose_bf16(x, out_t, stream=None):
    _check(lib().f8_transpose_bf16(_ptr(x), x.stride(0), x.shape[0], x.shape[1], _ptr(out_t), _stream(stream)))


def add(a, b, out, stream=None):
    _check(lib().f8_add(_ptr(a), _ptr(b), a.numel(), _ptr(out), _stream(stream)))


def rmsnorm_bwd(x, g, rstd, dy, dx, dg, workspace=None, stream=None):
    M, D = x.shape
    wp, wb = _ws(workspace)
    _check(lib().f8_rmsnorm_bwd(_ptr(x), _ptr(g), _ptr(rstd), _ptr(dy), M, D, _ptr(dx), _ptr(dg), wp, wb, _stream(stream)))


def rmsnorm_bwd_add(x, g, rstd, dy, add_t, dx, dg, workspace=None, stream=None, amax_dx_inout=None):
    M, D = x.shape
    wp, wb = _ws(workspace)
    _check(lib().f8_rmsnorm_bwd_add(_ptr(x), _ptr(g), _ptr(rstd), _ptr(dy), _ptr(add_t), M, D, _ptr(dx), _ptr(dg),
                                    _ptr(amax_dx_inout), wp, wb, _stream(stream)))


def sdpa_fwd(q, k, vt, B, S, Hq, Hkv, hd, o, lse, stream=None, amax_o=None):
    _check(lib().f8_sdpa_fwd(_ptr(q), q.stride(0), _ptr(k), k.stride(0), _ptr(vt), B, S, Hq, Hkv, hd, _ptr(o), o.stride(0),
                             _ptr(lse), _ptr(amax_o), _stream(stream)))


def sdpa_bwd_workspace_bytes(B, S, Hq, Hkv, hd):
    return int(lib().f8_sdpa_bwd_workspace_bytes(B, S, Hq, Hkv, hd))


def sdpa_bwd(q, qt, k, kt, v, o, do, dot, lse, B, S, Hq, Hkv, hd, dq, dk, dv, delta, workspace=None, stream=None,
             amax_dv_inout=None):
    wp, wb = _ws(workspace)
    _check(lib().f8_sdpa_bwd(_ptr(q), q.stride(0), _ptr(qt), _ptr(k), k.stride(0), _ptr(kt), _ptr(v), v.stride(0),
                             _ptr(o), o.stride(0), _ptr(do), do.stride(0), _ptr(dot), _ptr(lse), B, S, Hq, Hkv, hd,
                             _ptr(dq), dq.stride(0), _ptr(dk), dk.stride(0), _ptr(dv), dv.stride(0), _ptr(delta),
                             _ptr(amax_dv_inout), wp, wb, _stream(stream)))


# ---- measuring helpers ---------------------------------------------------------------

def probe_mfma(operands, iters, ticks=None, sink=None, stream=None, shape=0):
    """Launches the matrix-pipe-only loop (shape 0: 16x16x128 as the GEMM kernel, 1: 32x32x64);
    returns the floating-point operations of the launch."""
    if sink is None:
        sink = torch.zeros(1, dtype=torch.float32, device=operands.device)
    fl = _i64(0)
    _check(lib().f8_probe_mfma(int(shape), _ptr(operands), operands.numel() * operands.element_size(), int(iters), _ptr(ticks),
                               _ptr(sink), C.byref(fl), _stream(stream)))
    return fl.value


def probe_copy(src, dst, stream=None):
    _check(lib().f8_probe_copy(_ptr(src), _ptr(dst), src.numel() * src.element_size(), _stream(stream)))


def probe_read(src, sink, stream=None):
    _check(lib().f8_probe_read(_ptr(src), src.numel() * src.element_size(), _ptr(sink), _stream(stream)))


PROBE_CLOCK_SLOTS = 2048


def probe_clock(out, stream=None):
    """out: 4 * PROBE_CLOCK_SLOTS int64 on the device, zeroed: per compute unit u, out[4u] = 1,
    out[4u+1] = shader-clock cycles, out[4u+2] = 100 MHz ticks."""
    _check(lib().f8_probe_clock(_ptr(out), _stream(stream)))


def clock_ghz_between(before, after):
    """Mean shader clock between two probe_clock samples (CPU int64 tensors of 4 * PROBE_CLOCK_SLOTS),
    the median over the compute units that filled their slot in both; None if none did."""
    b, a = before.view(-1, 4), after.view(-1, 4)
    ok = (b[:, 0] == 1) & (a[:, 0] == 1) & (a[:, 2] > b[:, 2])
    if not bool(ok.any()):
        return None
    ghz = 0.1 * (a[ok, 1] - b[ok, 1]).double() / (a[ok, 2] - b[ok, 2]).double()
    return float(ghz.median())
