"""A CPU model of WHERE the attention backward rounds to bf16, for deriving the tolerance of its
parity tests: the definition of the backward in fp64 with exactly the kernel's three roundings put
in - the forward's output O (inside delta = sum_d O dO), the probabilities P as the operand of
dV = P^T dO, and dS = P (dP - delta) as the operand of dQ = dS K and dK = dS^T Q - and the bf16
rounding of the results.  Everything else (scores, softmax, the sums) stays in fp64, so the model's
distance from the unrounded definition is the error that these roundings alone cause.  It shares no
code with the library or with the oracle."""
import numpy as np


def round_bf16(x):
    """fp64 -> nearest bf16 (ties to even) -> fp64, through fp32 (two roundings; the second one is the
    only one that matters at the magnitudes used here)."""
    u = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) >> 16 << 16
    return u.astype(np.uint32).view(np.float32).astype(np.float64)


def _split(x, B, S, nh, hd):
    return x.reshape(B, S, nh, hd).transpose(0, 2, 1, 3)


def _merge(x):
    B, nh, S, hd = x.shape
    return x.transpose(0, 2, 1, 3).reshape(B * S, nh * hd)


def sdpa_bwd_with_bf16_roundings(q, k, v, do, B, S, Hq, Hkv, hd, rounded=True):
    """q, k, v, do: fp64 arrays [B*S, heads*hd] holding bf16 values.  Returns dq, dk, dv as fp64
    (bf16 values if `rounded`, else the plain fp64 definition)."""
    r = round_bf16 if rounded else (lambda t: t)
    g = Hq // Hkv
    qh, doh = _split(q, B, S, Hq, hd), _split(do, B, S, Hq, hd)
    kh = np.repeat(_split(k, B, S, Hkv, hd), g, axis=1)
    vh = np.repeat(_split(v, B, S, Hkv, hd), g, axis=1)
    sc = 1.0 / np.sqrt(float(hd))
    s = np.matmul(qh, np.swapaxes(kh, 2, 3)) * sc
    s = np.where(np.tril(np.ones((S, S), dtype=bool)), s, -np.inf)
    e = np.exp(s - s.max(axis=-1, keepdims=True))
    P = e / e.sum(axis=-1, keepdims=True)
    O = r(np.matmul(P, vh))                                   # the forward's stored output
    delta = (O * doh).sum(axis=-1, keepdims=True)
    dv = np.matmul(np.swapaxes(r(P), 2, 3), doh)
    dS = r(P * (np.matmul(doh, np.swapaxes(vh, 2, 3)) - delta))
    dq = np.matmul(dS, kh) * sc
    dk = np.matmul(np.swapaxes(dS, 2, 3), qh) * sc
    dk = dk.reshape(B, Hkv, g, S, hd).sum(axis=2)
    dv = dv.reshape(B, Hkv, g, S, hd).sum(axis=2)
    return r(_merge(dq)), r(_merge(dk)), r(_merge(dv))


def mean_relative_errors(q, k, v, do, B, S, Hq, Hkv, hd):
    """(dq, dk, dv): mean |model - definition| / mean |definition| of each gradient."""
    a = sdpa_bwd_with_bf16_roundings(q, k, v, do, B, S, Hq, Hkv, hd, True)
    b = sdpa_bwd_with_bf16_roundings(q, k, v, do, B, S, Hq, Hkv, hd, False)
    return tuple(float(np.abs(x - y).mean() / np.abs(y).mean()) for x, y in zip(a, b))
