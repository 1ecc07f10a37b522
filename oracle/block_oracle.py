"""CPU oracle for the bf16 operations that join the Float8 linears of one transformer block
(Section 2.2.4 of the paper applies Float8 to the linear layers only; everything between them
stays in bf16): rotary position embedding, causal grouped-query attention, the backward of
RMSNorm and the residual addition.

Test infrastructure only: plain numpy in fp64 on the values of the bf16 inputs, rounded at the end
to fp32 and from there to bf16 (two roundings to nearest even), no blocking, no online softmax, no
fusion.  The product never imports this.

Each function is the textbook definition written out:
  rope          (x0, x1) -> (x0 cos t - x1 sin t, x0 sin t + x1 cos t), t = pos * theta^(-2i/hd)
                for the i-th adjacent pair of a head (the interleaved-pair form of Llama, which
                is what the paper's Llama 3.1 models use)
  sdpa          O = softmax(Q K^T / sqrt(hd) + causal mask) V per head, query head h reading
                key/value head h // (Hq / Hkv); lse = log sum exp of the masked scores
  sdpa_bwd      the derivative of that definition
  rmsnorm_bwd   the derivative of y = x * rsqrt(mean(x^2) + eps) * g
  add           bf16(a + b)
Pinned in tests/test_block_oracle_pins.py against closed forms, invariants, PyTorch's own CPU
attention and complex multiplication, PyTorch autograd and finite differences.
The paper prints none of these formulas (it names the Llama 3.1 models, Section 3); what the pins
cannot fix are the choices of that architecture itself, taken here as readings: adjacent-pair
(interleaved) rotation with theta = 500000, positions counted per sequence, 1 / sqrt(hd) scaling
with a causal mask, query head h reading key/value head h // (Hq / Hkv), eps inside the root.
"""
import numpy as np


def _f64(bits):
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def _bf16(x):
    """fp64 -> fp32 -> bf16 bits, round to nearest even (no NaN / Inf in these tests)."""
    f = np.ascontiguousarray(x, dtype=np.float64).astype(np.float32)
    u = f.view(np.uint32)
    r = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + r) >> 16).astype(np.uint16)


# ---- rotary position embedding --------------------------------------------------------

def rope_f64(x, S, hd, theta=500000.0, inverse=False):
    """x: [M, nh * hd] fp64, row m is position m % S of its sequence."""
    M, W = x.shape
    assert W % hd == 0 and hd % 2 == 0
    pos = (np.arange(M) % S).astype(np.float64)
    i = np.arange(hd // 2, dtype=np.float64)
    ang = pos[:, None] * theta ** (-2.0 * i / hd)[None, :]            # [M, hd/2]
    if inverse:
        ang = -ang
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    xr = x.reshape(M, W // hd, hd // 2, 2)
    out = np.empty_like(xr)
    out[..., 0] = xr[..., 0] * c - xr[..., 1] * s
    out[..., 1] = xr[..., 0] * s + xr[..., 1] * c
    return out.reshape(M, W)


def rope(x_bits, S, hd, theta=500000.0, inverse=False):
    return _bf16(rope_f64(_f64(x_bits), S, hd, theta, inverse))


# ---- causal grouped-query attention -----------------------------------------------------

def _heads(x, B, S, nh, hd):
    return x.reshape(B, S, nh, hd).transpose(0, 2, 1, 3)              # [B, nh, S, hd]


def _unheads(x):
    B, nh, S, hd = x.shape
    return x.transpose(0, 2, 1, 3).reshape(B * S, nh * hd)


def _probabilities(q, k, hd):
    """q [B, Hq, S, hd], k [B, Hq, S, hd] (already repeated) -> P [B, Hq, S, S], lse [B, Hq, S]."""
    S = q.shape[2]
    s = np.matmul(q, np.swapaxes(k, 2, 3)) / np.sqrt(float(hd))
    mask = np.tril(np.ones((S, S), dtype=bool))
    s = np.where(mask, s, -np.inf)
    m = s.max(axis=-1, keepdims=True)
    e = np.exp(s - m)
    z = e.sum(axis=-1, keepdims=True)
    return e / z, (m + np.log(z))[..., 0]


def sdpa_f64(q, k, v, B, S, Hq, Hkv, hd):
    g = Hq // Hkv
    qh = _heads(q, B, S, Hq, hd)
    kh = np.repeat(_heads(k, B, S, Hkv, hd), g, axis=1)
    vh = np.repeat(_heads(v, B, S, Hkv, hd), g, axis=1)
    P, lse = _probabilities(qh, kh, hd)
    return _unheads(np.matmul(P, vh)), lse


def sdpa(q_bits, k_bits, v_bits, B, S, Hq, Hkv, hd):
    """-> (O [B*S, Hq*hd] bf16 bits, lse [B, Hq, S] fp32)."""
    o, lse = sdpa_f64(_f64(q_bits), _f64(k_bits), _f64(v_bits), B, S, Hq, Hkv, hd)
    return _bf16(o), lse.astype(np.float32)


def sdpa_bwd_f64(q, k, v, do, B, S, Hq, Hkv, hd):
    g = Hq // Hkv
    qh, doh = _heads(q, B, S, Hq, hd), _heads(do, B, S, Hq, hd)
    kh = np.repeat(_heads(k, B, S, Hkv, hd), g, axis=1)
    vh = np.repeat(_heads(v, B, S, Hkv, hd), g, axis=1)
    P, _ = _probabilities(qh, kh, hd)
    dv = np.matmul(np.swapaxes(P, 2, 3), doh)
    dP = np.matmul(doh, np.swapaxes(vh, 2, 3))
    dS = P * (dP - (P * dP).sum(axis=-1, keepdims=True))
    sc = 1.0 / np.sqrt(float(hd))
    dq = np.matmul(dS, kh) * sc
    dk = np.matmul(np.swapaxes(dS, 2, 3), qh) * sc
    # the query heads of one group share a key/value head: their gradients add
    dk = dk.reshape(B, Hkv, g, S, hd).sum(axis=2)
    dv = dv.reshape(B, Hkv, g, S, hd).sum(axis=2)
    return _unheads(dq), _unheads(dk), _unheads(dv)


def sdpa_bwd(q_bits, k_bits, v_bits, do_bits, B, S, Hq, Hkv, hd):
    dq, dk, dv = sdpa_bwd_f64(_f64(q_bits), _f64(k_bits), _f64(v_bits), _f64(do_bits), B, S, Hq, Hkv, hd)
    return _bf16(dq), _bf16(dk), _bf16(dv)


def _rows_probabilities(q, k, v, rows, S, Hq, Hkv, hd):
    """The definition restricted to the query tokens `rows` (global token indices): P [Hq, R, B*S]
    over ALL tokens (zero outside the row's own sequence and after its position), lse [Hq, R]."""
    g = Hq // Hkv
    rows = np.asarray(rows)
    M = k.shape[0]
    tok = np.arange(M)
    visible = (tok[None, :] // S == rows[:, None] // S) & (tok[None, :] <= rows[:, None])      # [R, M]
    P = np.empty((Hq, len(rows), M))
    lse = np.empty((Hq, len(rows)))
    for h in range(Hq):
        kh = k[:, (h // g) * hd:(h // g + 1) * hd]
        s = np.where(visible, q[rows, h * hd:(h + 1) * hd] @ kh.T / np.sqrt(float(hd)), -np.inf)
        m = s.max(axis=1, keepdims=True)
        e = np.exp(s - m)
        z = e.sum(axis=1, keepdims=True)
        P[h], lse[h] = e / z, (m + np.log(z))[:, 0]
    return P, lse


def sdpa_rows_f64(q, k, v, rows, B, S, Hq, Hkv, hd):
    """O[rows] [R, Hq*hd] and lse [Hq, R] of the attention for the query tokens `rows` only (for
    sizes at which the full S x S probabilities are too slow to form)."""
    g = Hq // Hkv
    P, lse = _rows_probabilities(q, k, v, rows, S, Hq, Hkv, hd)
    o = np.concatenate([P[h] @ v[:, (h // g) * hd:(h // g + 1) * hd] for h in range(Hq)], axis=1)
    return o, lse


def sdpa_bwd_rows_f64(q, k, v, do, rows, B, S, Hq, Hkv, hd):
    """dq[rows] [R, Hq*hd], and the contribution of the query tokens `rows` to dk and dv
    [B*S, Hkv*hd]: complete for every key that no other query can see (with rows = all tokens
    from t on of the last sequence, complete for the keys from t on)."""
    g = Hq // Hkv
    rows = np.asarray(rows)
    P, _ = _rows_probabilities(q, k, v, rows, S, Hq, Hkv, hd)
    sc = 1.0 / np.sqrt(float(hd))
    dq = np.empty((len(rows), Hq * hd))
    dk, dv = np.zeros_like(k), np.zeros_like(v)
    for h in range(Hq):
        hs, ks = slice(h * hd, (h + 1) * hd), slice((h // g) * hd, (h // g + 1) * hd)
        doh = do[rows, hs]
        dP = doh @ v[:, ks].T
        dS = P[h] * (dP - (P[h] * dP).sum(axis=1, keepdims=True))
        dq[:, hs] = dS @ k[:, ks] * sc
        dk[:, ks] += dS.T @ q[rows, hs] * sc
        dv[:, ks] += P[h].T @ doh
    return dq, dk, dv


# ---- RMSNorm backward, residual ----------------------------------------------------------

def rmsnorm_bwd_f64(x, g, dy, eps=1e-5):
    D = x.shape[1]
    r = 1.0 / np.sqrt((x * x).mean(axis=1, keepdims=True) + eps)
    gdy = g[None, :] * dy
    dx = r * gdy - x * (r ** 3) * (x * gdy).sum(axis=1, keepdims=True) / D
    dg = (dy * x * r).sum(axis=0)
    return dx, dg


def rmsnorm_bwd(x_bits, g_bits, dy_bits, eps=1e-5):
    """-> (dx [M, D] bf16 bits, dg [D] fp32)."""
    dx, dg = rmsnorm_bwd_f64(_f64(x_bits), _f64(g_bits), _f64(dy_bits), eps)
    return _bf16(dx), dg.astype(np.float32)


def add(a_bits, b_bits):
    return _bf16(_f64(a_bits) + _f64(b_bits))


def transpose(x_bits):
    return np.ascontiguousarray(np.asarray(x_bits, dtype=np.uint16).T)
