"""Pins of oracle/block_oracle.py (rotary embedding, causal grouped-query attention, RMSNorm
backward) against things other than itself: closed forms, invariants, PyTorch's own CPU complex
multiplication / attention / autograd, and finite differences."""
import numpy as np
import pytest
import torch

from oracle import block_oracle as bo


def rnd(shape, seed, scale=1.0):
    return np.random.default_rng(seed).standard_normal(shape) * scale


# ---- rope -----------------------------------------------------------------------------------

def test_rope_hand_values():
    # hd = 4, theta = 100: pair 0 turns by pos radians, pair 1 by pos / 10 radians
    x = np.array([[1.0, 0.0, 0.0, 2.0]] * 3)
    y = bo.rope_f64(x, S=3, hd=4, theta=100.0)
    assert np.allclose(y[0], x[0], atol=0)                                   # position 0: identity
    assert np.allclose(y[1], [np.cos(1.0), np.sin(1.0), -2 * np.sin(0.1), 2 * np.cos(0.1)], atol=1e-15)
    assert np.allclose(y[2], [np.cos(2.0), np.sin(2.0), -2 * np.sin(0.2), 2 * np.cos(0.2)], atol=1e-15)


def test_rope_positions_restart_per_sequence_and_inverse():
    x = rnd((12, 2 * 8), 1)
    y = bo.rope_f64(x, S=4, hd=8)
    assert np.array_equal(y[0], x[0]) and np.array_equal(y[4], x[4]) and np.array_equal(y[8], x[8])
    # rows with the same position in different sequences turn by the same angle
    x2 = np.tile(x[:4], (3, 1))
    y2 = bo.rope_f64(x2, S=4, hd=8)
    assert np.array_equal(y2[:4], y2[4:8]) and np.array_equal(y2[:4], y2[8:])
    assert np.allclose(bo.rope_f64(y, S=4, hd=8, inverse=True), x, atol=1e-14)


def test_rope_keeps_pair_norms_and_depends_on_relative_position_only():
    hd = 16
    q, k = rnd((1, hd), 2), rnd((1, hd), 3)
    S = 64
    Q = bo.rope_f64(np.tile(q, (S, 1)), S, hd)
    K = bo.rope_f64(np.tile(k, (S, 1)), S, hd)
    pairs = lambda a: (a.reshape(-1, hd // 2, 2) ** 2).sum(-1)
    assert np.allclose(pairs(Q), pairs(np.tile(q, (S, 1))), rtol=1e-13)
    dots = Q @ K.T                                                           # [m, n]
    for d in (0, 1, 7):
        diag = np.array([dots[m + d, m] for m in range(S - d)])
        assert np.allclose(diag, diag[0], rtol=1e-10, atol=1e-12)
    assert abs(dots[9, 2] - dots[2, 9]) > 1e-3                               # and the sign of m - n matters


def test_rope_equals_torch_complex_multiplication():
    M, nh, hd, S, theta = 24, 3, 32, 8, 500000.0
    x = rnd((M, nh * hd), 4)
    freqs = 1.0 / (theta ** (torch.arange(0, hd, 2, dtype=torch.float64) / hd))
    ang = torch.outer((torch.arange(M) % S).double(), freqs)
    cis = torch.polar(torch.ones_like(ang), ang)                             # [M, hd/2]
    xc = torch.view_as_complex(torch.from_numpy(x).reshape(M, nh, hd // 2, 2))
    ref = torch.view_as_real(xc * cis[:, None, :]).reshape(M, nh * hd).numpy()
    assert np.allclose(bo.rope_f64(x, S, hd, theta), ref, rtol=1e-13, atol=1e-13)


def test_rope_bits_round_once():
    x = rnd((8, 16), 5)
    xb = bo._bf16(x)
    y = bo.rope(xb, 8, 16)
    assert np.array_equal(y, bo._bf16(bo.rope_f64(bo._f64(xb), 8, 16)))
    assert np.array_equal(y[0], xb[0])


# ---- attention ------------------------------------------------------------------------------

def torch_sdpa(q, k, v, B, S, Hq, Hkv, hd):
    t = lambda a, nh: torch.from_numpy(a).reshape(B, S, nh, hd).transpose(1, 2)
    g = Hq // Hkv
    qh, kh, vh = t(q, Hq), t(k, Hkv).repeat_interleave(g, dim=1), t(v, Hkv).repeat_interleave(g, dim=1)
    o = torch.nn.functional.scaled_dot_product_attention(qh, kh, vh, is_causal=True)
    return o.transpose(1, 2).reshape(B * S, Hq * hd).numpy()


@pytest.mark.parametrize("B,S,Hq,Hkv,hd", [(1, 16, 2, 2, 8), (2, 33, 4, 2, 16), (1, 64, 8, 2, 32)])
def test_sdpa_equals_torch_cpu_attention(B, S, Hq, Hkv, hd):
    q, k, v = rnd((B * S, Hq * hd), 6), rnd((B * S, Hkv * hd), 7), rnd((B * S, Hkv * hd), 8)
    o, lse = bo.sdpa_f64(q, k, v, B, S, Hq, Hkv, hd)
    assert np.allclose(o, torch_sdpa(q, k, v, B, S, Hq, Hkv, hd), rtol=1e-12, atol=1e-12)
    # lse: brute force for a few (b, h, position) triples
    g = Hq // Hkv
    for b, h, p in [(0, 0, 0), (B - 1, Hq - 1, S - 1), (0, 1, S // 2)]:
        qv = q[b * S + p, h * hd:(h + 1) * hd]
        sc = [qv @ k[b * S + j, (h // g) * hd:(h // g + 1) * hd] / np.sqrt(hd) for j in range(p + 1)]
        assert np.isclose(lse[b, h, p], np.log(np.sum(np.exp(sc))), rtol=1e-12)


def test_sdpa_invariants():
    B, S, Hq, Hkv, hd = 2, 12, 4, 2, 8
    q, k, v = rnd((B * S, Hq * hd), 9), rnd((B * S, Hkv * hd), 10), rnd((B * S, Hkv * hd), 11)
    o, _ = bo.sdpa_f64(q, k, v, B, S, Hq, Hkv, hd)
    # first token of every sequence attends to itself only: O = V of its key/value head
    for b in range(B):
        for h in range(Hq):
            assert np.allclose(o[b * S, h * hd:(h + 1) * hd], v[b * S, (h // 2) * hd:(h // 2 + 1) * hd], atol=1e-14)
    # causal: changing the last tokens leaves the earlier outputs alone; sequences do not mix
    k2, v2 = k.copy(), v.copy()
    k2[S - 3:S] += 5.0
    v2[S - 3:S] -= 3.0
    o2, _ = bo.sdpa_f64(q, k2, v2, B, S, Hq, Hkv, hd)
    assert np.array_equal(o2[:S - 3], o[:S - 3]) and np.array_equal(o2[S:], o[S:])
    assert not np.allclose(o2[S - 3:S], o[S - 3:S])
    # probabilities sum to one: constant values come back unchanged
    oc, _ = bo.sdpa_f64(q, k, np.full_like(v, 0.75), B, S, Hq, Hkv, hd)
    assert np.allclose(oc, 0.75, atol=1e-14)


def test_sdpa_bwd_equals_torch_autograd_and_finite_differences():
    B, S, Hq, Hkv, hd = 2, 9, 4, 2, 8
    q, k, v = rnd((B * S, Hq * hd), 12), rnd((B * S, Hkv * hd), 13), rnd((B * S, Hkv * hd), 14)
    do = rnd((B * S, Hq * hd), 15)
    dq, dk, dv = bo.sdpa_bwd_f64(q, k, v, do, B, S, Hq, Hkv, hd)
    tq, tk, tv = (torch.from_numpy(a).requires_grad_() for a in (q, k, v))
    t = lambda a, nh: a.reshape(B, S, nh, hd).transpose(1, 2)
    o = torch.nn.functional.scaled_dot_product_attention(
        t(tq, Hq), t(tk, Hkv).repeat_interleave(2, dim=1), t(tv, Hkv).repeat_interleave(2, dim=1), is_causal=True)
    o.transpose(1, 2).reshape(B * S, Hq * hd).backward(torch.from_numpy(do))
    assert np.allclose(dq, tq.grad.numpy(), rtol=1e-10, atol=1e-12)
    assert np.allclose(dk, tk.grad.numpy(), rtol=1e-10, atol=1e-12)
    assert np.allclose(dv, tv.grad.numpy(), rtol=1e-10, atol=1e-12)
    # central differences of the oracle's own forward, a few coordinates of each input
    f = lambda q_, k_, v_: (bo.sdpa_f64(q_, k_, v_, B, S, Hq, Hkv, hd)[0] * do).sum()
    h = 1e-6
    for arr, grad, idx in ((q, dq, (5, 3)), (k, dk, (2, 9)), (v, dv, (11, 4)), (k, dk, (S + 1, 0))):
        p, m = arr.copy(), arr.copy()
        p[idx] += h
        m[idx] -= h
        args_p = [p if a is arr else a for a in (q, k, v)]
        args_m = [m if a is arr else a for a in (q, k, v)]
        assert np.isclose((f(*args_p) - f(*args_m)) / (2 * h), grad[idx], rtol=1e-6, atol=1e-9)


def test_row_restricted_attention_equals_the_full_definition():
    """sdpa_rows_f64 / sdpa_bwd_rows_f64 (used at sizes where S x S is too slow) against the full
    oracle: sampled rows anywhere, and the key gradients of the last tokens from the last rows."""
    B, S, Hq, Hkv, hd = 2, 24, 4, 2, 8
    M = B * S
    q, k, v = rnd((M, Hq * hd), 30), rnd((M, Hkv * hd), 31), rnd((M, Hkv * hd), 32)
    do = rnd((M, Hq * hd), 33)
    o, lse = bo.sdpa_f64(q, k, v, B, S, Hq, Hkv, hd)
    dq, dk, dv = bo.sdpa_bwd_f64(q, k, v, do, B, S, Hq, Hkv, hd)
    rows = [0, 3, 23, 24, 30, 47]
    o_r, lse_r = bo.sdpa_rows_f64(q, k, v, rows, B, S, Hq, Hkv, hd)
    assert np.allclose(o_r, o[rows], rtol=1e-12, atol=1e-13)
    full_lse = lse.transpose(1, 0, 2).reshape(Hq, M)
    assert np.allclose(lse_r, full_lse[:, rows], rtol=1e-12)
    dq_r, _, _ = bo.sdpa_bwd_rows_f64(q, k, v, do, rows, B, S, Hq, Hkv, hd)
    assert np.allclose(dq_r, dq[rows], rtol=1e-10, atol=1e-13)
    t = M - 7                                             # the last 7 tokens of the last sequence
    tail = list(range(t, M))
    _, dk_t, dv_t = bo.sdpa_bwd_rows_f64(q, k, v, do, tail, B, S, Hq, Hkv, hd)
    assert np.allclose(dk_t[t:], dk[t:], rtol=1e-10, atol=1e-13) and np.allclose(dv_t[t:], dv[t:], rtol=1e-10, atol=1e-13)
    assert not np.allclose(dk_t[t - 3:t], dk[t - 3:t])    # earlier keys are seen by other queries too


# ---- rmsnorm backward, residual -----------------------------------------------------------

def test_rmsnorm_bwd_equals_torch_autograd_and_closed_form():
    M, D, eps = 7, 24, 1e-5
    x, g, dy = rnd((M, D), 16), rnd((D,), 17), rnd((M, D), 18)
    dx, dg = bo.rmsnorm_bwd_f64(x, g, dy, eps)
    tx, tg = torch.from_numpy(x).requires_grad_(), torch.from_numpy(g).requires_grad_()
    y = tx * torch.rsqrt(tx.pow(2).mean(-1, keepdim=True) + eps) * tg
    y.backward(torch.from_numpy(dy))
    assert np.allclose(dx, tx.grad.numpy(), rtol=1e-12, atol=1e-13)
    assert np.allclose(dg, tg.grad.numpy(), rtol=1e-12, atol=1e-13)
    # closed form: with eps = 0 the output does not change when x is scaled, so dx is orthogonal to x
    dx0, _ = bo.rmsnorm_bwd_f64(x, g, dy, 0.0)
    assert np.allclose((dx0 * x).sum(axis=1), 0.0, atol=1e-12)
    # one row, D = 1, eps = 0: y = sign(x) g, dx = 0, dg = dy sign(x)
    dx1, dg1 = bo.rmsnorm_bwd_f64(np.array([[-3.0]]), np.array([2.0]), np.array([[5.0]]), 0.0)
    assert abs(dx1[0, 0]) < 1e-15 and dg1[0] == -5.0


def test_add_and_transpose_bits():
    a, b = bo._bf16(rnd((4, 6), 19)), bo._bf16(rnd((4, 6), 20))
    s = bo.add(a, b)
    ref = (torch.from_numpy(bo._f64(a)).float() + torch.from_numpy(bo._f64(b)).float()).bfloat16()
    assert np.array_equal(s, ref.view(torch.int16).numpy().view(np.uint16))
    assert np.array_equal(bo.transpose(a), a.T)


def test_bf16_rounding_helper_matches_torch():
    x = rnd((1000,), 21, 3.0)
    x[:4] = [1.00390625, 1.01171875, -0.0, 3.0e-39]     # ties to even both ways, signed zero, subnormal
    ref = torch.from_numpy(x).float().bfloat16().view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bo._bf16(x), ref)
    assert np.array_equal(bo._f64(ref), torch.from_numpy(x).float().bfloat16().double().numpy())
