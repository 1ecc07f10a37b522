"""Causal grouped-query attention (forward and backward) through the C ABI against
oracle/block_oracle.py."""
import numpy as np
import pytest
import torch

import oracle as o
from oracle import block_oracle as bo
from paper_2410_06511_amd import f8
from paper_2410_06511_amd import workloads as wl
from attn_rounding_model import mean_relative_errors
from helpers import bits

pytestmark = pytest.mark.gpu
HD = 128


def gen(shape, seed, std=1.0):
    g = torch.Generator("cpu")
    g.manual_seed(seed)
    return wl.randn_bf16(shape, std, 0, generator=g)


def f64(t_bits):
    return o.bf16_to_f32(t_bits).astype(np.float64)


class Attn:
    """Device buffers and the call sequence: q, k, v are column slices of one [M, (Hq + 2 Hkv) hd]
    tensor, as they are slices of the fused q|k|v linear's output."""

    def __init__(self, B, S, Hq, Hkv, seed, std=1.0):
        self.B, self.S, self.Hq, self.Hkv = B, S, Hq, Hkv
        M = B * S
        self.qkv = gen((M, (Hq + 2 * Hkv) * HD), seed, std)
        d = self.qkv.cuda()
        self.q, self.k, self.v = d[:, :Hq * HD], d[:, Hq * HD:(Hq + Hkv) * HD], d[:, (Hq + Hkv) * HD:]
        bf = dict(dtype=torch.bfloat16, device="cuda")
        self.vt = torch.empty((Hkv * HD, M), **bf)
        self.o = torch.empty((M, Hq * HD), **bf)
        self.lse = torch.empty((Hq, M), device="cuda")
        self.amax = torch.full((1,), -1.0, device="cuda")

    def host_bits(self):
        b = bits(self.qkv)
        Hq, Hkv = self.Hq, self.Hkv
        return b[:, :Hq * HD], b[:, Hq * HD:(Hq + Hkv) * HD], b[:, (Hq + Hkv) * HD:]

    def forward(self):
        f8.transpose_bf16(self.v, self.vt)
        f8.sdpa_fwd(self.q, self.k, self.vt, self.B, self.S, self.Hq, self.Hkv, HD, self.o, self.lse, amax_o=self.amax)
        torch.cuda.synchronize()


def check_forward(a):
    qb, kb, vb = a.host_bits()
    B, S, Hq, Hkv = a.B, a.S, a.Hq, a.Hkv
    ref, lse = bo.sdpa_f64(f64(qb), f64(kb), f64(vb), B, S, Hq, Hkv, HD)
    # the probabilities are rounded to bf16 (2^-9 each, relative), so is the output: the error of
    # an output is bounded by 2^-8 of the probability-weighted mean of |v|; twice that is allowed
    weight, _ = bo.sdpa_f64(f64(qb), f64(kb), np.abs(f64(vb)), B, S, Hq, Hkv, HD)
    got = f64(bits(a.o))
    assert np.isfinite(got).all()
    err = np.abs(got - ref)
    assert (err <= 2.0 ** -7 * weight + 1e-30).all(), (err.max(), np.unravel_index(err.argmax(), err.shape))
    assert err.mean() <= 2.0 ** -10 * weight.mean()
    assert a.amax.item() == o.amax(bits(a.o))[0]          # exactly the maximum magnitude of what was written
    got_lse = a.lse.cpu().numpy().astype(np.float64).reshape(Hq, B, S).transpose(1, 0, 2)
    assert np.abs(got_lse - lse).max() <= 1e-4 * (1.0 + np.abs(lse).max())


@pytest.mark.parametrize("B,S,Hq,Hkv", [(1, 8, 1, 1), (1, 128, 2, 1), (2, 200, 4, 2), (1, 520, 8, 2), (3, 64, 2, 2)])
def test_sdpa_forward(B, S, Hq, Hkv):
    a = Attn(B, S, Hq, Hkv, seed=S + Hq)
    a.forward()
    check_forward(a)


def test_sdpa_forward_peaked_scores_and_first_token():
    """Large scores (a softmax close to one-hot, running maximum that keeps moving) and the first
    token of each sequence, which attends to itself only: its output is its value, bit for bit."""
    a = Attn(2, 264, 2, 1, seed=3, std=4.0)
    a.forward()
    check_forward(a)
    vb = a.host_bits()[2]
    got = bits(a.o)
    for b in range(2):
        for h in range(2):
            assert np.array_equal(got[b * 264, h * HD:(h + 1) * HD], vb[b * 264, :HD])


def run_backward(a, do_t):
    """do_t: [M, Hq * hd] bf16 on the host.  Returns device dq, dk, dv (slices of one [M, (Hq + 2 Hkv) hd]
    tensor, the layout of the fused q|k|v linear's output gradient)."""
    B, S, Hq, Hkv = a.B, a.S, a.Hq, a.Hkv
    M = B * S
    bf = dict(dtype=torch.bfloat16, device="cuda")
    do = do_t.cuda()
    qt, kt, dot = torch.empty((Hq * HD, M), **bf), torch.empty((Hkv * HD, M), **bf), torch.empty((Hq * HD, M), **bf)
    f8.transpose_bf16(a.q, qt)
    f8.transpose_bf16(a.k, kt)
    f8.transpose_bf16(do, dot)
    dqkv = torch.zeros((M, (Hq + 2 * Hkv) * HD), **bf)
    dq, dk, dv = dqkv[:, :Hq * HD], dqkv[:, Hq * HD:(Hq + Hkv) * HD], dqkv[:, (Hq + Hkv) * HD:]
    delta = torch.empty((Hq, M), device="cuda")
    ws = torch.empty(max(16, f8.sdpa_bwd_workspace_bytes(B, S, Hq, Hkv, HD)), dtype=torch.uint8, device="cuda")
    assert (ws.numel() > 16) == (Hq != Hkv)
    cell = torch.zeros(1, device="cuda") if Hq != Hkv else None
    f8.sdpa_bwd(a.q, qt, a.k, kt, a.v, a.o, do, dot, a.lse, B, S, Hq, Hkv, HD, dq, dk, dv, delta, ws, amax_dv_inout=cell)
    torch.cuda.synchronize()
    if cell is not None:   # exactly the maximum magnitude of the dv written
        assert cell.item() == o.amax(np.ascontiguousarray(bits(dqkv)[:, (Hq + Hkv) * HD:]))[0]
    return dqkv, delta


def check_backward(a, do_t, dqkv, delta):
    qb, kb, vb = a.host_bits()
    B, S, Hq, Hkv = a.B, a.S, a.Hq, a.Hkv
    q, k, v, do = f64(qb), f64(kb), f64(vb), f64(bits(do_t))
    rdq, rdk, rdv = bo.sdpa_bwd_f64(q, k, v, do, B, S, Hq, Hkv, HD)
    got = f64(bits(dqkv))
    gq, gk, gv = got[:, :Hq * HD], got[:, Hq * HD:(Hq + Hkv) * HD], got[:, (Hq + Hkv) * HD:]
    assert np.isfinite(got).all()
    # delta against its definition with the GPU's own (bf16) output O
    o_gpu = f64(bits(a.o))
    rdelta = (o_gpu * do).reshape(B, S, Hq, HD).sum(axis=3).transpose(2, 0, 1).reshape(Hq, B * S)
    mag = (np.abs(o_gpu) * np.abs(do)).reshape(B, S, Hq, HD).sum(axis=3).transpose(2, 0, 1).reshape(Hq, B * S)
    assert (np.abs(delta.cpu().numpy() - rdelta) <= 1e-5 * mag + 1e-30).all()
    # The kernel rounds P, dS, O (inside delta) and its results to bf16 and sums in fp32.  What these
    # roundings alone cost is computed, not assumed: the fp64 definition with the same roundings put
    # in (attn_rounding_model) against the definition without them.  The kernel's mean error may
    # exceed the model's by a tenth (its fp32 sums and its fast exponential are not in the model).
    model = mean_relative_errors(q, k, v, do, B, S, Hq, Hkv, HD)
    for name, g_, r_, m_ in (("dq", gq, rdq, model[0]), ("dk", gk, rdk, model[1]), ("dv", gv, rdv, model[2])):
        err = np.abs(g_ - r_)
        # the largest error: the same criterion as for the GEMMs of the linear, max |error| against max |reference|
        assert err.max() <= 1e-2 * np.abs(r_).max(), (name, err.max(), np.abs(r_).max())
        assert err.mean() <= (1.1 * m_ + 2.0 ** -13) * np.abs(r_).mean(), (name, err.mean() / np.abs(r_).mean(), m_)


@pytest.mark.parametrize("B,S,Hq,Hkv", [(1, 8, 1, 1), (1, 128, 2, 1), (2, 200, 4, 2), (1, 520, 8, 2), (3, 64, 2, 2)])
def test_sdpa_backward(B, S, Hq, Hkv):
    a = Attn(B, S, Hq, Hkv, seed=S + Hq + 1)
    a.forward()
    do_t = gen((B * S, Hq * HD), S, 1e-2)
    dqkv, delta = run_backward(a, do_t)
    check_backward(a, do_t, dqkv, delta)
    # reproducible: no atomics anywhere
    dqkv2, _ = run_backward(a, do_t)
    assert torch.equal(dqkv.view(torch.int16), dqkv2.view(torch.int16))


def test_sdpa_backward_peaked_scores():
    """Scores of order ten (a softmax close to one-hot, where P (dP - delta) cancels strongly)."""
    B, S, Hq, Hkv = 2, 264, 4, 2
    a = Attn(B, S, Hq, Hkv, seed=5, std=3.0)
    a.forward()
    do_t = gen((B * S, Hq * HD), 6, 1e-2)
    dqkv, delta = run_backward(a, do_t)
    # dS = P (dP - delta) cancels where P is close to one-hot (dP of the dominating key is nearly
    # delta itself): the bf16 rounding of O inside delta, 2^-9 of |delta|, is then a larger share of
    # the small difference, and the mean error of dq and dk is about three times that of unpeaked
    # scores - in the rounding model as on the GPU, which is what check_backward compares.
    check_backward(a, do_t, dqkv, delta)


def test_sdpa_full_size_sampled_against_oracle():
    """The 8B shape that bench.py times (1 x 8192 tokens, 32 query / 8 key-value heads), in the same
    launch configuration.  The 8192 x 8192 probabilities of 32 heads are too slow for the oracle,
    so it computes them for sampled query tokens (every head): the outputs, log-sum-exp and dq of
    those tokens, and dk, dv of the last 192 keys (which only the last 192 queries see)."""
    B, S, Hq, Hkv = 1, 8192, 32, 8
    a = Attn(B, S, Hq, Hkv, seed=99)
    a.forward()
    do_t = gen((B * S, Hq * HD), 98, 1e-2)
    dqkv, _ = run_backward(a, do_t)
    qb, kb, vb = a.host_bits()
    q, k, v, do = f64(qb), f64(kb), f64(vb), f64(bits(do_t))
    t = S - 192
    rows = sorted(set([0, 1, 31, 32, 63, 64, 127, 128, 129, 1000, 2047, 2048, 4095, 4100, 6143, 7000]) | set(range(t, S)))
    ref, lse = bo.sdpa_rows_f64(q, k, v, rows, B, S, Hq, Hkv, HD)
    weight, _ = bo.sdpa_rows_f64(q, k, np.abs(v), rows, B, S, Hq, Hkv, HD)
    got = f64(bits(a.o))[rows]
    assert (np.abs(got - ref) <= 2.0 ** -7 * weight + 1e-30).all()
    got_lse = a.lse.cpu().numpy().astype(np.float64)[:, rows]
    assert np.abs(got_lse - lse).max() <= 1e-4 * (1.0 + np.abs(lse).max())
    rdq, rdk, rdv = bo.sdpa_bwd_rows_f64(q, k, v, do, rows, B, S, Hq, Hkv, HD)
    g_ = f64(bits(dqkv))
    nq, nk = Hq * HD, Hkv * HD
    for name, gg, rr in (("dq", g_[rows, :nq], rdq), ("dk", g_[t:, nq:nq + nk], rdk[t:]), ("dv", g_[t:, nq + nk:], rdv[t:])):
        e = np.abs(gg - rr)
        assert e.max() <= 1e-2 * np.abs(rr).max(), (name, e.max(), np.abs(rr).max())
        # the rounding model (attn_rounding_model) is too slow at this size; for unit-variance inputs
        # it gives 1.15 to 1.2 x 2^-9 at every size it can run (test_attn_rounding_model.py)
        assert e.mean() <= 1.5 * 2.0 ** -9 * np.abs(rr).mean(), (name, e.mean() / np.abs(rr).mean() * 512)


def test_sdpa_argument_errors():
    a = Attn(1, 64, 2, 1, seed=1)
    with pytest.raises(f8.F8Error) as e:
        f8.sdpa_fwd(a.q, a.k, a.vt, 1, 64, 2, 1, 64, a.o, a.lse)       # head dimension other than 128
    assert e.value.code == 2
    with pytest.raises(f8.F8Error) as e:
        f8.sdpa_fwd(a.q, a.k, a.vt, 1, 60, 2, 1, HD, a.o, a.lse)       # S not a multiple of 8
    assert e.value.code == 2
    with pytest.raises(f8.F8Error) as e:
        f8.sdpa_fwd(a.q, a.k, a.vt, 1, 64, 3, 2, HD, a.o, a.lse)       # heads do not group
    assert e.value.code == 2
    with pytest.raises(f8.F8Error) as e:
        f8.sdpa_fwd(a.q, a.k, None, 1, 64, 2, 1, HD, a.o, a.lse)
    assert e.value.code == 1
