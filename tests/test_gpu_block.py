"""The bf16 operations between the Float8 linears of a transformer block, through the C ABI,
against oracle/block_oracle.py: rotary embedding, transposition, residual addition, RMSNorm
backward."""
import numpy as np
import pytest
import torch

import oracle as o
from oracle import block_oracle as bo
from paper_2410_06511_amd import f8
from paper_2410_06511_amd import workloads as wl
from helpers import bits

pytestmark = pytest.mark.gpu


def gen(shape, seed, std=1.0):
    g = torch.Generator("cpu")
    g.manual_seed(seed)
    return wl.randn_bf16(shape, std, 0, generator=g)


def assert_rope_close(got_bits, ref_bits, x_bits, what):
    """Each output is a sum of two products taken in fp32 (the oracle: fp64): one bf16 unit in the
    last place of the result plus a few fp32 roundings of the terms, which matter only where the
    two products cancel."""
    got, ref = (o.bf16_to_f32(b).astype(np.float64) for b in (got_bits, ref_bits))
    x = np.abs(o.bf16_to_f32(x_bits).astype(np.float64))
    pair = x.reshape(x.shape[0], -1, 2).sum(axis=2)
    mag = np.repeat(pair, 2, axis=1)
    assert (np.abs(got - ref) <= 2.0 ** -7 * np.abs(ref) + 2.0 ** -20 * mag + 1e-38).all(), what
    assert (got_bits == ref_bits).mean() > 0.98, what


@pytest.mark.parametrize("M,S,nh,hd", [(8, 8, 1, 8), (136, 24, 3, 64), (512, 512, 5, 128), (1024, 256, 2, 256)])
def test_rope_and_its_transposed_copy(M, S, nh, hd):
    x = gen((M, nh * hd), M + hd)
    out = torch.empty((M, nh * hd), dtype=torch.bfloat16, device="cuda")
    out_t = torch.empty((nh * hd, M), dtype=torch.bfloat16, device="cuda")
    f8.rope(x.cuda(), S, nh, hd, out, out_t)
    torch.cuda.synchronize()
    ref = bo.rope(bits(x), S, hd)
    assert_rope_close(bits(out), ref, bits(x), "rope")
    assert np.array_equal(bits(out_t), bits(out).T)
    # rows at position 0 come back bit for bit
    assert np.array_equal(bits(out)[::S], bits(x)[::S])
    # inverse rotation (the backward), only one of the outputs
    back = torch.empty_like(out)
    f8.rope(x.cuda(), S, nh, hd, back, None, inverse=True)
    only_t = torch.empty_like(out_t)
    f8.rope(x.cuda(), S, nh, hd, None, only_t, inverse=True)
    torch.cuda.synchronize()
    assert_rope_close(bits(back), bo.rope(bits(x), S, hd, inverse=True), bits(x), "rope inverse")
    assert np.array_equal(bits(only_t), bits(back).T)
    # amax cell: raised by each producer to the maximum of what it wrote
    cell = torch.zeros(1, device="cuda")
    f8.rope(x.cuda(), S, nh, hd, out, None, amax_inout=cell)
    torch.cuda.synchronize()
    first = cell.item()
    assert first == o.amax(bits(out))[0]
    f8.rope((x * 3).bfloat16().cuda(), S, nh, hd, back, None, amax_inout=cell)
    torch.cuda.synchronize()
    assert cell.item() == max(first, o.amax(bits(back))[0])


def test_rope_long_sequence_positions_and_column_slices():
    """Positions up to 8191 (the angle is reduced in fp64) on slices of a wider tensor, as q and k
    are slices of the fused q|k|v linear's output."""
    M, S, hq, hkv, hd = 8192, 8192, 2, 1, 128
    wide = gen((M, (hq + 2 * hkv) * hd), 7)
    wd = wide.cuda()
    q, k = wd[:, :hq * hd], wd[:, hq * hd:(hq + hkv) * hd]
    dst = torch.zeros((M, (hq + hkv) * hd), dtype=torch.bfloat16, device="cuda")
    kt = torch.empty((hkv * hd, M), dtype=torch.bfloat16, device="cuda")
    f8.rope(q, S, hq, hd, dst[:, :hq * hd], None)
    f8.rope(k, S, hkv, hd, dst[:, hq * hd:], kt)
    torch.cuda.synchronize()
    rq = bo.rope(bits(wide)[:, :hq * hd], S, hd)
    rk = bo.rope(bits(wide)[:, hq * hd:(hq + hkv) * hd], S, hd)
    got = bits(dst)
    assert_rope_close(got[:, :hq * hd], rq, bits(wide)[:, :hq * hd], "q")
    assert_rope_close(got[:, hq * hd:], rk, bits(wide)[:, hq * hd:(hq + hkv) * hd], "k")
    assert np.array_equal(bits(kt), got[:, hq * hd:].T)


@pytest.mark.parametrize("R,C", [(8, 8), (72, 200), (1024, 384)])
def test_transpose_and_add(R, C):
    x, y = gen((R, C), R), gen((R, C), C)
    t = torch.empty((C, R), dtype=torch.bfloat16, device="cuda")
    s = torch.empty((R, C), dtype=torch.bfloat16, device="cuda")
    f8.transpose_bf16(x.cuda(), t)
    f8.add(x.cuda(), y.cuda(), s)
    torch.cuda.synchronize()
    assert np.array_equal(bits(t), bo.transpose(bits(x)))
    assert np.array_equal(bits(s), bo.add(bits(x), bits(y)))      # one fp32 addition, one rounding: exact
    # a column slice as the source
    wide = gen((R, 2 * C), 3).cuda()
    f8.transpose_bf16(wide[:, C:], t)
    torch.cuda.synchronize()
    assert np.array_equal(bits(t), bits(wide)[:, C:].T)


@pytest.mark.parametrize("M,D", [(16, 16), (272, 336), (1024, 4096), (4112, 1024)])
def test_rmsnorm_backward(M, D):
    x, g, dy = gen((M, D), M), gen((D,), D, 0.5), gen((M, D), M + D, 1e-2)
    ws = f8.new_workspace(M, D)
    y = torch.empty((M, D), dtype=torch.bfloat16, device="cuda")
    rstd = torch.empty(M, device="cuda")
    dx = torch.empty((M, D), dtype=torch.bfloat16, device="cuda")
    dg = torch.empty(D, device="cuda")
    f8.rmsnorm(x.cuda(), g.cuda(), 1e-5, y, rstd)
    f8.rmsnorm_bwd(x.cuda(), g.cuda(), rstd, dy.cuda(), dx, dg, ws)
    torch.cuda.synchronize()
    rdx, rdg = bo.rmsnorm_bwd(bits(x), bits(g), bits(dy), 1e-5)
    # dx is a difference of two products: absolute error of a few fp32 roundings of its terms
    got, ref = o.bf16_to_f32(bits(dx)).astype(np.float64), o.bf16_to_f32(rdx).astype(np.float64)
    xf, gf, df = (o.bf16_to_f32(bits(t)).astype(np.float64) for t in (x, g, dy))
    r = 1.0 / np.sqrt((xf * xf).mean(axis=1, keepdims=True) + 1e-5)
    mag = np.abs(r * gf[None, :] * df) + np.abs(xf) * r ** 3 * np.abs((xf * gf[None, :] * df).sum(axis=1, keepdims=True)) / D
    assert (np.abs(got - ref) <= 2.0 ** -7 * mag + 1e-30).all()
    assert (bits(dx) == rdx).mean() > 0.97
    # dg: fp32 sums of M terms against fp64
    terms = np.abs(df * xf * r).sum(axis=0)
    assert (np.abs(dg.cpu().numpy().astype(np.float64) - rdg) <= 1e-5 * terms + 1e-30).all()
    # reproducible, and each output alone gives the same values
    dx2, dg2 = torch.empty_like(dx), torch.empty_like(dg)
    f8.rmsnorm_bwd(x.cuda(), g.cuda(), rstd, dy.cuda(), dx2, None)
    f8.rmsnorm_bwd(x.cuda(), g.cuda(), rstd, dy.cuda(), None, dg2, ws)
    torch.cuda.synchronize()
    assert torch.equal(dx.view(torch.int16), dx2.view(torch.int16)) and torch.equal(dg, dg2)
    # with the residual branch's gradient added inside: the bits of the two calls in sequence
    res = gen((M, D), 5 * M + D, 1e-2).cuda()
    ref_sum, fused, dg3 = torch.empty_like(dx), torch.empty_like(dx), torch.empty_like(dg)
    f8.add(res, dx, ref_sum)
    f8.rmsnorm_bwd_add(x.cuda(), g.cuda(), rstd, dy.cuda(), res, fused, dg3, ws)
    torch.cuda.synchronize()
    assert torch.equal(ref_sum.view(torch.int16), fused.view(torch.int16)) and torch.equal(dg, dg3)
    # the amax cell is raised to the maximum magnitude written, and never lowered
    cell = torch.zeros(1, device="cuda")
    f8.rmsnorm_bwd_add(x.cuda(), g.cuda(), rstd, dy.cuda(), res, fused, dg3, ws, amax_dx_inout=cell)
    torch.cuda.synchronize()
    assert cell.item() == o.amax(bits(fused))[0]
    cell.fill_(1e9)
    f8.rmsnorm_bwd_add(x.cuda(), g.cuda(), rstd, dy.cuda(), res, fused, dg3, ws, amax_dx_inout=cell)
    torch.cuda.synchronize()
    assert cell.item() == 1e9


def test_block_glue_argument_errors():
    x = torch.zeros((16, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(f8.F8Error) as e:
        f8.rope(x, 16, 1, 64, None, None)
    assert e.value.code == 1
    with pytest.raises(f8.F8Error) as e:
        f8.rope(x, 16, 16, 4, x, None)          # hd not a multiple of 8
    assert e.value.code == 2
    with pytest.raises(f8.F8Error) as e:
        f8.rope(x, 0, 1, 64, x, None)           # sequence length < 1
    assert e.value.code == 2
    dg = torch.zeros(64, device="cuda")
    rs = torch.zeros(16, device="cuda")
    with pytest.raises(f8.F8Error) as e:
        f8.rmsnorm_bwd(x, x[0], rs, x, None, dg, None)   # dg needs the workspace
    assert e.value.code == 5
