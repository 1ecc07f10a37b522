"""Chained Float8 linears: the amax of a GEMM output is taken in the epilogue and handed to the
next layer, whose quantisation of that tensor is then a single pass."""
import numpy as np
import pytest
import torch

import oracle as o
from paper_2410_06511_amd import f8
from paper_2410_06511_amd import workloads as wl
from helpers import bits, u8, f32, assert_gemm_close, qt_matches, codes_t

pytestmark = pytest.mark.gpu


def _bf(shape):
    return torch.empty(shape, dtype=torch.bfloat16, device="cuda")


def _from_bits(b):
    return torch.from_numpy(b.view(np.int16)).view(torch.bfloat16)


@pytest.mark.parametrize("gfmt", [f8.E4M3, f8.E5M2])
@pytest.mark.parametrize("M,K,N1,N2", [(272, 336, 208, 144), (512, 1024, 768, 256)])
def test_two_layer_chain_equals_unchained(M, K, N1, N2, gfmt):
    """X -> layer 1 -> Y1 -> layer 2 -> Y2, then back.  With the handed-over amax values every
    code, scale and output is bit-identical to the same layers run with their own amax passes."""
    g = torch.Generator("cpu")
    g.manual_seed(M + N2)
    X = wl.randn_bf16((M, K), 1.0, 0, generator=g).cuda()
    W1 = wl.randn_bf16((N1, K), 0.05, 0, generator=g).cuda()
    W2 = wl.randn_bf16((N2, N1), 0.05, 0, generator=g).cuda()
    dY2 = wl.randn_bf16((M, N2), 1e-3, 0, generator=g).cuda()
    d1, d2 = f8.linear_desc(M, K, N1, False, gfmt), f8.linear_desc(M, N1, N2, False, gfmt)
    ws = f8.new_workspace(1024, 1024)

    def run(chained):
        s1, s2 = f8.Saved(M, K, N1), f8.Saved(M, N1, N2)
        Y1, Y2, dX2, dW2, dX1, dW1 = _bf((M, N1)), _bf((M, N2)), _bf((M, N1)), _bf((N2, N1)), _bf((M, K)), _bf((N1, K))
        if chained:
            a_y1, a_y2, a_dx2, a_dx1 = (torch.full((1,), -1.0, device="cuda") for _ in range(4))
            f8.linear_fwd_chained(d1, X, None, W1, Y1, a_y1, s1, ws)
            f8.linear_fwd_chained(d2, Y1, a_y1, W2, Y2, a_y2, s2, ws)
            f8.linear_bwd_chained(d2, dY2, None, s2, dX2, a_dx2, dW2, ws)
            f8.linear_bwd_chained(d1, dX2, a_dx2, s1, dX1, a_dx1, dW1, ws)
            torch.cuda.synchronize()
            # the epilogue amax values are exactly the amax of what was stored
            for a, t in ((a_y1, Y1), (a_y2, Y2), (a_dx2, dX2), (a_dx1, dX1)):
                assert a.item() == o.amax(bits(t))[0]
        else:
            f8.linear_fwd(d1, X, W1, Y1, s1, ws)
            f8.linear_fwd(d2, Y1, W2, Y2, s2, ws)
            f8.linear_bwd(d2, dY2, s2, dX2, dW2, ws)
            f8.linear_bwd(d1, dX2, s1, dX1, dW1, ws)
            torch.cuda.synchronize()
        return (Y1, Y2, dX2, dW2, dX1, dW1), (s1, s2)

    (outs_c, saved_c), (outs_u, saved_u) = run(True), run(False)
    for a, b in zip(outs_c, outs_u):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    for sc, su in zip(saved_c, saved_u):
        for qc, qu in ((sc.x, su.x), (sc.w, su.w), (sc.dy, su.dy)):
            assert torch.equal(qc.q, qu.q) and qc.q_t is None and qu.q_t is None
            assert torch.equal(qc.amax, qu.amax) and torch.equal(qc.scale, qu.scale) and torch.equal(qc.inv_scale, qu.inv_scale)


def test_consumer_with_given_amax_against_oracle():
    """Layer 2 of a chain, fed with the ORACLE's layer-1 output and its amax: codes and scales
    bit-exact against the oracle's own layer 2, outputs within tolerance, and the amax values the
    GPU hands on agree with the oracle's within the GEMM tolerance."""
    M, K, N1, N2 = 2048, 1024, 4096, 1024
    g = torch.Generator("cpu")
    g.manual_seed(17)
    X = wl.randn_bf16((M, K), 1.0, 0, generator=g)
    W1 = wl.randn_bf16((N1, K), 0.02, 0, generator=g)
    W2 = wl.randn_bf16((N2, N1), 0.02, 0, generator=g)
    dY2 = wl.randn_bf16((M, N2), 1e-3, 0, generator=g)
    rY1, _, _ = o.linear_fwd(bits(X), bits(W1))
    rY2, xq2, wq2 = o.linear_fwd(rY1, bits(W2))
    rdX2, rdW2, dyq2 = o.linear_bwd(bits(dY2), xq2, wq2)
    a_y1_ref = o.amax(rY1)

    d2 = f8.linear_desc(M, N1, N2)
    s2 = f8.Saved(M, N1, N2)
    ws = f8.new_workspace(4096, 4096)
    Y1 = _from_bits(rY1).cuda()
    x_amax = torch.from_numpy(a_y1_ref).cuda()
    Y2, dX2, dW2 = _bf((M, N2)), _bf((M, N1)), _bf((N2, N1))
    a_y2, a_dx2 = torch.empty(1, device="cuda"), torch.empty(1, device="cuda")
    f8.linear_fwd_chained(d2, Y1, x_amax, W2.cuda(), Y2, a_y2, s2, ws)
    f8.linear_bwd_chained(d2, dY2.cuda(), None, s2, dX2, a_dx2, dW2, ws)
    torch.cuda.synchronize()
    for q, ref in ((s2.x, xq2), (s2.w, wq2), (s2.dy, dyq2)):
        assert np.array_equal(u8(q.q), ref.q) and qt_matches(q, ref.q.T)
        assert f32(q.amax)[0] == ref.amax[0] and f32(q.scale)[0] == ref.scale[0] and f32(q.inv_scale)[0] == ref.inv_scale[0]
    assert_gemm_close(bits(Y2), rY2, "Y2"), assert_gemm_close(bits(dX2), rdX2, "dX2"), assert_gemm_close(bits(dW2), rdW2, "dW2")
    assert abs(a_y2.item() - o.amax(rY2)[0]) <= 1e-2 * o.amax(rY2)[0]
    assert abs(a_dx2.item() - o.amax(rdX2)[0]) <= 1e-2 * o.amax(rdX2)[0]


def test_chained_full_size_pair_is_identical():
    """The 8B wq -> wo pair at M = 8192 in the launch configuration of the benchmark."""
    w = wl.WORKLOADS["llama8b"]
    X, Wq, _ = wl.make_linear_inputs(w, 0)
    _, Wo, dYo = wl.make_linear_inputs(w, 3)
    M, K, N = 8192, 4096, 4096
    d = f8.linear_desc(M, K, N)
    ws = f8.new_workspace(8192, 8192)
    Xd, Wqd, Wod, dYd = X.cuda(), Wq.cuda(), Wo.cuda(), dYo.cuda()
    res = []
    for chained in (True, False):
        s1, s2 = f8.Saved(M, K, N), f8.Saved(M, K, N)
        Y1, Y2, dX2, dW2, dX1, dW1 = (_bf((M, N)), _bf((M, N)), _bf((M, K)), _bf((N, K)), _bf((M, K)), _bf((N, K)))
        if chained:
            a1, a2, a3 = (torch.empty(1, device="cuda") for _ in range(3))
            f8.linear_fwd_chained(d, Xd, None, Wqd, Y1, a1, s1, ws)
            f8.linear_fwd_chained(d, Y1, a1, Wod, Y2, None, s2, ws)
            f8.linear_bwd_chained(d, dYd, None, s2, dX2, a2, dW2, ws)
            f8.linear_bwd_chained(d, dX2, a2, s1, dX1, a3, dW1, ws)
        else:
            f8.linear_fwd(d, Xd, Wqd, Y1, s1, ws)
            f8.linear_fwd(d, Y1, Wod, Y2, s2, ws)
            f8.linear_bwd(d, dYd, s2, dX2, dW2, ws)
            f8.linear_bwd(d, dX2, s1, dX1, dW1, ws)
        torch.cuda.synchronize()
        res.append((Y2, dX1, dW1, dW2, s2.x.q, codes_t(s1.dy), s2.x.scale, s1.dy.scale))
    for a, b in zip(*res):
        assert torch.equal(a.view(torch.uint8), b.view(torch.uint8))


def test_chained_argument_errors():
    t = torch.zeros((64, 64), dtype=torch.bfloat16, device="cuda")
    ws = f8.new_workspace(64, 64)
    with pytest.raises(f8.F8Error) as e:   # rowwise is not a chained mode
        f8.linear_fwd_chained(f8.linear_desc(64, 64, 64, True), t, None, t, t.clone(), None, f8.Saved(64, 64, 64, True), ws)
    assert e.value.code == 4
    with pytest.raises(f8.F8Error) as e:
        f8.linear_bwd_chained(f8.linear_desc(64, 64, 64), None, None, f8.Saved(64, 64, 64), t, None, t.clone(), ws)
    assert e.value.code == 1
