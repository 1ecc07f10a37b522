"""GPU parity of the whole Float8 linear (forward + backward) against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle as o
from paper_2410_06511_amd import f8
from paper_2410_06511_amd import workloads as wl
from helpers import bits, u8, f32, assert_gemm_close, sampled_check, qt_matches

pytestmark = pytest.mark.gpu


def run_linear(X, W, dY, rowwise=False, grad_fmt=f8.E4M3, transposed=False):
    """transposed: also keep transposed code tensors (tensorwise), which the backward then reads
    as F8_NT products; without them it reads the codes in place (F8_NN, F8_TN)."""
    M, K = X.shape
    N = W.shape[0]
    desc = f8.linear_desc(M, K, N, rowwise, grad_fmt)
    saved = f8.Saved(M, K, N, rowwise, transposed=transposed)
    ws = f8.new_workspace(max(M, K, N), max(M, K, N))
    Xd, Wd, dYd = X.cuda(), W.cuda(), dY.cuda()
    Y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    dX = torch.empty((M, K), dtype=torch.bfloat16, device="cuda")
    dW = torch.empty((N, K), dtype=torch.bfloat16, device="cuda")
    f8.linear_fwd(desc, Xd, Wd, Y, saved, ws)
    f8.linear_bwd(desc, dYd, saved, dX, dW, ws)
    torch.cuda.synchronize()
    return Y, dX, dW, saved


def check_quantised(q, ref, rowwise):
    """q: f8.QTensor on the GPU, ref: oracle Quantised.  Bit-exact."""
    assert np.array_equal(f32(q.amax), ref.amax)
    assert np.array_equal(f32(q.scale), ref.scale)
    assert np.array_equal(f32(q.inv_scale), ref.inv_scale)
    assert np.array_equal(u8(q.q), ref.q)
    if rowwise:
        assert np.array_equal(f32(q.amax_t), ref.amax_c)
        assert np.array_equal(f32(q.scale_t), ref.scale_c)
        assert np.array_equal(f32(q.inv_scale_t), ref.inv_scale_c)
        assert np.array_equal(u8(q.q_t), ref.q_c.T)
    else:
        assert qt_matches(q, ref.q.T)


@pytest.mark.parametrize("rowwise,grad_fmt,transposed", [(False, f8.E4M3, False), (False, f8.E5M2, False),
                                                        (False, f8.E4M3, True), (False, f8.E5M2, True),
                                                        (True, f8.E4M3, False), (True, f8.E5M2, False)])
def test_single_linear_config(rowwise, grad_fmt, transposed):
    """The small configuration: X [256,512] ~ N(0,1), W [1024,512] ~ N(0,0.02), dY [256,1024]
    ~ N(0,1e-3), seed 0.  Scales and codes bit-exact, Y / dX / dW within tolerance, in full."""
    X, W, dY = wl.make_linear_inputs(wl.WORKLOADS["single"], 0)
    Y, dX, dW, saved = run_linear(X, W, dY, rowwise, grad_fmt, transposed)
    assert (saved.x.q_t is not None) == (rowwise or transposed)
    rY, xq, wq = o.linear_fwd(bits(X), bits(W), rowwise)
    rdX, rdW, dyq = o.linear_bwd(bits(dY), xq, wq, rowwise, grad_fmt)
    check_quantised(saved.x, xq, rowwise)
    check_quantised(saved.w, wq, rowwise)
    check_quantised(saved.dy, dyq, rowwise)
    assert_gemm_close(bits(Y), rY, "Y")
    assert_gemm_close(bits(dX), rdX, "dX")
    assert_gemm_close(bits(dW), rdW, "dW")


def test_ragged_linear():
    """Sizes that are multiples of 16 only: ragged tiles in every kernel."""
    g = torch.Generator("cpu")
    g.manual_seed(77)
    M, K, N = 272, 336, 208
    X = wl.randn_bf16((M, K), 1.0, 0, generator=g)
    W = wl.randn_bf16((N, K), 0.02, 0, generator=g)
    dY = wl.randn_bf16((M, N), 1e-3, 0, generator=g)
    for rowwise, transposed in ((False, False), (False, True), (True, False)):
        Y, dX, dW, saved = run_linear(X, W, dY, rowwise, f8.E5M2, transposed)
        rY, xq, wq = o.linear_fwd(bits(X), bits(W), rowwise)
        rdX, rdW, dyq = o.linear_bwd(bits(dY), xq, wq, rowwise, o.E5M2)
        check_quantised(saved.x, xq, rowwise)
        check_quantised(saved.w, wq, rowwise)
        check_quantised(saved.dy, dyq, rowwise)
        assert_gemm_close(bits(Y), rY), assert_gemm_close(bits(dX), rdX), assert_gemm_close(bits(dW), rdW)


def test_linear_exact_case_bit_for_bit():
    """Inputs in {0, +-0.5, +-1, +-2} with one +-3.5: amax 3.5, scale 128, lossless casts and
    exact accumulation, so Y, dX, dW equal the bf16-rounded exact products bit for bit."""
    rng = np.random.default_rng(31)
    vals = np.array([0, 0.5, -0.5, 1, -1, 2, -2], np.float32)

    def draw(shape):
        t = vals[rng.integers(0, vals.size, shape)]
        t.flat[rng.integers(0, t.size)] = 3.5
        return t
    _exact_linear(draw, 512, 768, 256)


def test_linear_exact_case_with_split_contraction():
    """The same with a weight gradient of few output tiles and a long contraction (dW [512, 1024]
    over 4096 tokens): that product is split along its contraction into ranges whose fp32 partial
    sums a second kernel adds; every sum is exact, so the result is still bit for bit the rounded
    exact product."""
    rng = np.random.default_rng(32)
    vals = np.array([0, 0.5, -0.5, 1, -1, 2, -2], np.float32)

    def draw(shape):
        t = vals[rng.integers(0, vals.size, shape)]
        t.flat[rng.integers(0, t.size)] = 3.5
        return t
    _exact_linear(draw, 4096, 1024, 512)


def _exact_linear(draw, M, K, N):
    X, W, dY = draw((M, K)), draw((N, K)), draw((M, N))
    tb = lambda a: torch.from_numpy(a).to(torch.bfloat16)
    for gf, transposed in ((f8.E4M3, False), (f8.E5M2, False), (f8.E4M3, True)):
        Y, dX, dW, saved = run_linear(tb(X), tb(W), tb(dY), False, gf, transposed)
        assert f32(saved.x.scale)[0] == 128.0 and f32(saved.dy.scale)[0] == o.fmax(gf) / 3.5
        x64, w64, d64 = X.astype(np.float64), W.astype(np.float64), dY.astype(np.float64)
        ex = lambda a: torch.from_numpy(a).to(torch.bfloat16).view(torch.uint16).numpy()
        assert np.array_equal(bits(Y), ex(x64 @ w64.T))
        assert np.array_equal(bits(dX), ex(d64 @ w64))
        assert np.array_equal(bits(dW), ex(d64.T @ x64))


def _full_size_cases():
    """Every distinct linear shape of every Llama-shaped workload, in each of the variants the
    workload is run in (tensorwise / rowwise scaling, e4m3 / e5m2 gradients)."""
    cases = []
    seen = set()
    for key, w in wl.WORKLOADS.items():
        if key == "single":
            continue
        for li, lin in enumerate(w.linears):
            if (lin.M, lin.K, lin.N, w.variants) in seen:
                continue  # w3 repeats w1's shape, wv wk's, wo wq's; the fused block repeats wo and w2
            seen.add((lin.M, lin.K, lin.N, w.variants))
            for gran, gfmt in w.variants:
                cases.append(pytest.param(key, li, gran == "rowwise", f8.E5M2 if gfmt == "e5m2" else f8.E4M3, False,
                                          id=f"{key}-{lin.name}-{gran}-{gfmt}"))
    # the backward on transposed code copies (F8_NT products) at two 8B shapes
    for li in (1, 4):
        cases.append(pytest.param("llama8b", li, False, f8.E4M3, True,
                                  id=f"llama8b-{wl.WORKLOADS['llama8b'].linears[li].name}-tensorwise-e4m3-transposed-copies"))
    return cases


@pytest.mark.parametrize("key,li,rowwise,grad_fmt,transposed", _full_size_cases())
def test_full_size_linear(key, li, rowwise, grad_fmt, transposed):
    """Full-size linears of the Llama-shaped workloads, exactly as the benchmark launches them.
    amax / scales / codes compared in full; Y, dX, dW on at least 64 whole rows and 64 whole
    columns each (seeded, plus the lines on both sides of 256-tile boundaries), computed by the
    oracle from the same codes."""
    w = wl.WORKLOADS[key]
    X, W, dY = wl.make_linear_inputs(w, li)
    Y, dX, dW, saved = run_linear(X, W, dY, rowwise, grad_fmt, transposed)
    g = o.ROWWISE if rowwise else o.TENSORWISE
    rng = np.random.default_rng(li)
    xb, wb, dyb = bits(X), bits(W), bits(dY)
    ax, sx, isx, qx = o.amax_cast(xb, g, o.E4M3)
    aw, sw, isw, qw = o.amax_cast(wb, g, o.E4M3)
    ady, sdy, isdy, qdy = o.amax_cast(dyb, g, grad_fmt)
    for q, (a, s, i, c) in ((saved.x, (ax, sx, isx, qx)), (saved.w, (aw, sw, isw, qw)), (saved.dy, (ady, sdy, isdy, qdy))):
        assert np.array_equal(f32(q.amax), a) and np.array_equal(f32(q.scale), s) and np.array_equal(f32(q.inv_scale), i)
        assert np.array_equal(u8(q.q), c)
    sampled_check("Y", bits(Y), o.NT, qx, o.E4M3, qw, o.E4M3, isx, isw, g, rng)
    if not rowwise:
        for q in (saved.x, saved.w, saved.dy):
            assert (q.q_t is not None) == transposed
            if transposed:
                assert torch.equal(q.q_t, q.q.t().contiguous())
        sampled_check("dX", bits(dX), o.NN, qdy, grad_fmt, qw, o.E4M3, isdy, isw, g, rng)
        sampled_check("dW", bits(dW), o.TN, qdy, grad_fmt, qx, o.E4M3, isdy, isx, g, rng)
    else:
        _, _, iswc, qwc = o.amax_cast(wb, o.COLWISE, o.E4M3)
        _, _, isxc, qxc = o.amax_cast(xb, o.COLWISE, o.E4M3)
        _, _, isdyc, qdyc = o.amax_cast(dyb, o.COLWISE, grad_fmt)
        assert np.array_equal(u8(saved.w.q_t), qwc.T) and np.array_equal(u8(saved.x.q_t), qxc.T)
        assert np.array_equal(u8(saved.dy.q_t), qdyc.T)
        sampled_check("dX", bits(dX), o.NN, qdy, grad_fmt, qwc, o.E4M3, isdy, iswc, g, rng)
        sampled_check("dW", bits(dW), o.TN, qdyc, grad_fmt, qxc, o.E4M3, isdyc, isxc, g, rng)


@pytest.mark.parametrize("M,K,N,transposed", [(16, 16, 16, False), (272, 336, 208, False), (16, 4096, 2048, False),
                                              (4096, 4096, 1024, False), (2064, 2048, 4112, False), (272, 336, 208, True)])
def test_forward_quantisation_of_x_and_w_together(M, K, N, transposed):
    """f8_linear_fwd_quantise: X and W in one amax launch and one cast launch, the grid split between
    them by size (X the larger, W the larger, both larger than one launch's block budget so that
    the shares are proportional, tiny).  Each tensor's largest magnitude sits where only the last or
    the first thread of its share looks.  Bit-exact against the oracle, and the same bits as
    quantising each tensor by itself."""
    g = torch.Generator("cpu")
    g.manual_seed(1234 + M + N)
    X, W = wl.randn_bf16((M, K), 1.0, 0, generator=g), wl.randn_bf16((N, K), 0.02, 0, generator=g)
    X[-1, -1] = 37.5
    W[0, 0] = -0.75
    desc = f8.linear_desc(M, K, N, False)
    ws = f8.new_workspace(max(M, K, N), max(M, K, N))
    both, single = f8.Saved(M, K, N, False, transposed=transposed), f8.Saved(M, K, N, False, transposed=transposed)
    Xd, Wd = X.cuda(), W.cuda()
    f8.linear_fwd_quantise(desc, Xd, Wd, both, ws)
    f8.quantise(Xd, f8.TENSORWISE, f8.E4M3, single.x, ws)
    f8.quantise(Wd, f8.TENSORWISE, f8.E4M3, single.w, ws)
    torch.cuda.synchronize()
    for got, alone, t in ((both.x, single.x, X), (both.w, single.w, W)):
        a, sc, inv, q = o.amax_cast(bits(t), o.TENSORWISE, o.E4M3)
        assert np.array_equal(f32(got.amax), a) and np.array_equal(f32(got.scale), sc) and np.array_equal(f32(got.inv_scale), inv)
        assert np.array_equal(u8(got.q), q)
        assert qt_matches(got, q.T)
        assert torch.equal(got.q, alone.q) and torch.equal(got.scale, alone.scale)


@pytest.mark.parametrize("M,K,N1,N2", [(272, 336, 208, 96), (16384, 4096, 4096, 1024)])
def test_linears_on_a_shared_input_reuse_its_codes(M, K, N1, N2):
    """Two linears that read one activation (wq and wk; also at their size in the 16384-token block,
    as the benchmark runs them): the second runs on the first's X codes (f8_linear_fwd_xq, only its
    W is cast) and gives the bits of a forward + backward that casts X itself."""
    g = torch.Generator("cpu")
    g.manual_seed(91)
    X = wl.randn_bf16((M, K), 1.0, 0, generator=g).cuda()
    W1, W2 = wl.randn_bf16((N1, K), 0.02, 0, generator=g).cuda(), wl.randn_bf16((N2, K), 0.02, 0, generator=g).cuda()
    dY2 = wl.randn_bf16((M, N2), 1e-3, 0, generator=g).cuda()
    ws = f8.new_workspace(max(M, K, N1), max(M, K, N1))
    bf = dict(dtype=torch.bfloat16, device="cuda")
    d1, d2 = f8.linear_desc(M, K, N1), f8.linear_desc(M, K, N2)
    s1 = f8.Saved(M, K, N1)
    shared, own = f8.Saved(M, K, N2, x=s1.x), f8.Saved(M, K, N2)
    Y1, Ya, Yb = torch.empty((M, N1), **bf), torch.empty((M, N2), **bf), torch.empty((M, N2), **bf)
    f8.linear_fwd(d1, X, W1, Y1, s1, ws)
    f8.linear_fwd_xq(d2, f8.ScalingState(f8.DYNAMIC, 1), W2, Ya, shared, ws)
    f8.linear_fwd(d2, X, W2, Yb, own, ws)
    dXa, dXb = torch.empty((M, K), **bf), torch.empty((M, K), **bf)
    dWa, dWb = torch.empty((N2, K), **bf), torch.empty((N2, K), **bf)
    f8.linear_bwd(d2, dY2, shared, dXa, dWa, ws)
    f8.linear_bwd(d2, dY2, own, dXb, dWb, ws)
    torch.cuda.synchronize()
    assert shared.x.q.data_ptr() == s1.x.q.data_ptr() and torch.equal(s1.x.q, own.x.q)
    for a_, b_ in ((Ya, Yb), (dXa, dXb), (dWa, dWb)):
        assert torch.equal(a_.view(torch.int16), b_.view(torch.int16))


@pytest.mark.parametrize("rowwise", [False, True])
def test_forward_with_kept_weight_codes(rowwise):
    """A second micro-batch against the weight codes kept from the first: the same bits as a full
    f8_linear_fwd on that micro-batch, and the weight's saved state is left untouched."""
    M, K, N = 272, 336, 208
    g = torch.Generator("cpu")
    g.manual_seed(77)
    X1, X2 = wl.randn_bf16((M, K), 1.0, 0, generator=g).cuda(), wl.randn_bf16((M, K), 2.0, 0, generator=g).cuda()
    W = wl.randn_bf16((N, K), 0.02, 0, generator=g).cuda()
    desc = f8.linear_desc(M, K, N, rowwise)
    ws = f8.new_workspace(max(M, K, N), max(M, K, N))
    kept, full = f8.Saved(M, K, N, rowwise), f8.Saved(M, K, N, rowwise)
    Y1, Y2, Yref = (torch.empty((M, N), dtype=torch.bfloat16, device="cuda") for _ in range(3))
    f8.linear_fwd(desc, X1, W, Y1, kept, ws)
    torch.cuda.synchronize()
    w_before = kept.w.q.clone()
    f8.linear_fwd_wq(desc, X2, Y2, kept, ws)
    f8.linear_fwd(desc, X2, W, Yref, full, ws)
    torch.cuda.synchronize()
    assert torch.equal(Y2.view(torch.int16), Yref.view(torch.int16))
    assert torch.equal(kept.x.q, full.x.q) and torch.equal(kept.w.q, w_before)



@pytest.mark.parametrize("M,K,N,grad_fmt", [(528, 768, 784, f8.E4M3), (4368, 512, 4112, f8.E5M2), (2048, 1024, 4096, f8.E4M3)])
def test_backward_in_place_equals_backward_on_transposed_copies(M, K, N, grad_fmt):
    """dX and dW from the codes read in place (F8_NN / F8_TN: the kernel turns the k-major
    operand) against the same products on transposed code copies (F8_NT): the same k order
    inside every matrix instruction and the same tiles, so the same bits."""
    g = torch.Generator("cpu")
    g.manual_seed(M + K + N)
    X = wl.randn_bf16((M, K), 1.0, 0, generator=g)
    W = wl.randn_bf16((N, K), 0.02, 0, generator=g)
    dY = wl.randn_bf16((M, N), 1e-3, 0, generator=g)
    Y0, dX0, dW0, s0 = run_linear(X, W, dY, False, grad_fmt, transposed=False)
    Y1, dX1, dW1, s1 = run_linear(X, W, dY, False, grad_fmt, transposed=True)
    assert torch.equal(s0.dy.q, s1.dy.q) and torch.equal(s1.dy.q_t, s1.dy.q.t().contiguous())
    for a, b in ((Y0, Y1), (dX0, dX1), (dW0, dW1)):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))


def test_backward_with_split_contraction_is_deterministic():
    """8B wk shape at 4096 tokens: dW [1024, 4096] has 64 output tiles and is computed in
    contraction ranges added in a fixed order; repeated calls give identical bits, and the result
    agrees with the oracle on sampled lines."""
    w = wl.WORKLOADS["llama8b"]
    X, W, dY = wl.make_linear_inputs(w, 1, M=4096)
    outs = [run_linear(X, W, dY)[1:3] for _ in range(3)]
    for dX, dW in outs[1:]:
        assert torch.equal(dX.view(torch.int16), outs[0][0].view(torch.int16))
        assert torch.equal(dW.view(torch.int16), outs[0][1].view(torch.int16))
    g = o.TENSORWISE
    _, _, isx, qx = o.amax_cast(bits(X), g, o.E4M3)
    _, _, isdy, qdy = o.amax_cast(bits(dY), g, o.E4M3)
    sampled_check("dW", bits(outs[0][1]), o.TN, qdy, o.E4M3, qx, o.E4M3, isdy, isx, g, np.random.default_rng(1))


@pytest.mark.parametrize("rowwise,transposed", [(True, False), (False, True), (False, False)])
def test_split_contraction_against_oracle(rowwise, transposed):
    """A linear whose weight gradient takes the split-contraction path (dW [512, 1024] over 4096
    tokens), with per-tensor and with per-row / per-column scales: everything against the oracle
    in full."""
    g = torch.Generator("cpu")
    g.manual_seed(4096)
    M, K, N = 4096, 1024, 512
    X = wl.randn_bf16((M, K), 1.0, 0, generator=g)
    W = wl.randn_bf16((N, K), 0.02, 0, generator=g)
    dY = wl.randn_bf16((M, N), 1e-3, 0, generator=g)
    Y, dX, dW, saved = run_linear(X, W, dY, rowwise, f8.E5M2, transposed)
    rY, xq, wq = o.linear_fwd(bits(X), bits(W), rowwise)
    rdX, rdW, dyq = o.linear_bwd(bits(dY), xq, wq, rowwise, o.E5M2)
    check_quantised(saved.dy, dyq, rowwise)
    assert_gemm_close(bits(Y), rY), assert_gemm_close(bits(dX), rdX), assert_gemm_close(bits(dW), rdW)
    # per-line criterion too, so that a wrong range of rows cannot hide behind the global maximum
    gf, rf = o.bf16_to_f32(bits(dW)).astype(np.float64), o.bf16_to_f32(rdW).astype(np.float64)
    assert (np.abs(gf - rf).max(axis=1) <= 1e-2 * np.abs(rf).max()).all()
