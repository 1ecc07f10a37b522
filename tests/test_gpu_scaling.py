"""GPU parity of delayed and static scaling (the two per-tensor strategies the paper names
beside dynamic scaling) against the CPU oracle: the measuring cast, the amax history, and the
linear layer over several steps."""
import numpy as np
import pytest
import torch

import oracle as o
from paper_2410_06511_amd import f8
from paper_2410_06511_amd import workloads as wl
from helpers import bits, u8, f32, assert_gemm_close, sampled_check, qt_matches, codes_t

pytestmark = pytest.mark.gpu


def _dev_f32(a):
    return torch.from_numpy(np.asarray(a, dtype=np.float32)).cuda()


@pytest.mark.parametrize("fmt", [f8.E4M3, f8.E5M2])
@pytest.mark.parametrize("rows,cols", [(16, 16), (272, 336), (128, 1024), (640, 384)])
def test_cast_amax_matches_cast_and_amax(fmt, rows, cols):
    g = torch.Generator("cpu")
    g.manual_seed(rows + cols)
    x = wl.randn_bf16((rows, cols), 2.0, 0, generator=g)
    xb = bits(x)
    scale = np.array([o.fmax(fmt) / 3.0], np.float32)       # saturates part of the tensor
    ws = f8.new_workspace(rows, cols)
    for want_out, want_t in ((True, True), (True, False), (False, True)):
        out = torch.full((rows, cols), 0xAA, dtype=torch.uint8, device="cuda") if want_out else None
        out_t = torch.full((cols, rows), 0xAA, dtype=torch.uint8, device="cuda") if want_t else None
        amax = torch.full((1,), -1.0, device="cuda")
        f8.cast_amax(x.cuda(), _dev_f32(scale), fmt, amax, out, out_t, ws)
        torch.cuda.synchronize()
        ref = o.cast(xb, scale, o.TENSORWISE, fmt)
        assert f32(amax)[0] == o.amax(xb)[0]
        if want_out:
            assert np.array_equal(u8(out), ref)
        if want_t:
            assert np.array_equal(u8(out_t), ref.T)


def test_cast_amax_padded_rows_and_empty():
    rows, cols, ld = 144, 80, 96
    g = torch.Generator("cpu")
    g.manual_seed(9)
    buf = wl.randn_bf16((rows, ld), 1.0, 0, generator=g)
    buf[:, cols:] = 1000.0          # outside the matrix: must not reach amax
    xd = buf.cuda()
    view = xd[:, :cols]
    scale = _dev_f32([7.0])
    out = torch.empty((rows, cols), dtype=torch.uint8, device="cuda")
    amax = torch.empty(1, device="cuda")
    ws = f8.new_workspace(rows, cols)
    f8.cast_amax(view, scale, f8.E4M3, amax, out, None, ws)
    torch.cuda.synchronize()
    xb = bits(buf)[:, :cols]
    assert f32(amax)[0] == o.amax(xb)[0]
    assert np.array_equal(u8(out), o.cast(xb, np.array([7.0], np.float32), o.TENSORWISE, o.E4M3))
    # empty tensor: amax 0, nothing else written (raw call: an empty torch tensor has no address)
    amax.fill_(5.0)
    code = f8.lib().f8_cast_amax(xd.data_ptr(), 0, 32, 32, scale.data_ptr(), 0, out.data_ptr(), 32, None, 0,
                                 amax.data_ptr(), ws.data_ptr(), ws.numel() * ws.element_size(), None)
    torch.cuda.synchronize()
    assert code == 0 and f32(amax)[0] == 0.0


@pytest.mark.parametrize("fmt", [f8.E4M3, f8.E5M2])
@pytest.mark.parametrize("H", [1, 3, 16])
def test_history_push_sequence(fmt, H):
    rng = np.random.default_rng(H)
    seq = (np.abs(rng.standard_normal(24)) * 5.0).astype(np.float32)
    seq[5] = 0.0
    hist_ref = np.zeros(H, np.float32)
    hist = torch.zeros(H, device="cuda")
    s, inv = torch.empty(1, device="cuda"), torch.empty(1, device="cuda")
    for a in seq:
        f8.amax_history_push(hist, _dev_f32([a]), fmt, s, inv)
        s_ref, inv_ref = o.history_push(hist_ref, a, fmt)
        assert f32(s)[0] == s_ref[0] and f32(inv)[0] == inv_ref[0]
        assert np.array_equal(f32(hist), hist_ref)


def _seed(state_gpu, state_ref, X, W, dY, gfmt, ws):
    """First-step initialisation on both sides: record the first batch's amax values."""
    a = torch.empty(1, device="cuda")
    for key, t, fmt in (("x", X, f8.E4M3), ("w", W, f8.E4M3), ("dy", dY, gfmt)):
        f8.amax(t.cuda(), f8.TENSORWISE, a, ws)
        f8.amax_history_push(getattr(state_gpu, "hist_" + key), a, fmt, getattr(state_gpu, "scale_" + key))
        state_ref.scale[key], _ = o.history_push(state_ref.hist[key], o.amax(bits(t))[0], fmt)


def _check_q(q, ref, with_amax=True):
    assert np.array_equal(u8(q.q), ref.q) and qt_matches(q, ref.q.T)
    assert f32(q.scale)[0] == ref.scale[0] and f32(q.inv_scale)[0] == ref.inv_scale[0]
    if with_amax:
        assert f32(q.amax)[0] == ref.amax[0]


@pytest.mark.parametrize("gfmt", [f8.E4M3, f8.E5M2])
@pytest.mark.parametrize("M,K,N,H", [(272, 336, 208, 3), (512, 768, 256, 2)])
def test_linear_delayed_over_several_steps(M, K, N, H, gfmt):
    """Six steps whose tensors grow and shrink from step to step, so that the window maximum
    is sometimes stale (saturation) and sometimes expires.  Codes, scales, amax, histories and
    next-step scales bit-exact at every step; Y, dX, dW within the GEMM tolerance."""
    g = torch.Generator("cpu")
    g.manual_seed(M + H)
    factors = [1.0, 4.0, 0.5, 0.25, 0.125, 2.0]
    desc = f8.linear_desc(M, K, N, False, gfmt)
    saved = f8.Saved(M, K, N, False)
    ws = f8.new_workspace(max(M, K, N), max(M, K, N))
    st = f8.ScalingState(f8.DELAYED, H)
    st_ref = o.ScalingState(o.DELAYED, H)
    Y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    dX = torch.empty((M, K), dtype=torch.bfloat16, device="cuda")
    dW = torch.empty((N, K), dtype=torch.bfloat16, device="cuda")
    for step, fac in enumerate(factors):
        X = wl.randn_bf16((M, K), 1.0 * fac, 0, generator=g)
        W = wl.randn_bf16((N, K), 0.02 * (1.0 + 0.1 * step), 0, generator=g)
        dY = wl.randn_bf16((M, N), 1e-3 / fac, 0, generator=g)
        if step == 0:
            _seed(st, st_ref, X, W, dY, gfmt, ws)
        f8.linear_fwd_scaled(desc, st, X.cuda(), W.cuda(), Y, saved, ws)
        f8.linear_bwd_scaled(desc, st, dY.cuda(), saved, dX, dW, ws)
        torch.cuda.synchronize()
        rY, xq, wq = o.linear_fwd_scaled(bits(X), bits(W), st_ref)
        rdX, rdW, dyq = o.linear_bwd_scaled(bits(dY), xq, wq, st_ref, gfmt)
        _check_q(saved.x, xq), _check_q(saved.w, wq), _check_q(saved.dy, dyq)
        for key in ("x", "w", "dy"):
            assert np.array_equal(f32(getattr(st, "hist_" + key)), st_ref.hist[key]), (step, key)
            assert f32(getattr(st, "scale_" + key))[0] == st_ref.scale[key][0], (step, key)
        assert_gemm_close(bits(Y), rY, f"Y step {step}")
        assert_gemm_close(bits(dX), rdX, f"dX step {step}")
        assert_gemm_close(bits(dW), rdW, f"dW step {step}")


def test_linear_static():
    M, K, N = 272, 336, 208
    g = torch.Generator("cpu")
    g.manual_seed(5)
    st = f8.ScalingState(f8.STATIC)
    st_ref = o.ScalingState(o.STATIC)
    for key, v in (("x", 100.0), ("w", 4096.0), ("dy", 2.0 ** 17)):
        getattr(st, "scale_" + key).fill_(v)
        st_ref.scale[key][:] = v
    desc = f8.linear_desc(M, K, N, False, f8.E5M2)
    saved = f8.Saved(M, K, N, False)
    ws = f8.new_workspace(max(M, K, N), max(M, K, N))
    Y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    dX = torch.empty((M, K), dtype=torch.bfloat16, device="cuda")
    dW = torch.empty((N, K), dtype=torch.bfloat16, device="cuda")
    for step in range(2):
        X = wl.randn_bf16((M, K), 1.0, 0, generator=g)
        W = wl.randn_bf16((N, K), 0.02, 0, generator=g)
        dY = wl.randn_bf16((M, N), 1e-3, 0, generator=g)
        f8.linear_fwd_scaled(desc, st, X.cuda(), W.cuda(), Y, saved, ws)
        f8.linear_bwd_scaled(desc, st, dY.cuda(), saved, dX, dW, ws)
        torch.cuda.synchronize()
        rY, xq, wq = o.linear_fwd_scaled(bits(X), bits(W), st_ref)
        rdX, rdW, dyq = o.linear_bwd_scaled(bits(dY), xq, wq, st_ref, o.E5M2)
        _check_q(saved.x, xq, False), _check_q(saved.w, wq, False), _check_q(saved.dy, dyq, False)
        assert f32(st.scale_x)[0] == 100.0 and f32(st.scale_dy)[0] == 2.0 ** 17
        assert_gemm_close(bits(Y), rY), assert_gemm_close(bits(dX), rdX), assert_gemm_close(bits(dW), rdW)


def test_scaled_dynamic_mode_is_the_dynamic_linear():
    X, W, dY = wl.make_linear_inputs(wl.WORKLOADS["single"], 0)
    M, K = X.shape
    N = W.shape[0]
    desc = f8.linear_desc(M, K, N, False, f8.E4M3)
    ws = f8.new_workspace(max(M, K, N), max(M, K, N))
    outs = []
    for scaled in (False, True):
        saved = f8.Saved(M, K, N, False)
        Y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        dX = torch.empty((M, K), dtype=torch.bfloat16, device="cuda")
        dW = torch.empty((N, K), dtype=torch.bfloat16, device="cuda")
        if scaled:
            st = f8.ScalingState(f8.DYNAMIC)
            f8.linear_fwd_scaled(desc, st, X.cuda(), W.cuda(), Y, saved, ws)
            f8.linear_bwd_scaled(desc, st, dY.cuda(), saved, dX, dW, ws)
        else:
            f8.linear_fwd(desc, X.cuda(), W.cuda(), Y, saved, ws)
            f8.linear_bwd(desc, dY.cuda(), saved, dX, dW, ws)
        torch.cuda.synchronize()
        outs.append((Y, dX, dW, saved.x.q, codes_t(saved.dy)))
    for a, b in zip(*outs):
        assert torch.equal(a, b)


def test_scaled_argument_errors():
    M = K = N = 64
    desc = f8.linear_desc(M, K, N, True, f8.E4M3)        # rowwise is not a delayed mode
    st = f8.ScalingState(f8.DELAYED, 4)
    saved = f8.Saved(M, K, N, True)
    ws = f8.new_workspace(64, 64)
    t = torch.zeros((64, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(f8.F8Error) as e:
        f8.linear_fwd_scaled(desc, st, t, t, t.clone(), saved, ws)
    assert e.value.code == 4
    bad = f8.ScalingState(f8.DELAYED, 4)
    bad._struct.history_len = 0
    with pytest.raises(f8.F8Error) as e:
        f8.linear_fwd_scaled(f8.linear_desc(M, K, N), bad, t, t, t.clone(), f8.Saved(M, K, N), ws)
    assert e.value.code == 2
    hist = torch.zeros(4, device="cuda")
    with pytest.raises(f8.F8Error) as e:   # history longer than F8_MAX_HISTORY
        f8._check(f8.lib().f8_amax_history_push(hist.data_ptr(), 2000, hist.data_ptr(), 0, hist.data_ptr(), None, None))
    assert e.value.code == 2


def test_full_size_delayed_linear():
    """The 8B wq linear at M = 8192 under delayed scaling: seed with the first batch, then a
    second batch with twice the activation scale (stale window: saturation in X)."""
    w = wl.WORKLOADS["llama8b"]
    X0, W, dY0 = wl.make_linear_inputs(w, 0)
    X1, _, dY1 = wl.make_linear_inputs(w, 3)               # wo: same shapes, other seeds
    X1 = (X1.float() * 2.0).to(torch.bfloat16)
    lin = w.linears[0]
    M, K, N = lin.M, lin.K, lin.N
    desc = f8.linear_desc(M, K, N, False, f8.E4M3)
    saved = f8.Saved(M, K, N, False)
    ws = f8.new_workspace(max(M, K, N), max(M, K, N))
    st, st_ref = f8.ScalingState(f8.DELAYED, 16), o.ScalingState(o.DELAYED, 16)
    _seed(st, st_ref, X0, W, dY0, f8.E4M3, ws)
    Y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    dX = torch.empty((M, K), dtype=torch.bfloat16, device="cuda")
    dW = torch.empty((N, K), dtype=torch.bfloat16, device="cuda")
    rng = np.random.default_rng(0)
    for X, dY in ((X0, dY0), (X1, dY1)):
        f8.linear_fwd_scaled(desc, st, X.cuda(), W.cuda(), Y, saved, ws)
        f8.linear_bwd_scaled(desc, st, dY.cuda(), saved, dX, dW, ws)
        torch.cuda.synchronize()
        qs = {}
        for key, t, q in (("x", X, saved.x), ("w", W, saved.w), ("dy", dY, saved.dy)):
            tb = bits(t)
            s = st_ref.scale[key].copy()
            codes = o.cast(tb, s, o.TENSORWISE, o.E4M3)
            a = o.amax(tb)
            st_ref.scale[key], _ = o.history_push(st_ref.hist[key], a[0], o.E4M3)
            assert np.array_equal(u8(q.q), codes) and qt_matches(q, codes.T)
            assert f32(q.amax)[0] == a[0] and f32(q.scale)[0] == s[0]
            assert f32(getattr(st, "scale_" + key))[0] == st_ref.scale[key][0]
            qs[key] = (codes, np.float32(1.0) / s)
        (qx, isx), (qw, isw), (qdy, isdy) = qs["x"], qs["w"], qs["dy"]
        sampled_check("Y", bits(Y), o.NT, qx, o.E4M3, qw, o.E4M3, isx, isw, o.TENSORWISE, rng)
        sampled_check("dX", bits(dX), o.NN, qdy, o.E4M3, qw, o.E4M3, isdy, isw, o.TENSORWISE, rng)
        sampled_check("dW", bits(dW), o.TN, qdy, o.E4M3, qx, o.E4M3, isdy, isx, o.TENSORWISE, rng)
    assert (u8(saved.x.q) & 0x7F).max() == 0x7E             # the doubled batch saturated
