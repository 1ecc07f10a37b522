"""f8_linear_fwd_noalloc (the forward on the library's built-in scratch, for callers that cannot
allocate) against f8_linear_fwd with a caller's workspace: same bits, on two calls in a row, the
second with a smaller input; shapes beyond the scratch are refused before any launch."""
import ctypes as C

import pytest
import torch

from paper_2410_06511_amd import f8
from paper_2410_06511_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _inputs(M, K, N, seed):
    g = torch.Generator("cpu")
    g.manual_seed(seed)
    return wl.randn_bf16((M, K), 1.0, 0, generator=g).cuda(), wl.randn_bf16((N, K), 0.02, 0, generator=g).cuda()


def _same(a, b):
    return torch.equal(a.view(torch.uint8), b.view(torch.uint8))


@pytest.mark.parametrize("rowwise", [False, True])
def test_noalloc_forward_equals_forward_with_workspace(rowwise):
    # first a shape with several tiles and ragged edges in every kernel, then a smaller one: the
    # second call finds the first call's partial maxima in the scratch and must not be fooled by them
    for M, K, N in ((1040, 768, 1296), (272, 336, 208)):
        X, W = _inputs(M, K, N, M + K + N)
        desc = f8.linear_desc(M, K, N, rowwise)
        ws = f8.new_workspace(max(M, K, N), max(M, K, N))
        ref, got = f8.Saved(M, K, N, rowwise), f8.Saved(M, K, N, rowwise)
        Yref = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        Y = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
        f8.linear_fwd(desc, X, W, Yref, ref, ws)
        f8.linear_fwd_noalloc(desc, X, W, Y, got)
        torch.cuda.synchronize()
        assert _same(Y, Yref)
        for a, b in ((got.x, ref.x), (got.w, ref.w)):
            assert _same(a.q, b.q) and _same(a.amax, b.amax) and _same(a.scale, b.scale) and _same(a.inv_scale, b.inv_scale)
            if rowwise:
                assert _same(a.q_t, b.q_t) and _same(a.amax_t, b.amax_t) and _same(a.scale_t, b.scale_t)
                assert _same(a.inv_scale_t, b.inv_scale_t)


def test_noalloc_forward_refuses_shapes_beyond_its_scratch():
    # rowwise partial maxima of a tensor with 32784 columns need 64 * 32784 * 4 bytes > 8 MiB
    M, K, N = 16, 32784, 16
    assert 64 * K * 4 > 8 << 20
    X, W = _inputs(M, K, N, 3)
    saved = f8.Saved(M, K, N, True)
    Y = torch.full((M, N), 7.0, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(f8.F8Error) as e:
        f8.linear_fwd_noalloc(f8.linear_desc(M, K, N, True), X, W, Y, saved)
    torch.cuda.synchronize()
    assert e.value.code == 5 and bool((Y == 7.0).all())
    # the same shape under tensorwise scaling fits
    f8.linear_fwd_noalloc(f8.linear_desc(M, K, N), X, W, Y, f8.Saved(M, K, N))
    torch.cuda.synchronize()
    assert bool(torch.isfinite(Y.float()).all())
