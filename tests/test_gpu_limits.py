"""The largest sizes the interface admits (dimensions below 2^23), one dimension at a time."""
import numpy as np
import pytest
import torch

import oracle as o
from paper_2410_06511_amd import f8
from helpers import bits, u8, f32, assert_gemm_close

pytestmark = pytest.mark.gpu

BIG = (1 << 23) - 256       # the largest multiple of 256 below 2^23
BIG16 = (1 << 23) - 16      # the largest multiple of 16 below 2^23


def _codes(rng, shape):
    c = rng.integers(0, 0x58, shape, dtype=np.uint8)            # magnitudes up to 1.0 * 2^3
    return c | (rng.integers(0, 2, shape, dtype=np.uint8) << 7)


@pytest.mark.parametrize("M,N,K", [(16, 16, BIG), (BIG16, 16, 16), (16, BIG16, 16), (BIG16, 16, 256)])
def test_gemm_at_the_size_limits(M, N, K):
    """Longest contraction (fast kernel, 65534 K steps on one tile), most rows and most columns
    (generic kernel: one block per 64x64 tile in a one-dimensional grid; fast kernel for K = 256)."""
    rng = np.random.default_rng(K % 1000 + M % 7)
    A, B = _codes(rng, (M, K)), _codes(rng, (N, K))
    isa = isb = np.float32(2.0 ** -4)
    D = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    s = torch.from_numpy(np.array([isa], np.float32)).cuda()
    f8.gemm(f8.NT, M, N, K, torch.from_numpy(A).cuda(), o.E4M3, torch.from_numpy(B).cuda(), o.E4M3, s, s, f8.TENSORWISE, D)
    torch.cuda.synchronize()
    assert_gemm_close(bits(D), o.gemm(o.NT, A, o.E4M3, B, o.E4M3, isa, isb), (M, N, K))


@pytest.mark.parametrize("rows,cols", [(BIG16, 16), (16, BIG16)])
def test_quantise_at_the_size_limits(rows, cols):
    g = torch.Generator("cpu")
    g.manual_seed(rows % 97)
    x = (torch.randn((rows, cols), generator=g) * 2).to(torch.bfloat16)
    q = f8.QTensor(rows, cols, False, transposed=True)
    ws = f8.new_workspace(rows, cols)
    f8.quantise(x.cuda(), f8.TENSORWISE, f8.E4M3, q, ws)
    torch.cuda.synchronize()
    a, s, inv, codes = o.amax_cast(bits(x), o.TENSORWISE, o.E4M3)
    assert f32(q.amax)[0] == a[0] and f32(q.scale)[0] == s[0]
    assert np.array_equal(u8(q.q), codes) and np.array_equal(u8(q.q_t), codes.T)


def test_sizes_beyond_the_limit_are_refused():
    t = torch.zeros((16, 16), dtype=torch.uint8, device="cuda")
    one = torch.ones(1, device="cuda")
    D = torch.zeros((16, 16), dtype=torch.bfloat16, device="cuda")
    code = f8.lib().f8_gemm(0, 1 << 23, 16, 16, t.data_ptr(), 0, 16, t.data_ptr(), 0, 16, one.data_ptr(), one.data_ptr(), 0,
                            D.data_ptr(), 16, None, None)
    assert code == 2
