"""What "fp32 accumulation" means inside the chip's fp8 matrix instructions, pinned through
f8_gemm: the products of 8 consecutive k are aligned to the largest of them and 13 bits below it
are kept; groups, and successive instructions, add as full fp32.  The per-element bound of the GEMM
tests (helpers.assert_gemm_tight) is derived from exactly these two numbers."""
import numpy as np
import pytest

import oracle as o
from paper_2410_06511_amd import f8
from helpers import MFMA_GROUP, MFMA_KEPT_BITS
from test_gpu_gemm import run_gemm

pytestmark = pytest.mark.gpu

E5 = o.E5M2   # the wide-exponent format: products from 2^-28 to 2^30


def _code(v):
    return int(o.encode(np.array([v], np.float32), E5)[0])


def _product(K, terms):
    """D[3, 5] of a 32 x 32 x K product whose only nonzero columns k are terms = [(k, a, b)]."""
    A, B = np.zeros((32, K), np.uint8), np.zeros((32, K), np.uint8)
    for k, av, bv in terms:
        A[:, k], B[:, k] = _code(av), _code(bv)
    got = run_gemm(f8.NT, 32, 32, K, A, E5, B, E5, np.float32(1), np.float32(1), f8.TENSORWISE)
    return float(o.bf16_to_f32(got)[3, 5])


def _split(e):
    """Two powers of two whose product is 2^e, both representable."""
    ea = e // 2
    return 2.0 ** ea, 2.0 ** (e - ea)


# K = 256 runs on the tiled kernel (16x16x128 instructions), K = 32 on the generic one (16x16x32)
@pytest.mark.parametrize("K", [256, 32])
def test_products_of_eight_consecutive_k_are_aligned_together(K):
    """+2^14 at k = 0 and -2^14 at a neighbour cancel exactly; a term 2^-2 (16 bits below) at k1
    survives exactly when k1 is not among the 8 consecutive k that hold the big pair."""
    for k1 in range(1, min(K, 48)):
        k2 = 1 if k1 != 1 else 2
        v = _product(K, [(0, 2.0 ** 7, 2.0 ** 7), (k1, 2.0 ** -1, 2.0 ** -1), (k2, -2.0 ** 7, 2.0 ** 7)])
        assert v == (0.0 if k1 < MFMA_GROUP else 2.0 ** -2), (K, k1, v)
    # the groups are aligned: k = 8 .. 15 form the next one
    v = _product(K, [(8, 2.0 ** 7, 2.0 ** 7), (15, 2.0 ** -1, 2.0 ** -1), (9, -2.0 ** 7, 2.0 ** 7)])
    assert v == 0.0
    v = _product(K, [(8, 2.0 ** 7, 2.0 ** 7), (7, 2.0 ** -1, 2.0 ** -1), (9, -2.0 ** 7, 2.0 ** 7)])
    assert v == 2.0 ** -2


@pytest.mark.parametrize("K", [256, 32])
def test_thirteen_bits_below_the_group_maximum_are_kept(K):
    """Inside a group a term survives down to 2^-13 of the largest product and is dropped from
    2^-14 on; in another group it survives at any distance fp32 can hold."""
    far = 24 if K == 32 else 200
    for gap in range(8, 24):
        a, b = _split(14 - gap)
        inside = _product(K, [(0, 2.0 ** 7, 2.0 ** 7), (2, a, b), (1, -2.0 ** 7, 2.0 ** 7)])
        assert inside == (2.0 ** (14 - gap) if gap <= MFMA_KEPT_BITS else 0.0), (K, gap, inside)
        outside = _product(K, [(0, 2.0 ** 7, 2.0 ** 7), (far, a, b), (1, -2.0 ** 7, 2.0 ** 7)])
        assert outside == 2.0 ** (14 - gap), (K, gap, outside)


def test_a_cut_term_loses_less_than_one_unit_at_the_thirteenth_bit():
    """A term that straddles the cut (1.75 * 2^-12 below a maximum of 2^14, i.e. bits at 2^-12,
    2^-13 and 2^-14 relative) comes through short by less than 2^-13 of the maximum."""
    big = 2.0 ** 14
    v = _product(256, [(0, 2.0 ** 7, 2.0 ** 7), (2, 1.75, 2.0 ** 2), (1, -2.0 ** 7, 2.0 ** 7)])   # 7 = 1.75 * 2^2
    assert 0.0 <= 7.0 - v < big * 2.0 ** -MFMA_KEPT_BITS
