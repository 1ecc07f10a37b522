"""Shared pieces of the GPU parity tests: moving seeded inputs to the device and
comparing GEMM results with the oracle under the stated tolerances."""
import numpy as np
import torch

import oracle as o

# Tolerance of the GEMM outputs (stated by the benchmark spec): max-abs error relative to the max-abs
# of the fp32-accumulating oracle, on identical fp8 inputs and scales.
GEMM_REL_TOL = 1e-2


def dev(t):
    return t.cuda()


def bits(t):
    """bf16 tensor (any device) -> numpy uint16 bits."""
    return t.detach().cpu().contiguous().view(torch.uint16).numpy()


def u8(t):
    return t.detach().cpu().contiguous().numpy()


def f32(t):
    return t.detach().cpu().contiguous().numpy()


def qt_matches(q, expect_t):
    """The transposed code tensor of a QTensor equals expect_t (numpy), when there is one."""
    return q.q_t is None or np.array_equal(u8(q.q_t), expect_t)


def codes_t(q):
    """The tensor to snapshot for a QTensor's second orientation (q itself if it keeps none)."""
    return q.q if q.q_t is None else q.q_t


def bf16_from_f32(a):
    return torch.from_numpy(np.asarray(a, dtype=np.float32)).to(torch.bfloat16)


def assert_gemm_close(got_bits, ref_bits, what=""):
    got = o.bf16_to_f32(got_bits).astype(np.float64)
    ref = o.bf16_to_f32(ref_bits).astype(np.float64)
    assert np.isfinite(got).all(), what
    denom = np.abs(ref).max()
    err = np.abs(got - ref).max()
    assert err <= GEMM_REL_TOL * max(denom, 1e-30), (what, err, denom)
    return err / max(denom, 1e-30)


# The fp8 matrix cores add the products of 8 consecutive k (an aligned group) after aligning them
# to the group's largest product and keeping 13 bits below it; different groups and different
# matrix instructions add as full fp32.  tests/test_gpu_mfma_numerics.py pins both numbers on
# the chip.  A product therefore loses less than 2^-13 of its group's largest product (cut off,
# or dropped whole when it lies further below), a group of 8 less than 2^-10 of it.
MFMA_GROUP = 8
MFMA_KEPT_BITS = 13


def group_max_sum(layout, A, fa, B, fb, isa, isb, rowwise=False):
    """sum over the aligned groups of 8 consecutive k of max_k |a||b| (times the scales), per
    output element: what the matrix core's in-group alignment error is proportional to."""
    a, b = np.abs(o.decode(A, fa).astype(np.float64)), np.abs(o.decode(B, fb).astype(np.float64))
    if layout == o.TN:
        a = a.T                                  # [M, K]
    if layout != o.NT:
        b = b.T                                  # [N, K]
    M, K = a.shape
    N = b.shape[0]
    out = np.zeros((M, N))
    for k0 in range(0, K, MFMA_GROUP):
        g = np.zeros((M, N))
        for k in range(k0, min(k0 + MFMA_GROUP, K)):
            np.maximum(g, np.outer(a[:, k], b[:, k]), out=g)
        out += g
    sa, sb = np.atleast_1d(isa).astype(np.float64), np.atleast_1d(isb).astype(np.float64)
    return out * (sa[:, None] * sb[None, :] if rowwise else sa[0] * sb[0])


def assert_gemm_tight(got_bits, d64, dabs, K, what="", gmax=None):
    """Per element against the unrounded fp64 result: one bf16 rounding, the matrix core's
    in-group alignment loss (MFMA_GROUP products, each short of at most 2^-MFMA_KEPT_BITS of the
    group's largest: gmax = group_max_sum(...); without it the cruder sum |a||b| stands in, which
    is never smaller) and the fp32 additions between groups."""
    got = o.bf16_to_f32(got_bits).astype(np.float64)
    align = MFMA_GROUP * 2.0 ** -MFMA_KEPT_BITS * (dabs if gmax is None else gmax)
    bound = 2.0 ** -8 * np.abs(d64) * (1 + 2.0 ** -7) + align + 2.0 * K * 2.0 ** -24 * dabs + 1e-38
    bad = np.abs(got - d64) > bound
    assert not bad.any(), (what, int(bad.sum()), np.argwhere(bad)[:4])


def sample_lines(n_lines, rng, n=64, tile=256):
    """Indices of whole output rows (or columns) to compare: n seeded random ones, the first
    and the last, and both sides of the first, the last and three random 256-tile boundaries."""
    picks = set(rng.integers(0, n_lines, n).tolist()) | {0, n_lines - 1}
    nb = (n_lines - 1) // tile  # boundaries at tile, 2 * tile, ..., nb * tile
    if nb >= 1:
        for t in {1, nb} | set(rng.integers(1, nb + 1, 3).tolist()):
            picks |= {t * tile - 1, t * tile}
    return sorted(picks)


def sampled_check(name, got, layout, A, fa, B, fb, isa, isb, g, rng):
    M, N = got.shape
    rows, cols = sample_lines(M, rng), sample_lines(N, rng)
    ms, ns = np.repeat(rows, N), np.tile(np.arange(N), len(rows))
    assert_gemm_close(got[ms, ns], o.gemm_points(layout, A, fa, B, fb, isa, isb, ms, ns, g), name + " rows")
    ns, ms = np.repeat(cols, M), np.tile(np.arange(M), len(cols))
    assert_gemm_close(got[ms, ns], o.gemm_points(layout, A, fa, B, fb, isa, isb, ms, ns, g), name + " cols")
