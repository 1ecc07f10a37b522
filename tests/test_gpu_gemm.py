"""GPU parity of the fp8 GEMMs (steps 4-6) against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle as o
from paper_2410_06511_amd import f8
from helpers import bits, u8, assert_gemm_close, assert_gemm_tight, group_max_sum

pytestmark = pytest.mark.gpu


def finite_codes(fmt):
    if fmt == o.E4M3:
        return np.array([c for c in range(256) if (c & 0x7F) != 0x7F], np.uint8)
    return np.array([c for c in range(256) if (c & 0x7F) < 0x7C], np.uint8)


def rand_codes(rng, shape, fmt, moderate=True):
    fc = finite_codes(fmt)
    c = fc[rng.integers(0, fc.size, shape)]
    if moderate:
        c = (c & 0xDF).astype(np.uint8)      # clear the top exponent bit: no fp32 overflow in long sums
    return c


def shapes_of(layout, M, N, K):
    sa = (K, M) if layout == o.TN else (M, K)
    sb = (N, K) if layout == o.NT else (K, N)
    return sa, sb


def run_gemm(layout, M, N, K, A, fa, B, fb, isa, isb, g, workspace=None):
    Ad, Bd = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    sa = torch.from_numpy(np.atleast_1d(isa).astype(np.float32)).cuda()
    sb = torch.from_numpy(np.atleast_1d(isb).astype(np.float32)).cuda()
    D = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    f8.gemm(layout, M, N, K, Ad, fa, Bd, fb, sa, sb, g, D, workspace=workspace)
    if workspace is not None:
        torch.cuda.synchronize()
        return bits(D)
    # the same product with the output amax taken in the epilogue: identical D, and the amax
    # is exactly the largest magnitude among the stored bf16 values
    D2 = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    amax = torch.full((1,), -1.0, device="cuda")
    f8.gemm(layout, M, N, K, Ad, fa, Bd, fb, sa, sb, g, D2, amax_d=amax)
    torch.cuda.synchronize()
    assert torch.equal(D.view(torch.int16), D2.view(torch.int16))
    assert amax.item() == o.amax(bits(D2))[0]
    return bits(D)


# (M, N, K): single tile; several 64- and 256-tiles with ragged M and N; K not a multiple of
# 64 (generic kernel even for NT); K a multiple of 64 but not 256 (tail steps of the fast
# kernel); a shape that takes the 256x256 tiles with ragged edges.
SMALL = [(16, 16, 16), (64, 64, 64), (80, 144, 208), (272, 400, 192), (144, 80, 576), (528, 784, 256)]


@pytest.mark.parametrize("layout", [o.NT, o.NN, o.TN])
@pytest.mark.parametrize("fa,fb", [(o.E4M3, o.E4M3), (o.E5M2, o.E4M3), (o.E4M3, o.E5M2), (o.E5M2, o.E5M2)])
@pytest.mark.parametrize("M,N,K", SMALL)
def test_gemm_small_full_compare(layout, fa, fb, M, N, K):
    rng = np.random.default_rng(M + 3 * N + 7 * K + layout)
    sa, sb = shapes_of(layout, M, N, K)
    A, B = rand_codes(rng, sa, fa), rand_codes(rng, sb, fb)
    isa, isb = np.float32(0.0131), np.float32(0.73)
    got = run_gemm(layout, M, N, K, A, fa, B, fb, isa, isb, f8.TENSORWISE)
    ref = o.gemm(layout, A, fa, B, fb, isa, isb)
    assert_gemm_close(got, ref, (layout, fa, fb, M, N, K))
    d64, dabs = o.gemm_f64(layout, A, fa, B, fb, isa, isb)
    assert_gemm_tight(got, d64, dabs, K, (layout, fa, fb, M, N, K), group_max_sum(layout, A, fa, B, fb, isa, isb))


@pytest.mark.parametrize("layout", [o.NT, o.NN, o.TN])
@pytest.mark.parametrize("M,N,K", [(80, 144, 208), (272, 400, 256)])
def test_gemm_rowwise_scales(layout, M, N, K):
    rng = np.random.default_rng(11 + layout)
    sa, sb = shapes_of(layout, M, N, K)
    A, B = rand_codes(rng, sa, o.E4M3), rand_codes(rng, sb, o.E4M3)
    isa = (rng.uniform(0.5, 2.0, M) * 1e-2).astype(np.float32)
    isb = (rng.uniform(0.5, 2.0, N) * 1e-1).astype(np.float32)
    got = run_gemm(layout, M, N, K, A, o.E4M3, B, o.E4M3, isa, isb, f8.ROWWISE)
    d64, dabs = o.gemm_f64(layout, A, o.E4M3, B, o.E4M3, isa, isb, o.ROWWISE)
    assert_gemm_tight(got, d64, dabs, K, (layout, M, N, K), group_max_sum(layout, A, o.E4M3, B, o.E4M3, isa, isb, True))
    assert_gemm_close(got, o.gemm(layout, A, o.E4M3, B, o.E4M3, isa, isb, o.ROWWISE))


@pytest.mark.parametrize("layout", [o.NT, o.NN, o.TN])
@pytest.mark.parametrize("M,N,K", [(272, 400, 320), (512, 768, 1024)])
def test_gemm_exact_arithmetic_bit_for_bit(layout, M, N, K):
    """Operands on a grid where every partial sum is exact in fp32 in any order: codes of
    {0, +-64, +-128, +-256, +-448} and scales 2^-7.  GPU, oracle and the fp64 closed form must
    agree bit for bit: a tile-indexing and operand-layout test with zero tolerance."""
    rng = np.random.default_rng(21 + layout)
    vals = np.array([0, 64, -64, 128, -128, 256, -256, 448, -448], np.float32)
    grid = o.encode(vals, o.E4M3)
    sa, sb = shapes_of(layout, M, N, K)
    A, B = grid[rng.integers(0, 9, sa)], grid[rng.integers(0, 9, sb)]
    inv = np.float32(2.0 ** -7)
    got = run_gemm(layout, M, N, K, A, o.E4M3, B, o.E4M3, inv, inv, f8.TENSORWISE)
    a = o.decode(A, o.E4M3).astype(np.float64)
    b = o.decode(B, o.E4M3).astype(np.float64)
    exact = {o.NT: lambda: a @ b.T, o.NN: lambda: a @ b, o.TN: lambda: a.T @ b}[layout]() * 2.0 ** -14
    closed = torch.from_numpy(exact).to(torch.bfloat16).view(torch.uint16).numpy()
    assert np.array_equal(got, closed)
    assert np.array_equal(got, o.gemm(layout, A, o.E4M3, B, o.E4M3, inv, inv))


# More tiles than compute units, so that persistent workgroups walk several tiles (the load
# stream runs across tile boundaries) and the two-launch dispatch is taken: 8192 x 4096 = 512
# tiles of 256 x 256 (two rounds); 14336 x 4096 = 896 tiles = 3.5 rounds (whole rounds on a range
# of tile rows, the rest as 256 x 128 tiles); 4096 x 14336 likewise on a range of tile columns.
@pytest.mark.parametrize("layout", [o.NT, o.NN, o.TN])
@pytest.mark.parametrize("g", [f8.TENSORWISE, f8.ROWWISE])
@pytest.mark.parametrize("M,N,K", [(8192, 4096, 1024), (14336, 4096, 512), (4096, 14336, 512)])
def test_gemm_exact_arithmetic_multi_round(layout, g, M, N, K):
    """The exact-arithmetic grid (see above) at sizes where a workgroup computes several tiles:
    bit for bit against the fp64 product rounded once to bf16, scales powers of two (one per
    tensor, or one per row and per column)."""
    rng = np.random.default_rng(77 + layout + M)
    vals = np.array([0, 64, -64, 128, -128, 256, -256, 448, -448], np.float32)
    grid = o.encode(vals, o.E4M3)
    sa, sb = shapes_of(layout, M, N, K)
    A, B = grid[rng.integers(0, 9, sa)], grid[rng.integers(0, 9, sb)]
    if g == f8.TENSORWISE:
        isa, isb = np.float32(2.0 ** -7), np.float32(2.0 ** -6)
        sc = np.float64(2.0 ** -13)
    else:
        isa = (2.0 ** -(5.0 + (np.arange(M) % 4))).astype(np.float32)
        isb = (2.0 ** -(6.0 + (np.arange(N) % 3))).astype(np.float32)
        sc = isa.astype(np.float64)[:, None] * isb.astype(np.float64)[None, :]
    got = run_gemm(layout, M, N, K, A, o.E4M3, B, o.E4M3, isa, isb, g)
    a = torch.from_numpy(o.decode(A, o.E4M3).astype(np.float64))
    b = torch.from_numpy(o.decode(B, o.E4M3).astype(np.float64))
    exact = {o.NT: lambda: a @ b.T, o.NN: lambda: a @ b, o.TN: lambda: a.T @ b}[layout]() * torch.from_numpy(np.asarray(sc))
    closed = exact.to(torch.bfloat16).view(torch.uint16).numpy()
    assert np.array_equal(got, closed)


def test_gemm_exact_arithmetic_long_contraction():
    """The same grid with the 8B forward shape's contraction length (every sum still below 2^30
    in units of 2^12): the full-size launch configuration, zero tolerance."""
    rng = np.random.default_rng(5)
    M, N, K = 8192, 4096, 4096
    vals = np.array([0, 64, -64, 128, -128, 256, -256, 448, -448], np.float32)
    grid = o.encode(vals, o.E4M3)
    A, B = grid[rng.integers(0, 9, (M, K))], grid[rng.integers(0, 9, (K, N))]
    inv = np.float32(2.0 ** -7)
    got = run_gemm(o.NN, M, N, K, A, o.E4M3, B, o.E4M3, inv, inv, f8.TENSORWISE)
    a = torch.from_numpy(o.decode(A, o.E4M3).astype(np.float64))
    b = torch.from_numpy(o.decode(B, o.E4M3).astype(np.float64))
    closed = ((a @ b) * 2.0 ** -14).to(torch.bfloat16).view(torch.uint16).numpy()
    assert np.array_equal(got, closed)


@pytest.mark.parametrize("layout", [o.NT, o.NN, o.TN])
@pytest.mark.parametrize("g", [f8.TENSORWISE, f8.ROWWISE])
@pytest.mark.parametrize("M,N,K", [(512, 1024, 4096), (272, 400, 2048), (2048, 4096, 8192)])
def test_gemm_split_contraction_exact_arithmetic(layout, g, M, N, K):
    """f8_gemm_ws on products with few output tiles and a long contraction (8, 4 and 128 tiles of
    256 x 256): computed in contraction ranges whose fp32 sums a second kernel adds.  On the
    exact-arithmetic grid every partial sum is exact, so the result is bit for bit the fp64
    product rounded once to bf16 - and equal to the unsplit f8_gemm."""
    rng = np.random.default_rng(13 + layout + M)
    vals = np.array([0, 64, -64, 128, -128, 256, -256, 448, -448], np.float32)
    grid = o.encode(vals, o.E4M3)
    sa, sb = shapes_of(layout, M, N, K)
    A, B = grid[rng.integers(0, 9, sa)], grid[rng.integers(0, 9, sb)]
    if g == f8.TENSORWISE:
        isa, isb = np.float32(2.0 ** -7), np.float32(2.0 ** -6)
        sc = np.float64(2.0 ** -13)
    else:
        isa = (2.0 ** -(5.0 + (np.arange(M) % 4))).astype(np.float32)
        isb = (2.0 ** -(6.0 + (np.arange(N) % 3))).astype(np.float32)
        sc = isa.astype(np.float64)[:, None] * isb.astype(np.float64)[None, :]
    ws = f8.new_workspace(M, N)
    got = run_gemm(layout, M, N, K, A, o.E4M3, B, o.E4M3, isa, isb, g, workspace=ws)
    a = torch.from_numpy(o.decode(A, o.E4M3).astype(np.float64))
    b = torch.from_numpy(o.decode(B, o.E4M3).astype(np.float64))
    exact = {o.NT: lambda: a @ b.T, o.NN: lambda: a @ b, o.TN: lambda: a.T @ b}[layout]() * torch.from_numpy(np.asarray(sc))
    assert np.array_equal(got, exact.to(torch.bfloat16).view(torch.uint16).numpy())
    assert np.array_equal(got, run_gemm(layout, M, N, K, A, o.E4M3, B, o.E4M3, isa, isb, g))


@pytest.mark.parametrize("layout,fa,fb", [(o.TN, o.E5M2, o.E4M3), (o.NT, o.E4M3, o.E4M3), (o.NN, o.E4M3, o.E5M2)])
def test_gemm_split_contraction_random_codes(layout, fa, fb):
    """Random codes: the split product against the oracle and the fp64 bound element by element,
    deterministic over repeated calls, and a workspace too small for the partial sums gives the
    unsplit product's bits."""
    M, N, K = 1024, 528, 4096
    rng = np.random.default_rng(layout + 400)
    sa, sb = shapes_of(layout, M, N, K)
    A, B = rand_codes(rng, sa, fa), rand_codes(rng, sb, fb)
    isa, isb = np.float32(0.0131), np.float32(0.73)
    ws = f8.new_workspace(M, N)
    got = run_gemm(layout, M, N, K, A, fa, B, fb, isa, isb, f8.TENSORWISE, workspace=ws)
    assert_gemm_close(got, o.gemm(layout, A, fa, B, fb, isa, isb), (layout, fa, fb))
    d64, dabs = o.gemm_f64(layout, A, fa, B, fb, isa, isb)
    assert_gemm_tight(got, d64, dabs, K, (layout, fa, fb), group_max_sum(layout, A, fa, B, fb, isa, isb))
    for _ in range(2):
        assert np.array_equal(got, run_gemm(layout, M, N, K, A, fa, B, fb, isa, isb, f8.TENSORWISE, workspace=ws))
    small = torch.empty(4096, dtype=torch.uint8, device="cuda")
    unsplit = run_gemm(layout, M, N, K, A, fa, B, fb, isa, isb, f8.TENSORWISE)
    assert np.array_equal(unsplit, run_gemm(layout, M, N, K, A, fa, B, fb, isa, isb, f8.TENSORWISE, workspace=small))


def test_gemm_output_guard_band_and_ldd():
    """D with a leading dimension larger than N: columns beyond N stay untouched."""
    rng = np.random.default_rng(5)
    M, N, K, ldd = 272, 400, 256, 512
    A, B = rand_codes(rng, (M, K), o.E4M3), rand_codes(rng, (N, K), o.E4M3)
    Ad, Bd = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    one = torch.ones(1, dtype=torch.float32, device="cuda")
    buf = torch.full((M + 2, ldd), -7.0, dtype=torch.bfloat16, device="cuda")
    D = buf[1:M + 1, :N]                        # a view with stride ldd, 16-byte aligned (ldd*2*1 bytes offset)
    f8.gemm(f8.NT, M, N, K, Ad, o.E4M3, Bd, o.E4M3, one, one, f8.TENSORWISE, D)
    torch.cuda.synchronize()
    assert bool((buf[0] == -7).all()) and bool((buf[M + 1] == -7).all()) and bool((buf[1:M + 1, N:] == -7).all())
    assert_gemm_close(bits(D.contiguous()), o.gemm(o.NT, A, o.E4M3, B, o.E4M3, np.float32(1), np.float32(1)))


def sample_points(rng, M, N, tile=256, nrows=64, ncols=64):
    """>= 64 full rows and columns plus the first / last row and column of every tile boundary."""
    rows = set(rng.integers(0, M, nrows).tolist())
    cols = set(rng.integers(0, N, ncols).tolist())
    for t in range(0, M, tile):
        rows.update([t, min(t + tile, M) - 1])
    for t in range(0, N, tile):
        cols.update([t, min(t + tile, N) - 1])
    return sorted(rows), sorted(cols)


@pytest.mark.parametrize("M,N,K", [(8192, 4096, 4096), (8192, 1024, 4096), (4096, 14336, 8192)])
def test_gemm_llama_shapes_sampled(M, N, K):
    """Full-size GEMMs of the 8B workload (forward wq / wk shapes, and a dW-like shape with a
    long contraction) in the launch configuration the benchmark uses; the oracle computes
    whole sampled rows and columns one by one."""
    rng = np.random.default_rng(M + N + K)
    A = rand_codes(rng, (M, K), o.E4M3)
    B = rand_codes(rng, (N, K), o.E4M3)
    isa, isb = np.float32(1 / 97.0), np.float32(1 / 5120.0)
    got = run_gemm(f8.NT, M, N, K, A, o.E4M3, B, o.E4M3, isa, isb, f8.TENSORWISE)
    rows, cols = sample_points(rng, M, N, nrows=8, ncols=8)
    rows, cols = rows[::4], cols[::4]           # keep the CPU side to seconds
    ms = np.repeat(rows, N)
    ns = np.tile(np.arange(N), len(rows))
    ref = o.gemm_points(o.NT, A, o.E4M3, B, o.E4M3, isa, isb, ms, ns)
    assert_gemm_close(got[ms, ns], ref, "rows")
    ns = np.repeat(cols, M)
    ms = np.tile(np.arange(M), len(cols))
    ref = o.gemm_points(o.NT, A, o.E4M3, B, o.E4M3, isa, isb, ms, ns)
    assert_gemm_close(got[ms, ns], ref, "cols")
    assert np.isfinite(o.bf16_to_f32(got)).all()


def test_gemm_output_amax_full_size_and_oracle():
    """8B wk forward shape: the epilogue amax equals the amax of the stored output exactly and the
    oracle's amax of its own output within the GEMM tolerance."""
    rng = np.random.default_rng(12)
    M, N, K = 2048, 1024, 4096
    A, B = rand_codes(rng, (M, K), o.E4M3), rand_codes(rng, (N, K), o.E4M3)
    isa, isb = np.float32(2.0 ** -6), np.float32(2.0 ** -5)
    got = run_gemm(o.NT, M, N, K, A, o.E4M3, B, o.E4M3, isa, isb, o.TENSORWISE)   # checks exactness
    rows = np.arange(0, M, 16)
    ms, ns = np.repeat(rows, N), np.tile(np.arange(N), len(rows))
    ref = o.gemm_points(o.NT, A, o.E4M3, B, o.E4M3, np.array([isa]), np.array([isb]), ms, ns, o.TENSORWISE)
    a_got = o.amax(got[rows])[0]
    a_ref = o.amax(ref.reshape(len(rows), N))[0]
    assert abs(a_got - a_ref) <= 1e-2 * a_ref


def test_gemm_amax_of_empty_output_is_zero():
    one = torch.ones(1, device="cuda")
    buf = torch.zeros((16, 16), dtype=torch.uint8, device="cuda")
    D = torch.zeros((16, 16), dtype=torch.bfloat16, device="cuda")
    amax = torch.full((1,), 3.0, device="cuda")
    code = f8.lib().f8_gemm(0, 0, 16, 16, buf.data_ptr(), 0, 16, buf.data_ptr(), 0, 16, one.data_ptr(), one.data_ptr(),
                            0, D.data_ptr(), 16, amax.data_ptr(), None)
    torch.cuda.synchronize()
    assert code == 0 and amax.item() == 0.0


# Ragged shapes large enough to be dispatched to each tile configuration of the fast kernel
# (which one is chosen depends on how many tiles the shape has against the number of compute
# units): 256x256 tiles with a ragged last tile row and column, 256x128 tiles likewise, and
# shapes whose edges are narrower than one MFMA tile.  Compared in full.
@pytest.mark.parametrize("g", [f8.TENSORWISE, f8.ROWWISE])
# The last two have a partial last round of 256x256 tiles (18 x 16 and 16 x 18 tiles on 256 compute
# units): the whole rounds run on a sub-matrix, the remaining tile rows / tile columns as a
# second launch with 256x128 tiles, ragged edge included.
@pytest.mark.parametrize("M,N,K", [(4112, 4144, 256), (2064, 3600, 512), (4368, 4112, 512), (272, 65552, 256),
                                   (4368, 4000, 256), (4000, 4368, 256)])
@pytest.mark.parametrize("layout", [o.NT, o.NN, o.TN])
def test_gemm_fast_kernel_ragged_big_tiles(M, N, K, g, layout):
    rng = np.random.default_rng(M + N)
    sa, sb = shapes_of(layout, M, N, K)
    A, B = rand_codes(rng, sa, o.E4M3), rand_codes(rng, sb, o.E5M2)
    if g == f8.TENSORWISE:
        isa, isb = np.float32(2.0 ** -5), np.float32(2.0 ** -9)
    else:
        isa = (rng.uniform(0.5, 2.0, M) * 2.0 ** -5).astype(np.float32)
        isb = (rng.uniform(0.5, 2.0, N) * 2.0 ** -9).astype(np.float32)
    got = run_gemm(layout, M, N, K, A, o.E4M3, B, o.E5M2, isa, isb, g)
    ref = o.gemm(layout, A, o.E4M3, B, o.E5M2, isa, isb, g)
    assert_gemm_close(got, ref, (M, N, K, g, layout))
    # per-row check as well, so that a wrong edge row cannot hide behind the global maximum
    gf, rf = o.bf16_to_f32(got).astype(np.float64), o.bf16_to_f32(ref).astype(np.float64)
    row_err = np.abs(gf - rf).max(axis=1)
    assert (row_err <= 1e-2 * np.abs(rf).max()).all()
    col_err = np.abs(gf - rf).max(axis=0)
    assert (col_err <= 1e-2 * np.abs(rf).max()).all()


@pytest.mark.parametrize("layout", [f8.NT, f8.NN, f8.TN])
@pytest.mark.parametrize("M,N,K", [(8192, 4096, 4096), (8192, 1024, 4096), (1024, 4096, 8192)])
def test_gemm_is_deterministic(M, N, K, layout):
    """The persistent kernel's LDS pipeline has no run-to-run freedom: repeated launches (one per
    tile configuration of the 8B shapes), interleaved with a launch that disturbs the caches,
    give identical bits."""
    rng = np.random.default_rng(K)
    sa, sb = shapes_of(layout, M, N, K)
    Ad = torch.from_numpy(rand_codes(rng, sa, o.E4M3)).cuda()
    Bd = torch.from_numpy(rand_codes(rng, sb, o.E4M3)).cuda()
    one = torch.ones(1, device="cuda")
    big = torch.empty(1 << 28, dtype=torch.uint8, device="cuda")
    outs = []
    for i in range(6):
        D = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        if i % 2:
            big.fill_(i)
        f8.gemm(layout, M, N, K, Ad, o.E4M3, Bd, o.E4M3, one, one, f8.TENSORWISE, D)
        outs.append(D)
    torch.cuda.synchronize()
    for D in outs[1:]:
        assert torch.equal(D.view(torch.int16), outs[0].view(torch.int16))
