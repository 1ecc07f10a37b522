// fp8 GEMM kernels for gfx950 (steps 4-6 of the Float8 linear: Y = X W^T,
// dX = dY W, dW = dY^T X) and the f8_gemm entry point.
//
// Two kernels:
//   gemm_nt_kernel      the fast path.  Both operands contraction-contiguous
//                       ("NT"), K a multiple of 64.  Global -> LDS direct
//                       loads (no VGPR staging), a ring of four LDS stages,
//                       XOR-swizzled 64-byte rows, v_mfma_f32_32x32x64_f8f6f4,
//                       scales folded into the fp32 epilogue, bf16 stores.
//   gemm_generic_kernel any layout, any multiple-of-16 shape; 64x64 tiles and
//                       the 16x16x32 fp8 MFMA.  The fallback.
//
// In both, the MFMA's first operand is fed from the B matrix (n index) and the
// second from the A matrix (m index): the accumulator registers of a lane then
// hold four consecutive n for one m, so the bf16 results leave as 8-byte pieces
// of a row of D.
#include <type_traits>

#include "f8_device.hpp"
#include "f8_host.hpp"

namespace f8 {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------------------
// epilogue helper: four fp32 accumulators -> four bf16 at D[m, n..n+3]
// ---------------------------------------------------------------------------
template <int GRAN>
__device__ inline void store4(uint16_t* __restrict__ D, int64_t ldd, int64_t m, int64_t n, v4f acc,
                              float s_tensor, const float* __restrict__ isa,
                              const float* __restrict__ isb)
{
    float r0, r1, r2, r3;
    if constexpr (GRAN == F8_TENSORWISE) {
        r0 = acc[0] * s_tensor, r1 = acc[1] * s_tensor, r2 = acc[2] * s_tensor, r3 = acc[3] * s_tensor;
    } else {
        const float sa = isa[m];
        const float4 sb = *reinterpret_cast<const float4*>(isb + n);
        r0 = (acc[0] * sa) * sb.x, r1 = (acc[1] * sa) * sb.y;
        r2 = (acc[2] * sa) * sb.z, r3 = (acc[3] * sa) * sb.w;
    }
    uint2 o;
    o.x = f32_to_bf16_bits(r0) | (f32_to_bf16_bits(r1) << 16);
    o.y = f32_to_bf16_bits(r2) | (f32_to_bf16_bits(r3) << 16);
    *reinterpret_cast<uint2*>(D + m * ldd + n) = o;
}

// ---------------------------------------------------------------------------
// Tile order: consecutive workgroup ids go round-robin to the 8 XCDs, each with
// its own L2.  Give every XCD one contiguous run of logical tile ids, and walk
// the tiles in bands of kGroupM tile-rows so that the 32 CUs of an XCD share A
// rows and B rows.
// ---------------------------------------------------------------------------
constexpr int kXcds = 8;
constexpr int kGroupM = 8;

__device__ inline void tile_coords(int pid, int tiles_m, int tiles_n, int* tm, int* tn)
{
    const int total = tiles_m * tiles_n;
    const int q = total / kXcds, r = total % kXcds;
    const int xcd = pid % kXcds, idx = pid / kXcds;
    const int logical = xcd * q + (xcd < r ? xcd : r) + idx;
    const int band = kGroupM * tiles_n;
    const int g = logical / band;
    const int first_m = g * kGroupM;
    const int gsz = (tiles_m - first_m) < kGroupM ? (tiles_m - first_m) : kGroupM;
    const int in = logical % band;
    *tm = first_m + in % gsz;
    *tn = in / gsz;
}

// ---------------------------------------------------------------------------
// fast NT kernel
// ---------------------------------------------------------------------------
// Block tile BM x BN, K step 64 bytes, a ring of four LDS stages filled by
// direct global->LDS loads three steps ahead; v_mfma_f32_32x32x64_f8f6f4; the
// fragments of step t+1 are read from LDS into a second register set while the
// MFMAs of step t run, so neither the barrier nor LDS latency sits on the MFMA
// critical path.
constexpr int kBK = 64;     // bytes of K per LDS stage = one 32x32x64 MFMA step
constexpr int kStages = 4;

typedef float v16f __attribute__((ext_vector_type(16)));

// XOR swizzle of the four 16-byte chunks of a 64-byte LDS row: lanes that read
// the same logical chunk of consecutive rows spread over all bank groups, for
// any aligned group of 8 lanes (128-byte bank window) and of 16 lanes (256-byte).
__device__ inline int swz(int row) { return (((row >> 1) ^ (row >> 3)) & 1) | (((row >> 2) & 1) << 1); }

// s_waitcnt immediate for "vmcnt <= n", other counters unconstrained (gfx9 encoding:
// vmcnt[3:0] in bits 3:0, vmcnt[5:4] in bits 15:14, expcnt 6:4, lgkmcnt 11:8).
constexpr int vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | 0x0070 | 0x0F00; }

template <int BM, int BN, int WAVES_M, int WAVES_N, int FA, int FB, int GRAN>
__global__ __launch_bounds__(WAVES_M* WAVES_N * 64) void gemm_nt_kernel(
    const uint8_t* __restrict__ A, const uint8_t* __restrict__ B, uint16_t* __restrict__ D, int M,
    int N, int K, int64_t lda, int64_t ldb, int64_t ldd, const float* __restrict__ isa,
    const float* __restrict__ isb, int tiles_m, int tiles_n)
{
    constexpr int NW = WAVES_M * WAVES_N;
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;  // wave tile
    constexpr int TM = WM / 32, TN = WN / 32;            // MFMA tiles per wave
    constexpr int A_BYTES = BM * kBK, STAGE = (BM + BN) * kBK;
    constexpr int A_LOADS = BM / 16 / NW, B_LOADS = BN / 16 / NW;  // 1 KB (16 rows) per wave load
    constexpr int LOADS = A_LOADS + B_LOADS;
    static_assert(BM % (16 * NW) == 0 && BN % (16 * NW) == 0, "tile rows must split over the waves");
    static_assert(LOADS * (kStages - 1) < 64, "vmcnt is a 6-bit counter");

    // One array per stage: the compiler then knows that a load into one stage does not alias
    // reads of another and does not serialise them.
    __shared__ __attribute__((aligned(1024))) uint8_t st0[STAGE];
    __shared__ __attribute__((aligned(1024))) uint8_t st1[STAGE];
    __shared__ __attribute__((aligned(1024))) uint8_t st2[STAGE];
    __shared__ __attribute__((aligned(1024))) uint8_t st3[STAGE];

    int tm, tn;
    tile_coords(blockIdx.x, tiles_m, tiles_n, &tm, &tn);
    const int m0 = tm * BM, n0 = tn * BN;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;

    // ---- global -> LDS addressing: wave w fills rows [w*R, (w+1)*R) of each operand tile in
    // 16-row (1 KB) pieces; lane i lands at row i/4, physical chunk i%4 of its piece.
    uint32_t a_off[A_LOADS], b_off[B_LOADS];
#pragma unroll
    for (int j = 0; j < A_LOADS; ++j) {
        const int row = wave * (BM / NW) + 16 * j + (lane >> 2);
        const int c = (lane & 3) ^ swz(row);
        int gr = m0 + row;
        gr = gr < M ? gr : M - 1;  // rows past the edge re-read the last row; never stored
        a_off[j] = (uint32_t)((int64_t)(gr - m0) * lda + 16 * c);
    }
#pragma unroll
    for (int j = 0; j < B_LOADS; ++j) {
        const int row = wave * (BN / NW) + 16 * j + (lane >> 2);
        const int c = (lane & 3) ^ swz(row);
        int gr = n0 + row;
        gr = gr < N ? gr : N - 1;
        b_off[j] = (uint32_t)((int64_t)(gr - n0) * ldb + 16 * c);
    }
    const uint8_t* a_base = A + (int64_t)m0 * lda;
    const uint8_t* b_base = B + (int64_t)n0 * ldb;
    const int KT = K / kBK;

    auto stage_ptr = [&](auto S) -> uint8_t* {
        if constexpr (decltype(S)::value == 0) return st0;
        else if constexpr (decltype(S)::value == 1) return st1;
        else if constexpr (decltype(S)::value == 2) return st2;
        else return st3;
    };

    // Every step issues exactly LOADS loads (past the end of K the last step is loaded again
    // into a stage nobody reads), so the vmcnt arithmetic below is the same for every step.
    auto issue_loads = [&](int kt, auto S) {
        kt = kt < KT ? kt : KT - 1;
        const uint8_t* ap = a_base + (int64_t)kt * kBK;
        const uint8_t* bp = b_base + (int64_t)kt * kBK;
        uint8_t* la = stage_ptr(S) + wave * (BM / NW) * kBK;
        uint8_t* lb = stage_ptr(S) + A_BYTES + wave * (BN / NW) * kBK;
#pragma unroll
        for (int j = 0; j < A_LOADS; ++j)
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void*)(ap + a_off[j]),
                (__attribute__((address_space(3))) void*)(la + j * 1024), 16, 0, 0);
#pragma unroll
        for (int j = 0; j < B_LOADS; ++j)
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void*)(bp + b_off[j]),
                (__attribute__((address_space(3))) void*)(lb + j * 1024), 16, 0, 0);
    };

    // ---- LDS -> register addressing: lane reads row (l % 32) of a 32-row MFMA tile, logical
    // chunks 2g and 2g+1 (g = l / 32): 32 consecutive K bytes.
    const int fr = lane & 31, fg = lane >> 5;
    const int pc0 = (2 * fg) ^ swz(fr);
    const int a_rd = (wm * WM + fr) * kBK + 16 * pc0;  // + 32-row tile * 2048
    const int b_rd = A_BYTES + (wn * WN + fr) * kBK + 16 * pc0;
    const int rd_flip = ((pc0 ^ 1) - pc0) * 16;        // to the second chunk

    struct Frags {
        v8i a[TM];
        v8i b[TN];
    };
    auto read_frags = [&](Frags& f, auto S) {
        const uint8_t* sa = stage_ptr(S) + a_rd;
        const uint8_t* sb = stage_ptr(S) + b_rd;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int4 lo = *reinterpret_cast<const int4*>(sa + i * 32 * kBK);
            const int4 hi = *reinterpret_cast<const int4*>(sa + i * 32 * kBK + rd_flip);
            f.a[i] = v8i{lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int4 lo = *reinterpret_cast<const int4*>(sb + j * 32 * kBK);
            const int4 hi = *reinterpret_cast<const int4*>(sb + j * 32 * kBK + rd_flip);
            f.b[j] = v8i{lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
        }
    };

    v16f acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // MFMAs number lo..hi-1 of a step (numbered i * TN + j)
    auto mfmas = [&](const Frags& f, auto LO, auto HI) {
#pragma unroll
        for (int q = decltype(LO)::value; q < decltype(HI)::value; ++q) {
            const int i = q / TN, j = q % TN;
            acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(f.b[j], f.a[i], acc[i][j], FB, FA, 0, 0,
                                                                          0, 0);
        }
    };

    // wait until at most `keep` of this wave's loads are in flight and all of its LDS reads
    // have returned, then meet the other waves
    auto sync_step = [&](auto KEEP) {
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(decltype(KEEP)::value) & 0xF0FF);  // lgkmcnt(0) too
        __builtin_amdgcn_s_barrier();
    };
    using std::integral_constant;
    constexpr int L = LOADS;
    constexpr int NMFMA = TM * TN;
    constexpr int HEAD = NMFMA >= 8 ? 4 : 1;  // MFMAs queued before the barrier, to cover its wait

    // One K step.  On entry `cur` holds the fragments of step t (stage S).  A few MFMAs are
    // queued first so that the matrix pipe has work while the wave sits at the barrier; after
    // the barrier step t+1 is complete in stage S+1 for every wave, stage S is free for step
    // t+4, and the LDS reads of step t+1 and the new loads are interleaved with the remaining
    // MFMAs of step t.
    auto step = [&](int t, auto S, Frags& cur, Frags& next) {
        constexpr int s = decltype(S)::value;
        mfmas(cur, integral_constant<int, 0>{}, integral_constant<int, HEAD>{});
        __builtin_amdgcn_sched_barrier(0);
        sync_step(integral_constant<int, (kStages - 2) * L>{});
        __builtin_amdgcn_sched_barrier(0);
        read_frags(next, integral_constant<int, (s + 1) % kStages>{});
        issue_loads(t + kStages, S);
        mfmas(cur, integral_constant<int, HEAD>{}, integral_constant<int, NMFMA>{});
        // schedule shape for the compiler: after each MFMA up to two LDS reads and one load
#pragma unroll
        for (int q = 0; q < NMFMA - HEAD; ++q) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // one MFMA
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);  // two DS reads
            __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);  // one VMEM read
        }
        __builtin_amdgcn_sched_barrier(0);
    };

    // prologue: steps 0..3 in flight, step 0 into registers
    issue_loads(0, integral_constant<int, 0>{});
    issue_loads(1, integral_constant<int, 1>{});
    issue_loads(2, integral_constant<int, 2>{});
    issue_loads(3, integral_constant<int, 3>{});
    Frags f0, f1;
    sync_step(integral_constant<int, (kStages - 1) * L>{});
    read_frags(f0, integral_constant<int, 0>{});

    const int KT4 = KT & ~3;
    for (int t = 0; t < KT4; t += 4) {
        step(t, integral_constant<int, 0>{}, f0, f1);
        step(t + 1, integral_constant<int, 1>{}, f1, f0);
        step(t + 2, integral_constant<int, 2>{}, f0, f1);
        step(t + 3, integral_constant<int, 3>{}, f1, f0);
    }
    if (KT4 < KT) step(KT4, integral_constant<int, 0>{}, f0, f1);
    if (KT4 + 1 < KT) step(KT4 + 1, integral_constant<int, 1>{}, f1, f0);
    if (KT4 + 2 < KT) step(KT4 + 2, integral_constant<int, 2>{}, f0, f1);
    // no load may still be writing LDS when the block ends
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));

    // ---- epilogue: of each 32x32 tile, lane l holds m = l % 32 and
    // n = 8 * (r / 4) + 4 * (l / 32) + r % 4 for accumulator register r
    float s_tensor = 0.f;
    if constexpr (GRAN == F8_TENSORWISE) s_tensor = isa[0] * isb[0];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int m = m0 + wm * WM + 32 * i + fr;
        if (m >= M) continue;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int n = n0 + wn * WN + 32 * j + 8 * q + 4 * fg;
                const v4f v = v4f{acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
                if (n < N) store4<GRAN>(D, ldd, m, n, v, s_tensor, isa, isb);
            }
        }
    }
}

// ---------------------------------------------------------------------------
// generic kernel: 64x64 tile, 4 waves of 32x32, K step 64, 16x16x32 MFMA
// ---------------------------------------------------------------------------
template <int FOP_A, int FOP_B>  // formats of the MFMA's first / second operand
__device__ inline v4f mfma32(long a, long b, v4f c)
{
    if constexpr (FOP_A == F8_E4M3 && FOP_B == F8_E4M3) return __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(a, b, c, 0, 0, 0);
    else if constexpr (FOP_A == F8_E4M3 && FOP_B == F8_E5M2) return __builtin_amdgcn_mfma_f32_16x16x32_fp8_bf8(a, b, c, 0, 0, 0);
    else if constexpr (FOP_A == F8_E5M2 && FOP_B == F8_E4M3) return __builtin_amdgcn_mfma_f32_16x16x32_bf8_fp8(a, b, c, 0, 0, 0);
    else return __builtin_amdgcn_mfma_f32_16x16x32_bf8_bf8(a, b, c, 0, 0, 0);
}

constexpr int kGT = 64;        // generic tile (rows and K bytes)
constexpr int kGStride = 80;   // LDS row stride in bytes (64 + 16 pad, keeps 16-byte alignment)

// Fill a 64 x 64 (rows x K) LDS tile from an operand stored either [rows, K] (KCONTIG) or [K, rows].
template <bool KCONTIG>
__device__ inline void generic_load(uint8_t* __restrict__ tile, const uint8_t* __restrict__ P, int64_t ld,
                                    int row0, int nrows, int k0, int K)
{
    const int t = threadIdx.x;
    if constexpr (KCONTIG) {
        const int r = t >> 2, c = (t & 3) * 16;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (row0 + r < nrows && k0 + c < K)  // K is a multiple of 16: whole chunk in or out
            v = *reinterpret_cast<const uint4*>(P + (int64_t)(row0 + r) * ld + k0 + c);
        *reinterpret_cast<uint4*>(tile + r * kGStride + c) = v;
    } else {
        const int k = t >> 2, c = (t & 3) * 16;  // 16 consecutive rows of the tile at one k
        uint4 v = make_uint4(0, 0, 0, 0);
        if (k0 + k < K && row0 + c < nrows)
            v = *reinterpret_cast<const uint4*>(P + (int64_t)(k0 + k) * ld + row0 + c);
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 16; ++i) tile[(c + i) * kGStride + k] = (uint8_t)(w[i >> 2] >> (8 * (i & 3)));
    }
}

template <int LAYOUT, int FA, int FB, int GRAN>
__global__ __launch_bounds__(256) void gemm_generic_kernel(
    const uint8_t* __restrict__ A, const uint8_t* __restrict__ B, uint16_t* __restrict__ D, int M,
    int N, int K, int64_t lda, int64_t ldb, int64_t ldd, const float* __restrict__ isa,
    const float* __restrict__ isb)
{
    __shared__ __attribute__((aligned(16))) uint8_t As[kGT * kGStride];
    __shared__ __attribute__((aligned(16))) uint8_t Bs[kGT * kGStride];
    const int m0 = blockIdx.y * kGT, n0 = blockIdx.x * kGT;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int fr = lane & 15, fg = lane >> 4;

    v4f acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = v4f{0.f, 0.f, 0.f, 0.f};

    for (int k0 = 0; k0 < K; k0 += kGT) {
        __syncthreads();
        generic_load<LAYOUT != F8_TN>(As, A, lda, m0, M, k0, K);
        generic_load<LAYOUT == F8_NT>(Bs, B, ldb, n0, N, k0, K);
        __syncthreads();
#pragma unroll
        for (int ks = 0; ks < kGT; ks += 32) {
            long af[2], bf[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                af[i] = *reinterpret_cast<const long*>(As + (wm * 32 + 16 * i + fr) * kGStride + ks + 8 * fg);
                bf[i] = *reinterpret_cast<const long*>(Bs + (wn * 32 + 16 * i + fr) * kGStride + ks + 8 * fg);
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) acc[i][j] = mfma32<FB, FA>(bf[j], af[i], acc[i][j]);
        }
    }
    float s_tensor = 0.f;
    if constexpr (GRAN == F8_TENSORWISE) s_tensor = isa[0] * isb[0];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int m = m0 + wm * 32 + 16 * i + fr;
        if (m >= M) continue;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int n = n0 + wn * 32 + 16 * j + 4 * fg;
            if (n < N) store4<GRAN>(D, ldd, m, n, acc[i][j], s_tensor, isa, isb);
        }
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------

template <int BM, int BN, int WAVES_M, int WAVES_N, int FA, int FB, int GRAN>
static void launch_nt(int M, int N, int K, const uint8_t* A, int64_t lda, const uint8_t* B, int64_t ldb,
                      const float* isa, const float* isb, uint16_t* D, int64_t ldd, hipStream_t st)
{
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    gemm_nt_kernel<BM, BN, WAVES_M, WAVES_N, FA, FB, GRAN><<<tiles_m * tiles_n, WAVES_M * WAVES_N * 64, 0, st>>>(
        A, B, D, M, N, K, lda, ldb, ldd, isa, isb, tiles_m, tiles_n);
}

template <int FA, int FB, int GRAN>
static void dispatch_nt(int M, int N, int K, const uint8_t* A, int64_t lda, const uint8_t* B, int64_t ldb,
                        const float* isa, const float* isb, uint16_t* D, int64_t ldd, hipStream_t st)
{
    // 256x256 tiles when they give at least one full wave of workgroups over the 256 CUs,
    // otherwise 128x128 to keep more CUs busy.
    const int64_t big_tiles = (int64_t)((M + 255) / 256) * ((N + 255) / 256);
    if (big_tiles >= 256)
        launch_nt<256, 256, 2, 2, FA, FB, GRAN>(M, N, K, A, lda, B, ldb, isa, isb, D, ldd, st);
    else
        launch_nt<128, 128, 2, 2, FA, FB, GRAN>(M, N, K, A, lda, B, ldb, isa, isb, D, ldd, st);
}

template <int LAYOUT, int FA, int FB, int GRAN>
static void launch_generic(int M, int N, int K, const uint8_t* A, int64_t lda, const uint8_t* B, int64_t ldb,
                           const float* isa, const float* isb, uint16_t* D, int64_t ldd, hipStream_t st)
{
    dim3 grid((N + kGT - 1) / kGT, (M + kGT - 1) / kGT);
    gemm_generic_kernel<LAYOUT, FA, FB, GRAN><<<grid, 256, 0, st>>>(A, B, D, M, N, K, lda, ldb, ldd, isa, isb);
}

template <int FA, int FB, int GRAN>
static void dispatch_layout(int layout, int M, int N, int K, const uint8_t* A, int64_t lda, const uint8_t* B,
                            int64_t ldb, const float* isa, const float* isb, uint16_t* D, int64_t ldd,
                            hipStream_t st)
{
    if (layout == F8_NT) {
        if (K % kBK == 0 && K > 0)
            dispatch_nt<FA, FB, GRAN>(M, N, K, A, lda, B, ldb, isa, isb, D, ldd, st);
        else
            launch_generic<F8_NT, FA, FB, GRAN>(M, N, K, A, lda, B, ldb, isa, isb, D, ldd, st);
    } else if (layout == F8_NN) {
        launch_generic<F8_NN, FA, FB, GRAN>(M, N, K, A, lda, B, ldb, isa, isb, D, ldd, st);
    } else {
        launch_generic<F8_TN, FA, FB, GRAN>(M, N, K, A, lda, B, ldb, isa, isb, D, ldd, st);
    }
}

f8_status gemm(int layout, int64_t M, int64_t N, int64_t K, const uint8_t* A, int fa, int64_t lda,
               const uint8_t* B, int fb, int64_t ldb, const float* isa, const float* isb, int g, void* D,
               int64_t ldd, hipStream_t st)
{
    if (M == 0 || N == 0) return F8_OK;
    uint16_t* d = static_cast<uint16_t*>(D);
    const int m = (int)M, n = (int)N, k = (int)K;
#define F8_GEMM_CASE(FA_, FB_)                                                                     \
    do {                                                                                           \
        if (g == F8_TENSORWISE)                                                                    \
            dispatch_layout<FA_, FB_, F8_TENSORWISE>(layout, m, n, k, A, lda, B, ldb, isa, isb, d, ldd, st); \
        else                                                                                       \
            dispatch_layout<FA_, FB_, F8_ROWWISE>(layout, m, n, k, A, lda, B, ldb, isa, isb, d, ldd, st);    \
    } while (0)
    if (fa == F8_E4M3 && fb == F8_E4M3) F8_GEMM_CASE(F8_E4M3, F8_E4M3);
    else if (fa == F8_E5M2 && fb == F8_E4M3) F8_GEMM_CASE(F8_E5M2, F8_E4M3);
    else if (fa == F8_E4M3 && fb == F8_E5M2) F8_GEMM_CASE(F8_E4M3, F8_E5M2);
    else F8_GEMM_CASE(F8_E5M2, F8_E5M2);
#undef F8_GEMM_CASE
    return last_launch_status();
}

}  // namespace f8

using namespace f8;

extern "C" f8_status f8_gemm(f8_layout layout, int64_t M, int64_t N, int64_t K, const uint8_t* A,
                             f8_format fa, int64_t lda, const uint8_t* B, f8_format fb, int64_t ldb,
                             const float* inv_scale_a, const float* inv_scale_b, f8_granularity g,
                             void* D_bf16, int64_t ldd, void* stream)
{
    if ((int)layout < 0 || (int)layout > F8_TN || (int)fa < 0 || (int)fa > F8_E5M2 || (int)fb < 0 ||
        (int)fb > F8_E5M2 || ((int)g != F8_TENSORWISE && (int)g != F8_ROWWISE))
        return F8_ERR_ENUM;
    if (!A || !B || !D_bf16 || !inv_scale_a || !inv_scale_b) return F8_ERR_NULL;
    if (M < 0 || N < 0 || K < 0 || (M % 16) || (N % 16) || (K % 16) || (lda % 16) || (ldb % 16) || (ldd % 16))
        return F8_ERR_SHAPE;
    if (M >= (1 << 23) || N >= (1 << 23) || K >= (1 << 23) || lda >= (1 << 23) || ldb >= (1 << 23)) return F8_ERR_SHAPE;
    const int64_t a_cols = layout == F8_TN ? M : K, b_cols = layout == F8_NT ? K : N;
    if (lda < a_cols || ldb < b_cols || ldd < N) return F8_ERR_SHAPE;
    if (!aligned16(A) || !aligned16(B) || !aligned16(D_bf16)) return F8_ERR_ALIGN;
    if (g == F8_ROWWISE && !aligned16(inv_scale_b)) return F8_ERR_ALIGN;
    if (K == 0) {
        // empty contraction: D = 0.  The generic kernel's K loop does not run and stores zeros.
    }
    return gemm(layout, M, N, K, A, fa, lda, B, fb, ldb, inv_scale_a, inv_scale_b, g, D_bf16, ldd,
                (hipStream_t)stream);
}
