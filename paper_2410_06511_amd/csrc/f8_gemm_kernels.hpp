// fp8 GEMM kernels for gfx950 (steps 4-6 of the Float8 linear: Y = X W^T,
// dX = dY W, dW = dY^T X) (kernels and launch logic; f8_gemm.hip holds the entry points,
// f8_gemm_inst.hip is compiled once per operand-format pair and layout, in parallel).
//
// Two kernels:
//   gemm_tile_kernel    the fast path, K a multiple of 256, all three layouts.
//                       Persistent workgroups, global -> LDS direct loads (no
//                       VGPR staging), two LDS stages, v_mfma_f32_16x16x128_f8f6f4,
//                       scales folded into the fp32 epilogue, bf16 stores staged
//                       through LDS.  An operand whose contraction index is the
//                       fast one in memory ("row-major in K": both of F8_NT, A of
//                       F8_NN) is staged as XOR-swizzled 128-byte rows; one whose
//                       contraction index is the slow one ("k-major": B of F8_NN,
//                       both of F8_TN) is staged as it lies in memory and turned
//                       on its way from LDS to the registers by the transposing
//                       LDS read, so no transposed copy of any operand is needed.
//   gemm_generic_kernel any layout, any multiple-of-16 shape; 64x64 tiles and
//                       the 16x16x32 fp8 MFMA.  The fallback.
//
// In both, the MFMA's first operand is fed from the B matrix (n index) and the
// second from the A matrix (m index): the accumulator registers of a lane then
// hold four consecutive n for one m, so the bf16 results leave as 8-byte pieces
// of a row of D.
#pragma once
#include <type_traits>
#include <utility>

#include "f8_device.hpp"
#include "f8_host.hpp"

namespace f8 {

// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>), unrolled at compile time
template <int N, class F>
__device__ inline void static_for(F&& f)
{
    [&]<int... Is>(std::integer_sequence<int, Is...>) { (f(std::integral_constant<int, Is>{}), ...); }
    (std::make_integer_sequence<int, N>{});
}

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------------------
// epilogue helper: four fp32 accumulators -> four bf16 at D[m, n..n+3]
// ---------------------------------------------------------------------------
template <int GRAN>
__device__ inline uint2 store4(uint16_t* __restrict__ D, int64_t ldd, int64_t m, int64_t n, v4f acc,
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
    return o;
}

// amax of the bf16 output, kept as a bf16 magnitude in the upper half of a word so that the
// unsigned integer order of the words is the order of the magnitudes; combined across
// wavefronts with one atomic max per wavefront (the entry point zeroes the word first).
__device__ inline uint32_t amax_pair(uint32_t acc, uint2 o)
{
    return pkmax(pkmax(acc, o.x & 0x7FFF7FFFu), o.y & 0x7FFF7FFFu);
}
// `red`: one word of LDS per wavefront, free for use.  Called by every thread of the block.
// Same-address atomics from a thousand wavefronts serialise at the memory side, so the block
// combines its wavefronts first and skips the atomic when the published value is already at
// least as large (the value only ever grows, so a stale read costs one extra atomic, nothing else).
template <int NW>
__device__ inline void amax_publish(uint32_t acc, uint32_t* amax_bits, uint32_t* red)
{
    const uint32_t m = block_max_u32<NW>(pk_collapse(acc), red) << 16;
    if (threadIdx.x == 0 && m > __atomic_load_n(amax_bits, __ATOMIC_RELAXED)) atomicMax(amax_bits, m);
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
// fast kernel
// ---------------------------------------------------------------------------
// Persistent workgroups (one or two per CU) walk over BM x BN output tiles.  K advances in
// steps of 128 bytes = one LDS stage (a full cache line per row and load) = the contraction
// length of one v_mfma_f32_16x16x128_f8f6f4; two stages, filled by direct global->LDS loads.
// (Of the two fp8 matrix instructions of equal nominal rate, 16x16x128 and 32x32x64, the first
// is used: one instruction spans exactly one LDS stage, and the kernel built on it ran faster.
// With operands in registers and nothing else going on the two sustain the same rate.)
// A wave's 128 x 128 tile is 8 x 8 matrix-instruction tiles, i.e. 8 + 8 operand fragments per K
// step.  The load stream runs two K steps ahead of the MFMAs and does not stop at tile
// boundaries, so the next tile's first stages arrive while the current tile's epilogue runs.
// There are two barriers per K step (this stage is free to refill; the other stage has
// landed), each with MFMAs queued in front of it.
constexpr int kBK = 128;  // bytes of K per LDS stage

typedef float f2 __attribute__((ext_vector_type(2)));
typedef __bf16 b2 __attribute__((ext_vector_type(2)));

// XOR swizzle of the eight 16-byte chunks of a 128-byte LDS row.  The fragment read of a row-major
// operand is two ds_read_b128 per lane: lane l takes row l % 16 of the fragment, logical chunks
// 2 (l / 16) and 2 (l / 16) + 1.  LDS banks repeat every 256 bytes, so the row's parity already
// picks one half of them; bits 1 and 2 of the row are folded into the chunk number.  Measured
// with a four-wave read loop over all 4096 linear maps row -> chunk XOR: this one (like about a
// quarter of them) runs such a read at the rate of a contiguous one, 4 cycles per kilobyte; maps
// that also fold in bit 0 or bit 3 of the row take 8.
__device__ inline int swz(int row) { return (((row >> 1) & 1) << 2) | ((row >> 2) & 1); }

// ---- k-major operand tiles ----------------------------------------------------------
// An operand stored [K, R-direction] (B of F8_NN, both operands of F8_TN) is staged as it
// lies in memory: per stage 128 k-rows of R = BM or BN bytes.  The MFMA wants, per lane, 32
// consecutive k of one row of the operand (lane l: row l % 16 of the 16-row fragment, k range
// l / 16); ds_read_b64_tr_b8 forms them: within each group of 16 lanes, lane i receives byte
// i % 8 of the 8-byte pieces addressed by lanes i / 8, 2 + i / 8, ..., 14 + i / 8.  With lane s
// of the group pointing at k-row k0 + s / 2, bytes 8 (s % 2) .. + 7 of the fragment's 16-byte
// chunk of it, lane i ends up with k0 .. k0 + 7 of fragment row i, in natural k order; four
// such reads (k0 = 32 (l / 16) + 0, 8, 16, 24) make one 32-byte fragment register set.
// The 16-byte chunks of a k-row are permuted so that the 8 k-rows of one group, and the groups
// that read together (k ranges 32 apart), fall on different banks.
template <int R>
__device__ inline int kswz(int chunk, int krow)  // logical chunk of k-row -> physical chunk
{
    if constexpr (R == 256) {
        const int kx = (krow & 7) | (((krow >> 5) & 1) << 3);
        return (((chunk & 1) << 3) | (chunk >> 1)) ^ kx;  // chunk bit 0 goes to the 128-byte half
    } else {
        return chunk ^ (krow & 7) ^ ((krow >> 5) & 1);    // 128-byte rows: the row parity picks the half
    }
}
template <int R>
__device__ inline int kswz_inv(int phys, int krow)
{
    if constexpr (R == 256) {
        const int q = phys ^ ((krow & 7) | (((krow >> 5) & 1) << 3));
        return ((q & 7) << 1) | (q >> 3);
    } else {
        return phys ^ (krow & 7) ^ ((krow >> 5) & 1);
    }
}
// kswz<R>(c0 ^ idx, k) = kswz<R>(c0, k) ^ kswz_step<R>(idx): the permutation is linear in the chunk
template <int R>
constexpr int kswz_step(int idx) { return R == 256 ? (((idx & 1) << 3) | (idx >> 1)) : idx; }

typedef int v2i __attribute__((ext_vector_type(2)));
__device__ inline v2i lds_read_tr8(const uint8_t* p)
{
    return __builtin_amdgcn_ds_read_tr8_b64_v2i32((__attribute__((address_space(3))) v2i*)p);
}

// s_waitcnt immediate (gfx9 encoding: vmcnt[3:0] bits 3:0, vmcnt[5:4] bits 15:14, expcnt 6:4,
// lgkmcnt 11:8): wait for all vector-memory operations and all LDS operations.
constexpr int kWaitAllVmLgkm = 0x0070;

// AKM / BKM: operand A / B is k-major (A[K, M] with leading dimension lda, B[K, N] with ldb).
// SPLITK: the contraction is cut into `splits` equal ranges and a work item is (tile, range);
// item w is tile w % tiles, range w / tiles.  Instead of D the kernel then writes the unscaled
// fp32 sums of range s to partial[s][M][ldp]; splitk_reduce_kernel adds the ranges in order,
// applies the scales and rounds to bf16.  (For products with few output tiles and a long
// contraction, where whole tiles would leave most compute units idle.)
template <int BM, int BN, int WAVES_M, int WAVES_N, int FA, int FB, int GRAN, bool AMAX, bool AKM, bool BKM,
          bool SPLITK = false>
__global__ __launch_bounds__(WAVES_M* WAVES_N * 64) void gemm_tile_kernel(
    const uint8_t* __restrict__ A, const uint8_t* __restrict__ B, uint16_t* __restrict__ D, int M,
    int N, int K, int64_t lda, int64_t ldb, int64_t ldd, const float* __restrict__ isa,
    const float* __restrict__ isb, int tiles_m, int tiles_n, uint32_t* __restrict__ amax_bits,
    int splits = 1, float* __restrict__ partial = nullptr, int64_t ldp = 0)
{
    static_assert(!(SPLITK && AMAX), "the output amax is taken by the kernel that writes D");
    constexpr int NW = WAVES_M * WAVES_N;
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;  // wave tile
    constexpr int TM = WM / 16, TN = WN / 16;            // MFMA tiles (fragments) per wave
    constexpr int A_BYTES = BM * kBK, STAGE = (BM + BN) * kBK;
    constexpr int A_LOADS = BM / 8 / NW, B_LOADS = BN / 8 / NW;  // 1 KB (8 rows) per wave load
    static_assert(BM % (8 * NW) == 0 && BN % (8 * NW) == 0, "tile rows must split over the waves");
    static_assert(NW == 4, "four waves");
    static_assert(WAVES_M == 2 && WAVES_N == 2 && (BM == 256 || BM == 128) && (BN == 256 || BN == 128),
                  "the addressing assumes 2 x 2 waves on 128- or 256-wide tiles");
    // An epilogue pass stages 8 MFMA tiles: EPW of them side by side (the whole width of the wave's
    // tile if that is 128 columns: a store instruction then covers 4 rows x 256 bytes, measured
    // 1 % faster on the products than 8 rows x 128 bytes), 8 / EPW below each other
    constexpr int EPW = TN >= 8 ? 8 : 4, EPR = 8 / EPW;
    constexpr int EP_STRIDE = 16 * EPW * 2 + 16;    // bytes per staged epilogue row: the bf16 of a row + padding
    static_assert(TM % EPR == 0 && TN % EPW == 0, "the wave tile is a whole number of epilogue passes");

    // One array per stage: the compiler then knows that a load into one stage does not alias
    // LDS reads of the other and does not serialise them.
    __shared__ __attribute__((aligned(1024))) uint8_t st0[STAGE];
    __shared__ __attribute__((aligned(1024))) uint8_t st1[STAGE];
    __shared__ __attribute__((aligned(16))) uint8_t epb[NW * 16 * EPR * EP_STRIDE];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;
    const int tiles_mn = tiles_m * tiles_n;
    const int total_tiles = SPLITK ? tiles_mn * splits : tiles_mn;  // work items of the launch
    const int KT = SPLITK ? K / kBK / splits : K / kBK;             // K steps per work item

    using std::integral_constant;
    auto stage_ptr = [&](auto S) -> uint8_t* {
        if constexpr (decltype(S)::value == 0) return st0;
        else return st1;
    };

    // ---- load stream: (tile, K step) of the next stage to fetch -------------------------
    // wave w fills rows [w*R, (w+1)*R) of each operand tile in 8-row (1 KB) pieces; lane i
    // lands at row i/8, physical chunk i%8 of its piece.  A load is then only: LDS target into
    // M0, one instruction with a per-load lane offset (kept in a register, rebuilt per tile) and a
    // scalar base that moves with the K step.  Anything more per load would not fit between two
    // matrix instructions (32 cycles), and the matrix pipe would wait for the instruction stream.
    int ld_tile = blockIdx.x;
    // row-major operand: the lane's row of piece 0 in the tile decides its chunk terms (the
    // swizzle looks at bits 1 and 2 of the row only, so every 8-row piece has the same)
    const int a_row = wave * (BM / NW) + (lane >> 3);
    const int b_row = wave * (BN / NW) + (lane >> 3);
    // k-major operand: a 1 KB load covers 1024 / R k-rows; lane i lands at k-row i / (R / 16),
    // physical chunk i % (R / 16) of them and fetches the logical chunk that belongs there.  The
    // wave fills k-rows [32 * wave, 32 * wave + 32).  Of the k-row only bits 0-2 and 5 enter the
    // permutation: bit 5 is that of the wave; bits 0-2 are those of 4 * (load number % 2) +
    // lane's row for R = 256 (four rows per load), of the lane's row for R = 128 (eight per load).
    constexpr int A_CPR = BM / 16, B_CPR = BN / 16;  // chunks per k-row
    const int a_kr = lane / A_CPR, b_kr = lane / B_CPR;
    uint32_t a_c0, a_c1, b_c0, b_c1;  // byte offset of the lane's chunk for even / odd load numbers
    if constexpr (AKM) {
        a_c0 = 16 * kswz_inv<BM>(lane % A_CPR, 32 * wave + a_kr);
        a_c1 = 16 * kswz_inv<BM>(lane % A_CPR, 32 * wave + a_kr + (BM == 256 ? 4 : 0));
    } else {
        a_c0 = 16 * ((lane & 7) ^ swz(a_row)), a_c1 = 16 * ((lane & 7) ^ swz(a_row + 8));
    }
    if constexpr (BKM) {
        b_c0 = 16 * kswz_inv<BN>(lane % B_CPR, 32 * wave + b_kr);
        b_c1 = 16 * kswz_inv<BN>(lane % B_CPR, 32 * wave + b_kr + (BN == 256 ? 4 : 0));
    } else {
        b_c0 = 16 * ((lane & 7) ^ swz(b_row)), b_c1 = 16 * ((lane & 7) ^ swz(b_row + 8));
    }
    static_assert((BM / NW) % 16 == 0 && (BN / NW) % 16 == 0 && kBK / NW == 32, "swizzle period; 32 k-rows per wave");
    const uint8_t* a_base = A;
    const uint8_t* b_base = B;
    // The lane's byte offset of every load of a K step, relative to the step's base address
    // (a_base / b_base + K step * 128 bytes, or * 128 k-rows).  row-major: (row of the piece +
    // lane's row in it) * ld + chunk; pieces past the edge of the matrix (M and N are multiples
    // of 16, so a piece is all in or all out) re-read the last piece inside: their products are
    // never stored.  k-major: k-row * ld + chunk, with chunks past the edge re-reading the last
    // valid chunk of the k-row.
    uint32_t a_off[A_LOADS], b_off[B_LOADS];
    auto load_context = [&](int item) {
        int tm, tn;
        tile_coords(SPLITK ? item % tiles_mn : item, tiles_m, tiles_n, &tm, &tn);
        const int64_t koff = SPLITK ? (int64_t)(item / tiles_mn) * KT * kBK : 0;  // first k of the item's range
        if constexpr (AKM) {
            a_base = A + (int64_t)tm * BM + koff * lda;
            const uint32_t cmax = (uint32_t)(M - 16 - tm * BM);
#pragma unroll
            for (int idx = 0; idx < A_LOADS; ++idx)
                a_off[idx] = (uint32_t)(wave * (kBK / NW) + idx * (1024 / BM) + a_kr) * (uint32_t)lda +
                             (((idx & 1) ? a_c1 : a_c0) < cmax ? ((idx & 1) ? a_c1 : a_c0) : cmax);
        } else {
            a_base = A + (int64_t)tm * BM * lda + koff;
            const int pmax = M - 8 - tm * BM;  // first row of the last piece inside, relative to the tile
#pragma unroll
            for (int idx = 0; idx < A_LOADS; ++idx) {
                int prow = wave * (BM / NW) + 8 * idx;
                prow = prow < pmax ? prow : pmax;
                a_off[idx] = (uint32_t)(prow + (lane >> 3)) * (uint32_t)lda + ((idx & 1) ? a_c1 : a_c0);
            }
        }
        if constexpr (BKM) {
            b_base = B + (int64_t)tn * BN + koff * ldb;
            const uint32_t cmax = (uint32_t)(N - 16 - tn * BN);
#pragma unroll
            for (int j = 0; j < B_LOADS; ++j)
                b_off[j] = (uint32_t)(wave * (kBK / NW) + j * (1024 / BN) + b_kr) * (uint32_t)ldb +
                           (((j & 1) ? b_c1 : b_c0) < cmax ? ((j & 1) ? b_c1 : b_c0) : cmax);
        } else {
            b_base = B + (int64_t)tn * BN * ldb + koff;
            const int pmax = N - 8 - tn * BN;
#pragma unroll
            for (int j = 0; j < B_LOADS; ++j) {
                int prow = wave * (BN / NW) + 8 * j;
                prow = prow < pmax ? prow : pmax;
                b_off[j] = (uint32_t)(prow + (lane >> 3)) * (uint32_t)ldb + ((j & 1) ? b_c1 : b_c0);
            }
        }
    };
    // Load number `idx` (0 .. LOADS-1: first the A pieces, then the B pieces) of the K step whose
    // base addresses are ga / gb, into stage S.  Written as asm: 32-bit lane offset next to a
    // scalar base, LDS target in M0.  The compiler therefore does not see these as LDS writes;
    // ordering against the LDS reads is by the barriers and explicit waits of kstep.
    auto issue_one = [&](const uint8_t* ga, const uint8_t* gb, auto S, auto IDX) {
        constexpr int idx = decltype(IDX)::value;
        if constexpr (idx < A_LOADS) {
            uint8_t* lp = stage_ptr(S) + wave * (BM / NW) * kBK + idx * 1024;
            const uint32_t l32 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)lp;
            const uint32_t o = a_off[idx];
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(l32), "v"(o), "s"(ga) : "memory");
        } else {
            constexpr int j = idx - A_LOADS;
            uint8_t* lp = stage_ptr(S) + A_BYTES + wave * (BN / NW) * kBK + j * 1024;
            const uint32_t l32 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)lp;
            const uint32_t o = b_off[j];
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(l32), "v"(o), "s"(gb) : "memory");
        }
    };
    // base addresses of K step kt of the stream's current tile
    auto step_base_a = [&](int kt) { return AKM ? a_base + (int64_t)kt * kBK * lda : a_base + (int64_t)kt * kBK; };
    auto step_base_b = [&](int kt) { return BKM ? b_base + (int64_t)kt * kBK * ldb : b_base + (int64_t)kt * kBK; };
    auto issue_all = [&](int kt, auto S) {
        const uint8_t* ga = step_base_a(kt);
        const uint8_t* gb = step_base_b(kt);
        static_for<A_LOADS + B_LOADS>([&](auto L) { issue_one(ga, gb, S, L); });
    };
    // Move the load stream to this workgroup's next tile.  Past the last tile the stream
    // stays where it is: the same K steps are fetched again into stages nobody reads, so that
    // every K step issues the same number of loads and the wait counts below hold throughout.
    auto next_load_tile = [&]() {
        ld_tile += gridDim.x;
        if (ld_tile < total_tiles) load_context(ld_tile);
    };

    // ---- LDS -> register addressing.  A fragment is 16 rows of an operand x the stage's 128 K
    // bytes; lane l holds row l % 16, K bytes 32 (l / 16) .. + 31.
    // Row-major operand: the lane reads the logical chunks 2 (l / 16) and 2 (l / 16) + 1 of its row.
    const int fr = lane & 15, fg = lane >> 4;
    const int pc0 = (2 * fg) ^ swz(fr);
    const int flip1 = ((pc0 ^ 1) - pc0) * 16;          // to the second chunk of the pair
    // k-major operand: lane s of 16-lane group g points at k-row 32 g + s / 2 (+ 8 t for the t-th
    // of the four reads) and at the 8 bytes (s % 2) of the fragment's chunk.  Going to fragment idx
    // of the wave moves idx chunks on, which the permutation turns into an XOR of the address.
    auto km_read_base = [&](auto R_, int wave_row0) {
        constexpr int R = decltype(R_)::value;
        const int krow = 32 * fg + (fr >> 1);
        return krow * R + 16 * kswz<R>(wave_row0 / 16, krow) + 8 * (fr & 1);
    };
    int a_rd, b_rd;
    if constexpr (AKM) a_rd = km_read_base(integral_constant<int, BM>{}, wm * WM);
    else a_rd = (wm * WM + fr) * kBK + 16 * pc0;  // + fragment * 16 rows
    if constexpr (BKM) b_rd = A_BYTES + km_read_base(integral_constant<int, BN>{}, wn * WN);
    else b_rd = A_BYTES + (wn * WN + fr) * kBK + 16 * pc0;

    v8i fa[TM], fb[TN];  // operand fragments in registers
    v8i fb_early;        // the next K step's last B fragment, read while this step's is still in use
    auto read_km = [&](const uint8_t* p, auto R_) {
        constexpr int R = decltype(R_)::value;
        const v2i t0 = lds_read_tr8(p), t1 = lds_read_tr8(p + 8 * R), t2 = lds_read_tr8(p + 16 * R),
                  t3 = lds_read_tr8(p + 24 * R);
        return v8i{t0.x, t0.y, t1.x, t1.y, t2.x, t2.y, t3.x, t3.y};
    };
    auto read_rm = [&](const uint8_t* p) {
        const int4 lo = *reinterpret_cast<const int4*>(p);
        const int4 hi = *reinterpret_cast<const int4*>(p + flip1);
        return v8i{lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
    };
    auto read_a = [&](auto S, auto IDX) {
        constexpr int idx = decltype(IDX)::value;
        if constexpr (AKM) fa[idx] = read_km(stage_ptr(S) + (a_rd ^ (16 * kswz_step<BM>(idx))), integral_constant<int, BM>{});
        else fa[idx] = read_rm(stage_ptr(S) + a_rd + idx * 16 * kBK);
    };
    auto read_b = [&](auto S, auto IDX) {
        constexpr int idx = decltype(IDX)::value;
        if constexpr (BKM) fb[idx] = read_km(stage_ptr(S) + (b_rd ^ (16 * kswz_step<BN>(idx))), integral_constant<int, BN>{});
        else fb[idx] = read_rm(stage_ptr(S) + b_rd + idx * 16 * kBK);
    };

    uint32_t amax_acc = 0;  // AMAX: largest |bf16 output| this wavefront has produced (packed pairs)
    v4f acc[TM][TN];
    auto zero_acc = [&]() {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) acc[i][j] = v4f{0.f, 0.f, 0.f, 0.f};
    };

    // ---- the K step's MFMA order, TM * TN slots.  First half: the upper TM / 2 fragment rows of
    // A, row by row (every B fragment is live, the A fragments die one by one).  Second half: the
    // lower TM / 2 rows, column by column (the B fragments die one by one).  So registers free
    // up for the next K step's fragments while this one still computes, and never more than
    // TM + TN (+ 1) fragments are live: half of what double buffering both operands would take.
    constexpr int SLOTS = TM * TN, HALF = SLOTS / 2, HM = TM / 2;
    constexpr auto slot_i = [](int s) { return s < HALF ? s / TN : HM + (s - HALF) % HM; };
    constexpr auto slot_j = [](int s) { return s < HALF ? s % TN : (s - HALF) / HM; };
    // Written as asm with the accumulator as one read-write operand: left to itself the register
    // allocator gives an MFMA's result and its addend different registers and then shuffles
    // accumulators between the two register files inside the loop.  The first source operand
    // is the B fragment (cbsz = its format), the second the A fragment (blgp): see the top of
    // this file.  Consequence: the compiler does not know these are matrix instructions, so the
    // wait states between the last of them and the first ordinary read of an accumulator are
    // inserted by hand (mfma_drain).
    auto mfma_slot = [&](auto SLOT) {
        constexpr int s = decltype(SLOT)::value, i = slot_i(s), j = slot_j(s);
        v4f& c = acc[i][j];
        const v8i& b = fb[j];
        const v8i& a = fa[i];
        asm volatile("v_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, %0 cbsz:%3 blgp:%4" : "+a"(c) : "v"(b), "v"(a), "n"(FB), "n"(FA));
    };
    // an 8-pass matrix instruction's result may be read by an ordinary instruction 18 wait states
    // after its issue at the earliest, and nothing interlocks that
    auto mfma_drain = [&]() {
        asm volatile("s_nop 15\n\ts_nop 15");
    };
    using I0 = integral_constant<int, 0>;
    using I1 = integral_constant<int, 1>;

    // ---- epilogue of one tile.  Of each 16x16 MFMA tile, lane l holds m = l % 16 and
    // n = 4 * (l / 16) + r for accumulator register r.  Each wave turns a piece of 8 MFMA tiles
    // (16 EPR rows x 16 EPW columns) of its tile at a time into bf16, parks it in its private
    // piece of LDS and writes it out as 16-byte row pieces: every global store instruction then
    // covers whole row segments of 32 EPW bytes (a multiple of the 128-byte line).
    auto epilogue = [&](int item) {
        int tm, tn;
        tile_coords(SPLITK ? item % tiles_mn : item, tiles_m, tiles_n, &tm, &tn);
        const int m0 = tm * BM + wm * WM, n0 = tn * BN + wn * WN;  // of this wave's tile
        if constexpr (SPLITK) {
            // the unscaled sums of this range, as 16-byte pieces (four consecutive n of one m per lane)
            float* P = partial + (int64_t)(item / tiles_mn) * M * ldp;
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int m = m0 + 16 * i + fr;
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const int n = n0 + 16 * j + 4 * fg;
                    if (m < M && n < N)  // N is a multiple of 16: the piece is all in or all out
                        *reinterpret_cast<v4f*>(P + (int64_t)m * ldp + n) = acc[i][j];
                }
            }
            return;
        }
        uint8_t* ep = epb + wave * (16 * EPR * EP_STRIDE);
        float s_tensor = 0.f;
        if constexpr (GRAN == F8_TENSORWISE) s_tensor = isa[0] * isb[0];
        // A lane stores four 16-byte pieces per pass: row (64 / LPR) t + lane / LPR of the pass's
        // rows, columns 8 * (lane % LPR) .. +7 of its columns: uniform base + 32-bit lane offset.
        uint8_t* dbase = reinterpret_cast<uint8_t*>(D + (int64_t)m0 * ldd + n0);
        const uint32_t ldd_b = (uint32_t)ldd * 2;
        constexpr int LPR = 2 * EPW;  // lanes (16-byte pieces) per staged row
        const uint32_t voff = (uint32_t)(lane / LPR) * ldd_b + (uint32_t)(lane % LPR) * 16;
        const bool interior = tm * BM + BM <= M && tn * BN + BN <= N;  // no edge checks needed

        auto run = [&](auto INTERIOR) {
            // One pass = rows 16 EPR ip .., columns 16 EPW jp .. of the wave's tile = EPR x EPW MFMA
            // tiles.  Tensorwise: row bands outermost.  Per-row / per-column scales: column bands
            // outermost, so that the column scales a lane needs are loaded once per band (and
            // the row scales once per tile) instead of in every pass, where their latency would
            // sit in front of each conversion.
            constexpr int NP = (TM / EPR) * (TN / EPW);
            float sav[TM];
            float4 sbv[EPW];
            if constexpr (GRAN != F8_TENSORWISE) {
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    const int m_lane = m0 + 16 * i + fr;
                    sav[i] = isa[m_lane < M ? m_lane : M - 1];
                }
            }
            static_for<NP>([&](auto P) {
                constexpr int p = decltype(P)::value;
                constexpr int ip = GRAN == F8_TENSORWISE ? p / (TN / EPW) : p % (TM / EPR);
                constexpr int jp = GRAN == F8_TENSORWISE ? p % (TN / EPW) : p / (TM / EPR);
                if constexpr (GRAN != F8_TENSORWISE && ip == 0) {
#pragma unroll
                    for (int jj = 0; jj < EPW; ++jj) {
                        int n = n0 + 16 * EPW * jp + 16 * jj + 4 * fg;
                        n = n < N ? n : N - 4;
                        sbv[jj] = *reinterpret_cast<const float4*>(isb + n);
                    }
                }
#pragma unroll
                for (int ii = 0; ii < EPR; ++ii) {
                    const int i = EPR * ip + ii;
#pragma unroll
                    for (int jj = 0; jj < EPW; ++jj) {
                        const int j = EPW * jp + jj;
                        const int nl = 16 * jj + 4 * fg;  // column inside the pass
                        f2 lo, hi;
                        if constexpr (GRAN == F8_TENSORWISE) {
                            lo = f2{acc[i][j][0] * s_tensor, acc[i][j][1] * s_tensor};
                            hi = f2{acc[i][j][2] * s_tensor, acc[i][j][3] * s_tensor};
                        } else {
                            const float sa = sav[i];
                            const float4 sb = sbv[jj];
                            lo = f2{(acc[i][j][0] * sa) * sb.x, (acc[i][j][1] * sa) * sb.y};
                            hi = f2{(acc[i][j][2] * sa) * sb.z, (acc[i][j][3] * sa) * sb.w};
                        }
                        // fp32 -> bf16, round to nearest even (v_cvt_pk_bf16_f32)
                        uint2 o;
                        o.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(lo, b2));
                        o.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(hi, b2));
                        if constexpr (AMAX) {
                            // edge tiles hold results of re-read rows past M / N: not output
                            bool counted = true;
                            if constexpr (!decltype(INTERIOR)::value)
                                counted = m0 + 16 * i + fr < M && n0 + 16 * EPW * jp + nl < N;
                            if (counted) amax_acc = amax_pair(amax_acc, o);
                        }
                        *reinterpret_cast<uint2*>(ep + (16 * ii + fr) * EP_STRIDE + nl * 2) = o;
                    }
                }
                uint8_t* pbase = dbase + ((int64_t)(16 * EPR * ip) * ldd + 16 * EPW * jp) * 2;  // uniform
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const int idx = t * 64 + lane;
                    const uint4 v = *reinterpret_cast<const uint4*>(ep + (idx / LPR) * EP_STRIDE + (idx % LPR) * 16);
                    bool ok = true;
                    if constexpr (!decltype(INTERIOR)::value)
                        ok = m0 + 16 * EPR * ip + idx / LPR < M && n0 + 16 * EPW * jp + (idx % LPR) * 8 < N;
                    // Streaming store: D is not read again by this library, and lines that
                    // linger dirty in the L2 / Infinity Cache would be written back during the
                    // next, bandwidth-bound kernel instead of during this compute-bound one.
                    typedef unsigned int u4v __attribute__((ext_vector_type(4)));
                    if (ok)
                        __builtin_nontemporal_store(u4v{v.x, v.y, v.z, v.w},
                                                    reinterpret_cast<u4v*>(pbase + (voff + (uint32_t)(64 / LPR * t) * ldd_b)));
                }
                // one pass at a time: measured faster than letting the compiler interleave passes
                __builtin_amdgcn_sched_barrier(0);
            });
        };
        if (interior)
            run(std::true_type{});
        else
            run(std::false_type{});
    };

    // The fragments a K step starts with: the upper half of A's and all of B's, from stage S.
    auto read_first_set = [&](auto S) {
        static_for<HM>([&](auto I) { read_a(S, I); });
        static_for<TN>([&](auto J) { read_b(S, J); });
    };

    // ---- prologue: two stages in flight, the first K step's starting fragments into registers
    load_context(ld_tile);  // the grid never exceeds the tile count
    issue_all(0, I0{});
    issue_all(1, I1{});
    zero_acc();
    __builtin_amdgcn_s_waitcnt(kWaitAllVmLgkm);
    __syncthreads();
    read_first_set(I0{});

    // One K step out of stage S = SLOTS MFMA slots in a fixed order (every slot ends with a
    // scheduling fence).  On entry fa[0 .. HM) and all of fb hold this step's fragments.
    //   slots [0, HM):         + LDS reads of this step's lower A fragments fa[HM .. TM) (stage S)
    //   after slot SYNC_A-1:   barrier: every wave is done reading stage S
    //   slots [SYNC_A, L_END): + the loads that refill stage S with the stream's next K step,
    //                          at most one per slot and with gaps: a wave's load blocks its
    //                          instruction issue until the CU's address unit accepts it (16 cycles
    //                          per 1 KB load, shared by the four waves), so bunched loads would
    //                          starve the matrix pipe
    //   after slot SYNC_B-1:   wait until only this step's PRE_B loads are in flight (the
    //                          previous step's have then landed), barrier: the other stage is
    //                          complete for every wave
    //   slots [HALF, SLOTS):   + LDS reads of the next K step's starting fragments from the other
    //                          stage, each into the registers of a fragment that has just died:
    //                          the upper A fragments at once, B fragment j when column j is done
    // The MFMAs issued just before a barrier keep the matrix pipe busy while the wave waits.
    constexpr int SYNC_A = HM + (SLOTS >= 64 ? 8 : SLOTS >= 32 ? 4 : 1);  // the reads of slots [0, HM) are back by then
    constexpr int SYNC_B = HALF - 2;
    constexpr int LOADS = A_LOADS + B_LOADS;
    // spread thinly, but done an eighth of the step before its end: the last loads then have a few
    // hundred cycles more to land before the next step's second barrier waits for them (measured:
    // +1 to 4 % on products with k-major operands and a long contraction, nothing lost elsewhere)
    constexpr int L_END = SLOTS >= 64 ? SLOTS - SLOTS / 8 : SLOTS;
    static_assert(SYNC_A <= SYNC_B && L_END - SYNC_A >= LOADS / 2, "schedule does not fit");
    constexpr auto slot_of_load = [](int l) { return SYNC_A + l * (L_END - SYNC_A) / LOADS; };
    constexpr int PRE_B = [&] {
        int n = 0;
        for (int l = 0; l < LOADS; ++l) n += slot_of_load(l) < SYNC_B;
        return n;
    }();
    // B fragment j dies with the last MFMA of column j; the last columns' successors are read a
    // little early (into spare registers) so that they are back when the next step needs them
    constexpr auto slot_of_next_b = [](int j) {
        const int s = HALF + (j + 1) * HM - 1;
        return s < SLOTS - 3 ? s : SLOTS - 3;
    };
    // s_waitcnt vmcnt(PRE_B) lgkmcnt(0)
    constexpr int kWaitB = (PRE_B & 15) | ((PRE_B >> 4) << 14) | 0x0070;

    auto kstep = [&](auto S, int fetch_kt) {
        constexpr int s = decltype(S)::value;
        using OTHER = integral_constant<int, 1 - s>;
        const uint8_t* ga = step_base_a(fetch_kt);
        const uint8_t* gb = step_base_b(fetch_kt);
        static_for<SLOTS>([&](auto SLOT) {
            constexpr int slot = decltype(SLOT)::value;
            if constexpr (slot == SYNC_A) {
                __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): my reads of stage S are back
                __syncthreads();
                __builtin_amdgcn_sched_barrier(0);
            }
            if constexpr (slot == SYNC_B) {
                __builtin_amdgcn_s_waitcnt(kWaitB);
                __syncthreads();
                __builtin_amdgcn_sched_barrier(0);
            }
            mfma_slot(SLOT);
            if constexpr (slot < HM) read_a(S, integral_constant<int, HM + slot>{});
            if constexpr (slot >= HALF && slot < HALF + HM) read_a(OTHER{}, integral_constant<int, slot - HALF>{});
            static_for<TN>([&](auto J) {
                constexpr int j = decltype(J)::value;
                if constexpr (slot_of_next_b(j) == slot) {
                    if constexpr (slot < HALF + (j + 1) * HM - 1) {  // fb[j] is still needed: park its successor
                        static_assert(j == TN - 1, "one spare fragment");
                        const v8i keep = fb[j];
                        read_b(OTHER{}, J);
                        fb_early = fb[j];
                        fb[j] = keep;
                    } else {
                        read_b(OTHER{}, J);
                    }
                }
            });
            if constexpr (slot == SLOTS - 1 && slot_of_next_b(TN - 1) < SLOTS - 1) fb[TN - 1] = fb_early;
            static_for<LOADS>([&](auto L) {
                if constexpr (slot_of_load(decltype(L)::value) == slot) issue_one(ga, gb, S, L);
            });
            __builtin_amdgcn_sched_barrier(0);
        });
    };

    // ---- main loop over this workgroup's tiles.  KT is even, so every tile starts in stage 0.
    // The step computed at kt fetches step kt + 2; the last two steps of a tile fetch the first
    // two of the next tile.
    for (int tile = blockIdx.x; tile < total_tiles; tile += gridDim.x) {
        // Retire every earlier vector-memory operation (the previous tile's stores, register
        // spills) once per tile.  Otherwise the compiler, which must protect the data
        // registers of pending stores, places its own full wait inside the K loop, where it
        // would also wait for the freshly issued loads on every step.  The loads in flight
        // here are this tile's first two K steps, requested a whole epilogue ago.
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
        for (int kt = 0; kt < KT; kt += 2) {
            if (kt == KT - 2) next_load_tile();  // the last two steps fetch the next tile's first two
            const int f = kt == KT - 2 ? 0 : kt + 2;
            kstep(I0{}, f);
            kstep(I1{}, f + 1);
        }
        mfma_drain();
        epilogue(tile);
        zero_acc();
        // The next tile's starting fragments are read again here rather than kept in registers
        // across the epilogue (the last K step already fetched them once): registers less for
        // the epilogue to fight over.  Stage 0 is complete since that step's second barrier.
        read_first_set(I0{});
        asm volatile("s_nop 7");  // accumulators just written by ordinary instructions: let them settle
    }
    // no load may still be writing LDS when the workgroup ends
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    if constexpr (AMAX) {
        __syncthreads();  // every wave is past its last epilogue pass: the staging buffer is free
        amax_publish<NW>(amax_acc, amax_bits, reinterpret_cast<uint32_t*>(epb));
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
    const float* __restrict__ isb, uint32_t* __restrict__ amax_bits)
{
    __shared__ __attribute__((aligned(16))) uint8_t As[kGT * kGStride];
    __shared__ __attribute__((aligned(16))) uint8_t Bs[kGT * kGStride];
    // one-dimensional grid (the y dimension of a grid stops at 65535 blocks): tile = m-tile * tiles_n + n-tile
    const int tiles_n = (N + kGT - 1) / kGT;
    const int m0 = (int)(blockIdx.x / (unsigned)tiles_n) * kGT, n0 = (int)(blockIdx.x % (unsigned)tiles_n) * kGT;
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
    uint32_t amax_acc = 0;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int m = m0 + wm * 32 + 16 * i + fr;
        if (m >= M) continue;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int n = n0 + wn * 32 + 16 * j + 4 * fg;
            if (n < N) amax_acc = amax_pair(amax_acc, store4<GRAN>(D, ldd, m, n, acc[i][j], s_tensor, isa, isb));
        }
    }
    if (amax_bits) {  // uniform branch; every thread of the block takes part
        __syncthreads();
        amax_publish<4>(amax_acc, amax_bits, reinterpret_cast<uint32_t*>(As));
    }
}

// ---------------------------------------------------------------------------
// split-K: sum of the ranges' partial results, scales, bf16
// ---------------------------------------------------------------------------
// partial[s][M][ldp] fp32, s < splits, added in the order s = 0, 1, ... (fixed: results are
// reproducible run to run).  A thread owns eight consecutive n of one m.
template <int GRAN>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ partial, int splits, int M,
                                                            int N, int64_t ldp, const float* __restrict__ isa,
                                                            const float* __restrict__ isb, uint16_t* __restrict__ D,
                                                            int64_t ldd)
{
    const int chunks = N / 8;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)M * chunks) return;
    const int m = (int)(idx / chunks), n = (int)(idx % chunks) * 8;
    const float* p = partial + (int64_t)m * ldp + n;
    const int64_t stride = (int64_t)M * ldp;
    v4f lo = *reinterpret_cast<const v4f*>(p), hi = *reinterpret_cast<const v4f*>(p + 4);
    for (int s = 1; s < splits; ++s) {
        lo += *reinterpret_cast<const v4f*>(p + s * stride);
        hi += *reinterpret_cast<const v4f*>(p + s * stride + 4);
    }
    float r[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    if constexpr (GRAN == F8_TENSORWISE) {
        const float st = isa[0] * isb[0];
#pragma unroll
        for (int i = 0; i < 8; ++i) r[i] *= st;
    } else {
        const float sa = isa[m];
        const float4 s0 = *reinterpret_cast<const float4*>(isb + n), s1 = *reinterpret_cast<const float4*>(isb + n + 4);
        const float sb[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
#pragma unroll
        for (int i = 0; i < 8; ++i) r[i] = (r[i] * sa) * sb[i];
    }
    uint4 o;
    o.x = f32_to_bf16_bits(r[0]) | (f32_to_bf16_bits(r[1]) << 16);
    o.y = f32_to_bf16_bits(r[2]) | (f32_to_bf16_bits(r[3]) << 16);
    o.z = f32_to_bf16_bits(r[4]) | (f32_to_bf16_bits(r[5]) << 16);
    o.w = f32_to_bf16_bits(r[6]) | (f32_to_bf16_bits(r[7]) << 16);
    *reinterpret_cast<uint4*>(D + (int64_t)m * ldd + n) = o;
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------

template <int BM, int BN, int WAVES_M, int WAVES_N, int FA, int FB, int GRAN, bool AKM, bool BKM>
static void launch_tile(int M, int N, int K, const uint8_t* A, int64_t lda, const uint8_t* B, int64_t ldb,
                        const float* isa, const float* isb, uint16_t* D, int64_t ldd, uint32_t* amax_bits,
                        int max_blocks, hipStream_t st)
{
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const int total = tiles_m * tiles_n;
    const int grid = total < max_blocks ? total : max_blocks;
    if (amax_bits)
        gemm_tile_kernel<BM, BN, WAVES_M, WAVES_N, FA, FB, GRAN, true, AKM, BKM><<<grid, WAVES_M * WAVES_N * 64, 0, st>>>(
            A, B, D, M, N, K, lda, ldb, ldd, isa, isb, tiles_m, tiles_n, amax_bits);
    else
        gemm_tile_kernel<BM, BN, WAVES_M, WAVES_N, FA, FB, GRAN, false, AKM, BKM><<<grid, WAVES_M * WAVES_N * 64, 0, st>>>(
            A, B, D, M, N, K, lda, ldb, ldd, isa, isb, tiles_m, tiles_n, nullptr);
}

static int cu_count()
{
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
        n = 256;
    return n - n % kXcds;  // the persistent tile order assumes a multiple of the XCD count
}

// Number of contraction ranges for a product whose 256x256 tiles would occupy at most half of
// the compute units, or 1.  A range must be a multiple of 256 (two LDS stages) and at least 1024
// long, ranges x tiles must fit the compute units (one work item each), and the partial results
// must fit the workspace.  Chosen by estimated time, in units of one whole-K 256x256 tile:
// 1 / ranges + 0.04 for the fp32 epilogue + the reduction pass (a launch, ranges + 1/2 passes
// over an M x N fp32 matrix at about 5 TB/s) against the best unsplit configuration.
static int splitk_ranges(int M, int N, int K, int cus, double best_unsplit, size_t ws_bytes)
{
    const int64_t T = (int64_t)((M + 255) / 256) * ((N + 255) / 256);
    if (2 * T > cus || K < 2048) return 1;
    const double tile_us = (double)(K / kBK) * 1.05;  // a K step of a 256x256 tile takes about 2100 cycles
    int best = 1;
    double best_cost = best_unsplit;
    for (int s = 2; s <= 8; s *= 2) {
        if (s * T > cus || K % (s * 2 * kBK) || K / s < 1024) break;
        if ((size_t)s * (size_t)M * (size_t)N * sizeof(float) > ws_bytes) break;
        const double reduce_us = 3.0 + (s + 0.5) * (double)M * (double)N * 4.0 / 5.0e6;
        const double cost = 1.0 / s + 0.04 + reduce_us / tile_us;
        if (cost < best_cost) best = s, best_cost = cost;
    }
    return best;
}

template <int FA, int FB, int GRAN, bool AKM, bool BKM>
static void dispatch_tile(int M, int N, int K, const uint8_t* A, int64_t lda, const uint8_t* B, int64_t ldb,
                          const float* isa, const float* isb, uint16_t* D, int64_t ldd, uint32_t* amax_bits,
                          void* ws, size_t ws_bytes, hipStream_t st)
{
    // Tile configuration by estimated time, in units of one 256x256 tile's time on one compute
    // unit: T tiles on `cus` persistent workgroups take ceil(T / cus) rounds; a 256x128 tile costs
    // about 0.63 and a 128x128 tile about 0.58 of a 256x256 one (measured: their wave tiles need
    // more LDS bytes per MFMA).  Ties go to the larger tile.
    const int cus = cu_count();
    auto tiles = [&](int bm, int bn) { return (int64_t)((M + bm - 1) / bm) * ((N + bn - 1) / bn); };
    auto rounds = [&](int64_t t) { return (double)((t + cus - 1) / cus); };
    constexpr double kHalfTile = 0.63, kQuarterTile = 0.58;
    const int tm = (M + 255) / 256, tn = (N + 255) / 256;
    const int64_t T = (int64_t)tm * tn, whole = T / cus * cus, rest = T - whole;
    // Wave quantisation: a last round with at most half of the workgroups busy (e.g. 896 tiles =
    // 3.5 rounds) costs a whole one.  Then the whole rounds are launched on their own sub-matrix
    // (a range of tile rows or tile columns holding exactly `whole` tiles) and the rest with
    // 256x128 tiles: twice as many, still at most one per workgroup.
    const bool split_rows = whole > 0 && rest > 0 && 2 * rest <= cus && whole % tn == 0;
    const bool split_cols = !split_rows && whole > 0 && rest > 0 && 2 * rest <= cus && whole % tm == 0;
    const double c_full = (split_rows || split_cols) ? (double)(whole / cus) + kHalfTile : rounds(T);
    const double c_half = rounds(tiles(256, 128)) * kHalfTile;
    const double c_quarter = rounds(tiles(128, 128)) * kQuarterTile;
    const bool rw = GRAN != F8_TENSORWISE;
    if (ws && !amax_bits) {
        const double best = c_full < c_half ? (c_full < c_quarter ? c_full : c_quarter) : (c_half < c_quarter ? c_half : c_quarter);
        const int ranges = splitk_ranges(M, N, K, cus, best, ws_bytes);
        if (ranges > 1) {
            float* partial = static_cast<float*>(ws);
            gemm_tile_kernel<256, 256, 2, 2, FA, FB, GRAN, false, AKM, BKM, true><<<(unsigned)(T * ranges), 256, 0, st>>>(
                A, B, D, M, N, K, lda, ldb, ldd, isa, isb, tm, tn, nullptr, ranges, partial, (int64_t)N);
            const int64_t threads = (int64_t)M * (N / 8);
            splitk_reduce_kernel<GRAN><<<(unsigned)((threads + 255) / 256), 256, 0, st>>>(partial, ranges, M, N, (int64_t)N,
                                                                                         isa, isb, D, ldd);
            return;
        }
    }
#define F8_TILE(BM_, BN_) launch_tile<BM_, BN_, 2, 2, FA, FB, GRAN, AKM, BKM>
    if (c_full <= c_half && c_full <= c_quarter) {
        if (split_rows) {
            const int m1 = (int)(whole / tn) * 256;
            // rows m1 .. M-1 of A: m1 rows down (row-major) or m1 bytes along each k-row (k-major)
            const uint8_t* A2 = AKM ? A + m1 : A + (int64_t)m1 * lda;
            F8_TILE(256, 256)(m1, N, K, A, lda, B, ldb, isa, isb, D, ldd, amax_bits, cus, st);
            F8_TILE(256, 128)(M - m1, N, K, A2, lda, B, ldb, rw ? isa + m1 : isa, isb, D + (int64_t)m1 * ldd, ldd,
                              amax_bits, cus, st);
        } else if (split_cols) {
            const int n1 = (int)(whole / tm) * 256;
            const uint8_t* B2 = BKM ? B + n1 : B + (int64_t)n1 * ldb;
            F8_TILE(256, 256)(M, n1, K, A, lda, B, ldb, isa, isb, D, ldd, amax_bits, cus, st);
            F8_TILE(256, 128)(M, N - n1, K, A, lda, B2, ldb, isa, rw ? isb + n1 : isb, D + n1, ldd, amax_bits, cus, st);
        } else {
            F8_TILE(256, 256)(M, N, K, A, lda, B, ldb, isa, isb, D, ldd, amax_bits, cus, st);
        }
    } else if (c_half <= c_quarter) {
        F8_TILE(256, 128)(M, N, K, A, lda, B, ldb, isa, isb, D, ldd, amax_bits, cus, st);
    } else {
        // LDS allows two 128x128 workgroups per compute unit
        F8_TILE(128, 128)(M, N, K, A, lda, B, ldb, isa, isb, D, ldd, amax_bits, 2 * cus, st);
    }
#undef F8_TILE
}

template <int LAYOUT, int FA, int FB, int GRAN>
static void launch_generic(int M, int N, int K, const uint8_t* A, int64_t lda, const uint8_t* B, int64_t ldb,
                           const float* isa, const float* isb, uint16_t* D, int64_t ldd, uint32_t* amax_bits,
                           hipStream_t st)
{
    const unsigned grid = (unsigned)((int64_t)((N + kGT - 1) / kGT) * ((M + kGT - 1) / kGT));
    gemm_generic_kernel<LAYOUT, FA, FB, GRAN><<<grid, 256, 0, st>>>(A, B, D, M, N, K, lda, ldb, ldd, isa, isb,
                                                                    amax_bits);
}

// One layout of one operand-format pair: the fast kernel when the contraction length allows it
// (it alternates two LDS stages of 128 per tile), else the generic one.
template <int LAYOUT, int FA, int FB, int GRAN>
static void dispatch_layout(int M, int N, int K, const uint8_t* A, int64_t lda, const uint8_t* B, int64_t ldb,
                            const float* isa, const float* isb, uint16_t* D, int64_t ldd, uint32_t* amax_bits,
                            void* ws, size_t ws_bytes, hipStream_t st)
{
    if (K % (2 * kBK) == 0 && K > 0)
        dispatch_tile<FA, FB, GRAN, LAYOUT == F8_TN, LAYOUT != F8_NT>(M, N, K, A, lda, B, ldb, isa, isb, D, ldd,
                                                                       amax_bits, ws, ws_bytes, st);
    else
        launch_generic<LAYOUT, FA, FB, GRAN>(M, N, K, A, lda, B, ldb, isa, isb, D, ldd, amax_bits, st);
}

// All launches of one operand-format pair and layout: the granularity is a run-time choice.
template <int LAYOUT, int FA, int FB>
static void gemm_formats(int g, int M, int N, int K, const uint8_t* A, int64_t lda, const uint8_t* B, int64_t ldb,
                         const float* isa, const float* isb, uint16_t* D, int64_t ldd, uint32_t* amax_bits,
                         void* ws, size_t ws_bytes, hipStream_t st)
{
    if (g == F8_TENSORWISE)
        dispatch_layout<LAYOUT, FA, FB, F8_TENSORWISE>(M, N, K, A, lda, B, ldb, isa, isb, D, ldd, amax_bits, ws, ws_bytes, st);
    else
        dispatch_layout<LAYOUT, FA, FB, F8_ROWWISE>(M, N, K, A, lda, B, ldb, isa, isb, D, ldd, amax_bits, ws, ws_bytes, st);
}

}  // namespace f8
