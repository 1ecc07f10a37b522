// Causal grouped-query attention in bf16 between the Float8 linears of a transformer block
// (Section 2.2.4 applies Float8 to the linear layers only: everything else stays in bf16).  Flash-style: scores are never
// written; bf16 MFMA (v_mfma_f32_32x32x16_bf16) with fp32 accumulation and an online softmax.
//
// Orientation.  Of a 32x32 MFMA result, a lane holds one column (the row index of the SECOND
// operand) and 16 rows (row indices of the FIRST operand: 8 * (r / 4) + 4 * (lane / 32) + r % 4
// for register r).  The kernels form S^T = K Q^T (keys along registers, one query per lane), so
// the softmax statistics of a query live in one lane (plus its partner lane + 32), and the
// probabilities are already laid out as the operand of the next product, whose contraction runs
// over keys: 8 consecutive registers are the 8 contraction slots of a lane.  The other operand
// only has to present the same keys in the same slots: it is read from a copy that is contiguous
// along tokens (V^T here; Q^T, K^T, dO^T in the backward), which the producers write on the way
// (f8_rope's transposed output, f8_transpose_bf16).  No operand is transposed in registers.
#include <atomic>

#include "f8_device.hpp"
#include "f8_host.hpp"

namespace f8 {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kAttnThreads = 256;
constexpr int kHd = 128;   // head dimension of every model the paper trains
constexpr int kBk = 64;    // keys per step
// operand reads ahead of their product (deeper did not help)
constexpr int kFwdAhead = 4, kDqAhead = 4, kDkvAhead = 4;
constexpr int kKp = kHd + 8;   // LDS row pitch (bf16) of a [tokens][hd] tile: 272 bytes
constexpr int kTp = kBk + 4;   // LDS row pitch (bf16) of a [hd][tokens] tile: 136 bytes = 34 words, an odd multiple of 2:
                               // the 8-byte reads of 32 consecutive rows fall into 32 different bank pairs

template <bool B>
struct BoolC {
    static constexpr bool value = B;
};

__device__ inline f32x16 mma(uint4 first, uint4 second, f32x16 acc)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, first), __builtin_bit_cast(bf16x8, second), acc,
                                                   0, 0, 0);
}

__device__ inline uint32_t pack2(float lo, float hi)
{
    // v_cvt_pk_bf16_f32: round to nearest even
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    bf16x2 r = {(__bf16)lo, (__bf16)hi};
    return __builtin_bit_cast(uint32_t, r);
}

// registers 8u .. 8u+7 of an accumulator as a bf16 operand (8 contraction slots)
__device__ inline uint4 slots(const f32x16& c, int u)
{
    return make_uint4(pack2(c[8 * u], c[8 * u + 1]), pack2(c[8 * u + 2], c[8 * u + 3]), pack2(c[8 * u + 4], c[8 * u + 5]),
                      pack2(c[8 * u + 6], c[8 * u + 7]));
}

// the operand that matches slots(c, u) of a 32-token block starting at column t0 of a
// [rows][tokens] LDS tile: tokens t0 + 16u + 4g + {0..3} and t0 + 16u + 8 + 4g + {0..3}
__device__ inline uint4 token_slots(const uint16_t* tile_row, int t0, int u, int g)
{
    const uint2 a = *reinterpret_cast<const uint2*>(tile_row + t0 + 16 * u + 4 * g);
    const uint2 b = *reinterpret_cast<const uint2*>(tile_row + t0 + 16 * u + 8 + 4 * g);
    return make_uint4(a.x, a.y, b.x, b.y);
}

// N products use(i, frag(i)) whose LDS operand reads (one DS instruction each) run AHEAD products
// ahead of their use.  Left to itself the scheduler reads each operand right before its product
// and every product waits out the LDS latency; the group barriers pin the interleaving.
template <int N, int AHEAD, class Frag, class Use>
__device__ inline void pipelined_products(Frag frag, Use use)
{
    uint4 f[N];
#pragma unroll
    for (int i = 0; i < AHEAD && i < N; ++i) f[i] = frag(i);
    __builtin_amdgcn_sched_group_barrier(0x100, AHEAD < N ? AHEAD : N, 0);  // DS reads
#pragma unroll
    for (int i = 0; i < N; ++i) {
        if (i + AHEAD < N) f[i + AHEAD] = frag(i + AHEAD);
        use(i, f[i]);
        if (i + AHEAD < N) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                  // one MFMA
    }
}

// Tile loaders: global -> registers (issued early) -> LDS (after the barrier that frees it).
// [ROWS tokens][kHd] from a token-major tensor; rows at or beyond `limit` read as zero.
template <int ROWS, int NT = kAttnThreads>
struct RowTile {
    static constexpr int N = ROWS * (kHd / 8) / NT;
    static_assert(N >= 1 && N * NT == ROWS * (kHd / 8), "the tile's chunks divide evenly over the threads");
    uint4 v[N];
    __device__ void load(const uint16_t* base, int64_t ld, int row0, int limit)
    {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int c = threadIdx.x + NT * i, r = c / (kHd / 8), cc = c % (kHd / 8);
            v[i] = (row0 + r < limit) ? *reinterpret_cast<const uint4*>(base + (int64_t)(row0 + r) * ld + cc * 8) : make_uint4(0, 0, 0, 0);
        }
    }
    __device__ void store(uint16_t* lds) const
    {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int c = threadIdx.x + NT * i, r = c / (kHd / 8), cc = c % (kHd / 8);
            *reinterpret_cast<uint4*>(lds + r * kKp + cc * 8) = v[i];
        }
    }
};
// [kHd][COLS tokens] from a transposed (token-minor) tensor with row pitch ld; columns at or beyond
// `limit` read as zero (limit and col0 are multiples of 8).
template <int COLS, int NT = kAttnThreads>
struct ColTile {
    static constexpr int N = kHd * (COLS / 8) / NT;
    static_assert(N >= 1 && N * NT == kHd * (COLS / 8), "the tile's chunks divide evenly over the threads");
    static constexpr int P = COLS + 4;  // rows are 8-byte aligned only: stored as two 8-byte halves
    uint4 v[N];
    __device__ void load(const uint16_t* base, int64_t ld, int col0, int limit)
    {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int c = threadIdx.x + NT * i, r = c / (COLS / 8), cc = c % (COLS / 8);
            v[i] = (col0 + cc * 8 < limit) ? *reinterpret_cast<const uint4*>(base + (int64_t)r * ld + col0 + cc * 8) : make_uint4(0, 0, 0, 0);
        }
    }
    __device__ void store(uint16_t* lds) const
    {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int c = threadIdx.x + NT * i, r = c / (COLS / 8), cc = c % (COLS / 8);
            *reinterpret_cast<uint2*>(lds + r * P + cc * 8) = make_uint2(v[i].x, v[i].y);
            *reinterpret_cast<uint2*>(lds + r * P + cc * 8 + 4) = make_uint2(v[i].z, v[i].w);
        }
    }
};

// ---- forward ------------------------------------------------------------------------------
// One block: NW waves of 32 queries each of one (sequence, head).  Loop over 64-key
// steps up to the diagonal; K and V^T tiles double-buffered in LDS, the next step's tiles
// prefetched into registers while this step computes.
template <int NW>
__global__ __launch_bounds__(64 * NW, 512 / (64 * NW)) void sdpa_fwd_kernel(const uint16_t* __restrict__ Q, int64_t ldq,
                                                                const uint16_t* __restrict__ K, int64_t ldk,
                                                                const uint16_t* __restrict__ Vt, int64_t M, int S, int Hq,
                                                                int group, float scale_log2e, uint16_t* __restrict__ O,
                                                                int64_t ldo, float* __restrict__ lse, int nqt,
                                                                uint32_t* __restrict__ amax_bits /* nullable */)
{
    constexpr int NT = 64 * NW, QB = 32 * NW;  // threads and queries per block
    __shared__ __attribute__((aligned(16))) uint16_t sK[2][kBk * kKp];
    __shared__ __attribute__((aligned(16))) uint16_t sV[2][kHd * kTp];

    // long (late) query tiles first, over all heads: the tile index varies slowest
    const int nbh = Hq * (int)(M / S), qt = nqt - 1 - (int)(blockIdx.x / nbh);
    const int bh = blockIdx.x % nbh, h = bh % Hq, b = bh / Hq, kvh = h / group;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, ln = lane & 31, g = lane >> 5;
    const int q_first = qt * QB + wave * 32;  // of this wave
    const int q_pos = q_first + ln;            // position of this lane's query in its sequence
    const int64_t tok0 = (int64_t)b * S;
    const uint16_t* Kb = K + tok0 * ldk + (int64_t)kvh * kHd;
    const uint16_t* Vb = Vt + (int64_t)kvh * kHd * M + tok0;

    uint4 qf[kHd / 16];
    {
        const bool ok = q_pos < S;
        const uint16_t* row = Q + (tok0 + (ok ? q_pos : 0)) * ldq + (int64_t)h * kHd + 8 * g;
#pragma unroll
        for (int s = 0; s < kHd / 16; ++s) qf[s] = ok ? *reinterpret_cast<const uint4*>(row + 16 * s) : make_uint4(0, 0, 0, 0);
    }

    int key_end = (qt + 1) * QB;  // keys at or beyond it are masked for every query of the block
    if (key_end > S) key_end = S;
    const int nkt = (key_end + kBk - 1) / kBk;

    f32x16 acc_o[kHd / 32];
#pragma unroll
    for (int d = 0; d < kHd / 32; ++d) acc_o[d] = f32x16{0};
    float m_run = -INFINITY, l_run = 0.0f;  // running maximum of the raw scores and this lane's share of the sum

    RowTile<kBk, NT> kt_regs;
    ColTile<kBk, NT> vt_regs;
    kt_regs.load(Kb, ldk, 0, S);
    vt_regs.load(Vb, M, 0, S);
    for (int t = 0; t < nkt; ++t) {
        const int buf = t & 1, key0 = t * kBk;
        kt_regs.store(sK[buf]);
        vt_regs.store(sV[buf]);
        __syncthreads();
        if (t + 1 < nkt) {
            kt_regs.load(Kb, ldk, key0 + kBk, S);
            vt_regs.load(Vb, M, key0 + kBk, S);
        }
        if (key0 > q_first + 31) continue;  // every key of the step lies after every query of the wave

        // S^T = K Q^T: [64 keys][32 queries] as two 32x32 results
        f32x16 sc[2] = {f32x16{0}, f32x16{0}};
        pipelined_products<2 * (kHd / 16), kFwdAhead>(
            [&](int i) { return *reinterpret_cast<const uint4*>(&sK[buf][(32 * (i / 8) + ln) * kKp + 16 * (i % 8) + 8 * g]); },
            [&](int i, uint4 kf) { sc[i / 8] = mma(kf, qf[i % 8], sc[i / 8]); });
        // The maximum is taken over the raw scores (the scale is positive), so the scaling and the
        // subtraction of the maximum are one fused multiply-add per score.
        const bool diagonal = key0 + kBk - 1 > q_first;
        float mx = -INFINITY;
        if (diagonal) {  // wave-uniform: only the steps at the diagonal have anything to mask
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = key0 + 32 * kb + 8 * (r >> 2) + 4 * g + (r & 3);
                    if (key > q_pos) sc[kb][r] = -INFINITY;
                }
        }
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sc[kb][r]);
        mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
        const float m_new = fmaxf(m_run, mx);  // finite: key 0 is visible to every query
        const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * scale_log2e);
        m_run = m_new;
        const float neg_m = -m_new * scale_log2e;
        float psum = 0.0f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[kb][r], scale_log2e, neg_m));
                sc[kb][r] = p;
                psum += p;
            }
        l_run = l_run * alpha + psum;
        if (__builtin_amdgcn_ballot_w64(alpha != 1.0f)) {  // after the first few steps the maximum rarely moves
#pragma unroll
            for (int d = 0; d < kHd / 32; ++d)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc_o[d][r] *= alpha;
        }

        // O^T += V^T P^T: [128 hd][32 queries], contraction over the 64 keys in four 16-slot steps
        const uint4 pf[4] = {slots(sc[0], 0), slots(sc[0], 1), slots(sc[1], 0), slots(sc[1], 1)};  // [2 kb + u]
        pipelined_products<16, kFwdAhead>(
            [&](int i) { return token_slots(&sV[buf][(32 * (i % 4) + ln) * kTp], 32 * (i / 8), (i / 4) % 2, g); },
            [&](int i, uint4 vf) { acc_o[i % 4] = mma(vf, pf[i / 4], acc_o[i % 4]); });
    }

    const float l_tot = l_run + __shfl_xor(l_run, 32, kWave);
    uint32_t mag = 0;  // packed pair of the largest 15-bit magnitudes written
    if (q_pos < S) {
        const float inv = 1.0f / l_tot;
        uint16_t* orow = O + (tok0 + q_pos) * ldo + (int64_t)h * kHd + 4 * g;
#pragma unroll
        for (int d = 0; d < kHd / 32; ++d)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint2 w = make_uint2(pack2(acc_o[d][4 * j] * inv, acc_o[d][4 * j + 1] * inv),
                                           pack2(acc_o[d][4 * j + 2] * inv, acc_o[d][4 * j + 3] * inv));
                *reinterpret_cast<uint2*>(orow + 32 * d + 8 * j) = w;
                mag = pkmax(pkmax(mag, w.x & 0x7FFF7FFFu), w.y & 0x7FFF7FFFu);
            }
        if (g == 0) lse[(int64_t)h * M + tok0 + q_pos] = (m_run * scale_log2e + __builtin_amdgcn_logf(l_tot)) * 0.69314718055994530942f;
    }
    if (amax_bits) {
        // the exact maximum magnitude of the bf16 values written, as float bits: a maximum of
        // non-negative floats is a maximum of their bit patterns, and does not depend on the order
        const uint32_t m = wave_max_u32(pk_collapse(mag)) << 16;
        if (lane == 0 && m > __atomic_load_n(amax_bits, __ATOMIC_RELAXED)) atomicMax(amax_bits, m);
    }
}

__global__ void zero_amax_kernel(uint32_t* p) { p[0] = 0; }

// ---- backward -----------------------------------------------------------------------------
// With P = exp(S / sqrt(hd) - lse) recomputed from the saved lse and delta[q] = sum_d dO O:
//   dV = P^T dO,  dP = dO V^T,  dS = P (dP - delta),  dQ = dS K / sqrt(hd),  dK = dS^T Q / sqrt(hd)
// Three kernels, none with atomics: dQ per query tile (loop over keys, S^T orientation, which
// also produces delta), then dK and dV per key tile and query head (loop over queries, S
// orientation: one key per lane); with grouped heads the shares of a group's query heads are
// kept in fp32 and summed in head order by a small fourth kernel.

// dQ^T = K^T dS^T.  Per 64-key step: S^T = K Q^T, dP^T = V dO^T, dS^T, then the product over keys.
template <int NW>
__global__ __launch_bounds__(64 * NW, 512 / (64 * NW)) void sdpa_bwd_dq_kernel(
    const uint16_t* __restrict__ Q, int64_t ldq, const uint16_t* __restrict__ K, int64_t ldk, const uint16_t* __restrict__ Kt,
    const uint16_t* __restrict__ V, int64_t ldv, const uint16_t* __restrict__ O, int64_t ldo, const uint16_t* __restrict__ dO,
    int64_t lddo, const float* __restrict__ lse, int64_t M, int S, int Hq, int group, float scale_log2e, float scale,
    uint16_t* __restrict__ dQ, int64_t lddq, float* __restrict__ delta, int nqt)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
    constexpr int NT = 64 * NW, QB = 32 * NW;  // threads and queries per block
    constexpr int kBufElems = 2 * kBk * kKp + kHd * kTp;  // K rows, V rows, K^T; twice: the next step's
                                                          // tiles are stored while slower waves still read this step's

    const int nbh = Hq * (int)(M / S), qt = nqt - 1 - (int)(blockIdx.x / nbh);
    const int bh = blockIdx.x % nbh, h = bh % Hq, b = bh / Hq, kvh = h / group;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, ln = lane & 31, g = lane >> 5;
    const int q_first = qt * QB + wave * 32, q_pos = q_first + ln;
    const int64_t tok0 = (int64_t)b * S;
    const uint16_t* Kb = K + tok0 * ldk + (int64_t)kvh * kHd;
    const uint16_t* Vb = V + tok0 * ldv + (int64_t)kvh * kHd;
    const uint16_t* Ktb = Kt + (int64_t)kvh * kHd * M + tok0;
    const bool q_ok = q_pos < S;
    const int64_t tok = tok0 + (q_ok ? q_pos : 0);

    uint4 qf[kHd / 16], dof[kHd / 16];
    float dl = 0.0f;
    {
        const uint16_t* qrow = Q + tok * ldq + (int64_t)h * kHd + 8 * g;
        const uint16_t* drow = dO + tok * lddo + (int64_t)h * kHd + 8 * g;
        const uint16_t* orow = O + tok * ldo + (int64_t)h * kHd + 8 * g;
#pragma unroll
        for (int s = 0; s < kHd / 16; ++s) {
            qf[s] = q_ok ? *reinterpret_cast<const uint4*>(qrow + 16 * s) : make_uint4(0, 0, 0, 0);
            dof[s] = q_ok ? *reinterpret_cast<const uint4*>(drow + 16 * s) : make_uint4(0, 0, 0, 0);
            const uint4 ov = q_ok ? *reinterpret_cast<const uint4*>(orow + 16 * s) : make_uint4(0, 0, 0, 0);
            const uint32_t dw[4] = {dof[s].x, dof[s].y, dof[s].z, dof[s].w}, ow[4] = {ov.x, ov.y, ov.z, ov.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) dl += bf16_lo(dw[j]) * bf16_lo(ow[j]) + bf16_hi(dw[j]) * bf16_hi(ow[j]);
        }
    }
    dl += __shfl_xor(dl, 32, kWave);
    if (q_ok && g == 0) delta[(int64_t)h * M + tok] = dl;
    const float lse2 = q_ok ? lse[(int64_t)h * M + tok] * 1.4426950408889634074f : 0.0f;

    int key_end = (qt + 1) * QB;
    if (key_end > S) key_end = S;
    const int nkt = (key_end + kBk - 1) / kBk;

    f32x16 acc[kHd / 32];
#pragma unroll
    for (int d = 0; d < kHd / 32; ++d) acc[d] = f32x16{0};

    RowTile<kBk, NT> k_regs, v_regs;
    ColTile<kBk, NT> kt_regs;
    k_regs.load(Kb, ldk, 0, S);
    v_regs.load(Vb, ldv, 0, S);
    kt_regs.load(Ktb, M, 0, S);
    for (int t = 0; t < nkt; ++t) {
        const int key0 = t * kBk;
        uint16_t* sK = smem + (t & 1) * kBufElems;  // [kBk][hd]
        uint16_t* sV = sK + kBk * kKp;              // [kBk][hd]
        uint16_t* sKt = sV + kBk * kKp;             // [hd][kBk]
        k_regs.store(sK);
        v_regs.store(sV);
        kt_regs.store(sKt);
        __syncthreads();
        if (t + 1 < nkt) {
            k_regs.load(Kb, ldk, key0 + kBk, S);
            v_regs.load(Vb, ldv, key0 + kBk, S);
            kt_regs.load(Ktb, M, key0 + kBk, S);
        }
        if (key0 > q_first + 31) continue;
        const uint16_t *tK = sK, *tV = sV, *tKt = sKt;
        const bool diagonal = key0 + kBk - 1 > q_first;
        auto block32 = [&](int kb, auto masked) {  // masked: BoolC, two versions of the code
            f32x16 sc = f32x16{0}, dp = f32x16{0};
            pipelined_products<2 * (kHd / 16), kDqAhead>(  // even: a K operand for S^T, odd: a V operand for dP^T
                [&](int i) { return *reinterpret_cast<const uint4*>(((i & 1) ? tV : tK) + (32 * kb + ln) * kKp + 16 * (i / 2) + 8 * g); },
                [&](int i, uint4 f) {
                    if (i & 1) dp = mma(f, dof[i / 2], dp);
                    else sc = mma(f, qf[i / 2], sc);
                });
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float p = __builtin_amdgcn_exp2f(sc[r] * scale_log2e - lse2);
                if constexpr (decltype(masked)::value) {
                    const int key = key0 + 32 * kb + 8 * (r >> 2) + 4 * g + (r & 3);
                    if (key > q_pos) p = 0.0f;
                }
                sc[r] = p * (dp[r] - dl);
            }
            const uint4 df[2] = {slots(sc, 0), slots(sc, 1)};
            pipelined_products<8, kDqAhead>(
                [&](int i) { return token_slots(tKt + (32 * (i % 4) + ln) * kTp, 32 * kb, i / 4, g); },
                [&](int i, uint4 f) { acc[i % 4] = mma(f, df[i / 4], acc[i % 4]); });
        };
        if (diagonal) {
#pragma unroll 1
            for (int kb = 0; kb < 2; ++kb) block32(kb, BoolC<true>{});   // one 32-key block at a time (not unrolled: registers)
        } else {
#pragma unroll 1
            for (int kb = 0; kb < 2; ++kb) block32(kb, BoolC<false>{});
        }
    }
    if (q_ok) {
        uint16_t* row = dQ + tok * lddq + (int64_t)h * kHd + 4 * g;
#pragma unroll
        for (int d = 0; d < kHd / 32; ++d)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                *reinterpret_cast<uint2*>(row + 32 * d + 8 * j) =
                    make_uint2(pack2(acc[d][4 * j] * scale, acc[d][4 * j + 1] * scale),
                               pack2(acc[d][4 * j + 2] * scale, acc[d][4 * j + 3] * scale));
    }
}

// dK^T = Q^T dS and dV^T = dO^T P, as two instantiations of one kernel (DK: the dK half).  One
// block: NW waves, 32 keys each (one key per lane), of one (sequence, query head); loop over
// QS-query steps.  Eight waves (256 keys) per block: every block streams the Q / dO tiles of all
// later queries of its head, and a larger key tile halves that traffic and the prefetch
// registers per thread.  Both halves recompute S = Q K^T; taken together they
// would need the key and value operands, two sets of accumulators and four tiles per step, more
// than the 256 registers a wave has at two waves per SIMD.
template <bool DK, int QS, int NW>
__global__ __launch_bounds__(64 * NW, 512 / (64 * NW)) void sdpa_bwd_dkv_kernel(
    const uint16_t* __restrict__ Q, int64_t ldq, const uint16_t* __restrict__ Qt, const uint16_t* __restrict__ K, int64_t ldk,
    const uint16_t* __restrict__ V, int64_t ldv, const uint16_t* __restrict__ dO, int64_t lddo, const uint16_t* __restrict__ dOt,
    const float* __restrict__ lse, const float* __restrict__ delta, int64_t M, int S, int Hq, int group, float scale_log2e,
    float scale, uint16_t* __restrict__ dst, int64_t ldd, float* __restrict__ part)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
    constexpr int NT = 64 * NW, KB = 32 * NW;  // threads and keys per block
    constexpr int TP = ColTile<QS, NT>::P;     // row pitch of the [hd][queries] tile
    // every tile twice: the next step's tiles are stored while slower waves still read this step's
    constexpr int kTileElems = QS * kKp + kHd * TP + (DK ? QS * kKp : 0);  // bf16 elements of one buffer
    constexpr int kBufElems = kTileElems + 4 * QS;                          // + lse and delta (2 QS floats)
    static_assert((kBufElems * 2) % 16 == 0, "buffers stay 16-byte aligned");

    // early key tiles see the most queries: they are the slowest-varying index, so they start first
    const int bh = blockIdx.x % (Hq * (int)(M / S)), kt = blockIdx.x / (Hq * (int)(M / S));
    const int hq = bh % Hq, b = bh / Hq, kvh = hq / group, gi = hq % group;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, ln = lane & 31, g = lane >> 5;
    const int key_first = kt * KB + wave * 32, key_pos = key_first + ln;
    const int64_t tok0 = (int64_t)b * S;
    const bool k_ok = key_pos < S;
    const int64_t tok = tok0 + (k_ok ? key_pos : 0);

    uint4 kf[kHd / 16], vf[DK ? kHd / 16 : 1];
    {
        const uint16_t* krow = K + tok * ldk + (int64_t)kvh * kHd + 8 * g;
        const uint16_t* vrow = V + tok * ldv + (int64_t)kvh * kHd + 8 * g;
#pragma unroll
        for (int s = 0; s < kHd / 16; ++s) {
            kf[s] = k_ok ? *reinterpret_cast<const uint4*>(krow + 16 * s) : make_uint4(0, 0, 0, 0);
            if constexpr (DK) vf[s] = k_ok ? *reinterpret_cast<const uint4*>(vrow + 16 * s) : make_uint4(0, 0, 0, 0);
        }
    }
    f32x16 acc[kHd / 32];
#pragma unroll
    for (int d = 0; d < kHd / 32; ++d) acc[d] = f32x16{0};

    const int q_start = kt * KB;                        // a multiple of the query step
    const int steps = (S - q_start + QS - 1) / QS;    // >= 1: the block exists only if q_start < S
    const uint16_t* Qb = Q + tok0 * ldq + (int64_t)hq * kHd;
    const uint16_t* Db = dO + tok0 * lddo + (int64_t)hq * kHd;
    const uint16_t* Tb = (DK ? Qt : dOt) + (int64_t)hq * kHd * M + tok0;
    const float* lse_b = lse + (int64_t)hq * M + tok0;
    const float* del_b = delta + (int64_t)hq * M + tok0;

    RowTile<QS, NT> q_regs, d_regs;
    ColTile<QS, NT> t_regs;
    float stat_reg = 0.0f;  // threads 0..63: lse of query threadIdx.x of the step; 64..127: delta (DK)
    auto load_step = [&](int q0) {
        q_regs.load(Qb, ldq, q0, S);
        t_regs.load(Tb, M, q0, S);
        if constexpr (DK) d_regs.load(Db, lddo, q0, S);
        if (threadIdx.x < (DK ? 2 : 1) * QS) {
            const int i = threadIdx.x & (QS - 1);
            const float* src = threadIdx.x < QS ? lse_b : del_b;
            stat_reg = (q0 + i < S) ? src[q0 + i] : 0.0f;
            if (threadIdx.x < QS) stat_reg *= 1.4426950408889634074f;
        }
    };
    // Queries from the end of the sequence down to the diagonal: the blocks of one head (which share
    // an XCD: the head index is the fastest-varying part of blockIdx) then walk the same Q / dO tiles
    // at the same time.
    load_step(q_start + (steps - 1) * QS);
    for (int it = 0; it < steps; ++it) {
        const int q0 = q_start + (steps - 1 - it) * QS;
        uint16_t* sQ = smem + (it & 1) * kBufElems;            // [QS queries][hd]: Q rows
        uint16_t* sT = sQ + QS * kKp;                          // [hd][QS]: DK: Q^T, else dO^T
        uint16_t* sD = sT + kHd * TP;                          // [QS][hd], DK only: dO rows
        float* sLse = reinterpret_cast<float*>(sQ + kTileElems);  // [QS], already times log2(e)
        float* sDel = sLse + QS;                               // [QS], DK only
        q_regs.store(sQ);
        t_regs.store(sT);
        if constexpr (DK) d_regs.store(sD);
        if (threadIdx.x < QS) sLse[threadIdx.x] = stat_reg;
        else if (DK && threadIdx.x < 2 * QS) sDel[threadIdx.x - QS] = stat_reg;
        __syncthreads();
        if (it + 1 < steps) load_step(q0 - QS);
        if (q0 + QS - 1 < key_first) continue;  // every query of the step lies before every key of the wave
        // one 32-query block at a time; registers: queries 32 qb + 8 j + 4 g + i of the step; lane: one key
        // only the steps at the diagonal or at the end of the sequence have anything to mask (wave-uniform)
        const bool edge = q0 < key_first + 32 || q0 + QS > S;
        auto block32 = [&](int qb, auto masked) {  // masked: integral_constant<bool>, two versions of the code
            f32x16 sc = f32x16{0}, dp = f32x16{0};
            if constexpr (DK) {
                pipelined_products<2 * (kHd / 16), kDkvAhead>(  // even: a Q operand for S, odd: a dO operand for dP
                    [&](int i) { return *reinterpret_cast<const uint4*>(((i & 1) ? sD : sQ) + (32 * qb + ln) * kKp + 16 * (i / 2) + 8 * g); },
                    [&](int i, uint4 f) {
                        if (i & 1) dp = mma(f, vf[i / 2], dp);
                        else sc = mma(f, kf[i / 2], sc);
                    });
            } else {
                pipelined_products<kHd / 16, kDkvAhead>(
                    [&](int i) { return *reinterpret_cast<const uint4*>(sQ + (32 * qb + ln) * kKp + 16 * i + 8 * g); },
                    [&](int i, uint4 f) { sc = mma(f, kf[i], sc); });
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int ql = 32 * qb + 8 * j + 4 * g;
                const float4 l4 = *reinterpret_cast<const float4*>(sLse + ql);
                const float lv[4] = {l4.x, l4.y, l4.z, l4.w};
                float dv[4] = {0.0f, 0.0f, 0.0f, 0.0f};
                if constexpr (DK) {
                    const float4 d4 = *reinterpret_cast<const float4*>(sDel + ql);
                    dv[0] = d4.x, dv[1] = d4.y, dv[2] = d4.z, dv[3] = d4.w;
                }
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int r = 4 * j + i, qp = q0 + ql + i;
                    float p = __builtin_amdgcn_exp2f(sc[r] * scale_log2e - lv[i]);
                    if constexpr (decltype(masked)::value) {
                        if (key_pos > qp || qp >= S) p = 0.0f;
                    }
                    sc[r] = DK ? p * (dp[r] - dv[i]) : p;
                }
            }
            const uint4 pf[2] = {slots(sc, 0), slots(sc, 1)};
            pipelined_products<8, kDkvAhead>(
                [&](int i) { return token_slots(sT + (32 * (i % 4) + ln) * TP, 32 * qb, i / 4, g); },
                [&](int i, uint4 f) { acc[i % 4] = mma(f, pf[i / 4], acc[i % 4]); });
        };
        auto step = [&](auto masked) {
            if constexpr (DK) {
#pragma unroll 1
                for (int qb = 0; qb < QS / 32; ++qb) block32(qb, masked);  // not unrolled: two blocks in flight would not fit the registers
            } else {
#pragma unroll
                for (int qb = 0; qb < QS / 32; ++qb) block32(qb, masked);  // unrolled: one block's exponentials overlap the other's products
            }
        };
        if (edge) step(BoolC<true>{});
        else step(BoolC<false>{});
    }
    if (!k_ok) return;
    const float mul = DK ? scale : 1.0f;
    if (group == 1) {
        uint16_t* row = dst + tok * ldd + (int64_t)kvh * kHd + 4 * g;
#pragma unroll
        for (int d = 0; d < kHd / 32; ++d)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                *reinterpret_cast<uint2*>(row + 32 * d + 8 * j) =
                    make_uint2(pack2(acc[d][4 * j] * mul, acc[d][4 * j + 1] * mul), pack2(acc[d][4 * j + 2] * mul, acc[d][4 * j + 3] * mul));
    } else {
        // this query head's share, fp32: [group][token][Hkv * hd]; summed in a fixed order afterwards
        const int64_t w = (int64_t)(Hq / group) * kHd;
        float* row = part + ((int64_t)gi * M + tok) * w + (int64_t)kvh * kHd + 4 * g;
#pragma unroll
        for (int d = 0; d < kHd / 32; ++d)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                *reinterpret_cast<float4*>(row + 32 * d + 8 * j) =
                    make_float4(acc[d][4 * j] * mul, acc[d][4 * j + 1] * mul, acc[d][4 * j + 2] * mul, acc[d][4 * j + 3] * mul);
    }
}

// out[tok][c] = bf16(sum over the group's query heads, in order, of part[gi][tok][c]); 8 columns per thread
__global__ __launch_bounds__(kAttnThreads) void sdpa_group_sum_kernel(const float* __restrict__ part_k, const float* __restrict__ part_v,
                                                                      int64_t M, int64_t w, int group,
                                                                      uint16_t* __restrict__ dK, int64_t lddk,
                                                                      uint16_t* __restrict__ dV, int64_t lddv,
                                                                      uint32_t* __restrict__ amax_dv_bits /* nullable: max-updated */)
{
    uint32_t mag = 0;
    const int64_t chunks = M * (w / 8);
    for (int64_t c = (int64_t)blockIdx.x * kAttnThreads + threadIdx.x; c < 2 * chunks; c += (int64_t)gridDim.x * kAttnThreads) {
        const bool is_v = c >= chunks;
        const int64_t cc = is_v ? c - chunks : c, tok = cc / (w / 8), col = (cc % (w / 8)) * 8;
        const float* src = (is_v ? part_v : part_k) + tok * w + col;
        float4 a = *reinterpret_cast<const float4*>(src), b2 = *reinterpret_cast<const float4*>(src + 4);
        for (int gi = 1; gi < group; ++gi) {
            const float4 x = *reinterpret_cast<const float4*>(src + (int64_t)gi * M * w);
            const float4 y = *reinterpret_cast<const float4*>(src + (int64_t)gi * M * w + 4);
            a.x += x.x, a.y += x.y, a.z += x.z, a.w += x.w;
            b2.x += y.x, b2.y += y.y, b2.z += y.z, b2.w += y.w;
        }
        uint16_t* dst = is_v ? dV + tok * lddv + col : dK + tok * lddk + col;
        const uint4 o = make_uint4(pack2(a.x, a.y), pack2(a.z, a.w), pack2(b2.x, b2.y), pack2(b2.z, b2.w));
        *reinterpret_cast<uint4*>(dst) = o;
        if (is_v) mag = absmax_acc(mag, o);
    }
    if (amax_dv_bits) {
        const uint32_t m = wave_max_u32(pk_collapse(mag)) << 16;
        if ((threadIdx.x & (kWave - 1)) == 0 && m > __atomic_load_n(amax_dv_bits, __ATOMIC_RELAXED)) atomicMax(amax_dv_bits, m);
    }
}

constexpr int kDqWaves = 8;  // 256 queries per block, one block per compute unit
constexpr size_t kDqLds = 2 * (size_t)(2 * kBk * kKp + kHd * kTp) * sizeof(uint16_t);
constexpr int kDkvWaves = 8;             // 256 keys per block, one block per compute unit
constexpr int kDkQs = 64, kDvQs = 64;    // queries per step of the dK and the dV kernel
constexpr size_t kDkLds = 2 * ((size_t)(2 * kDkQs * kKp + kHd * ColTile<kDkQs>::P) * sizeof(uint16_t) + 2 * kDkQs * sizeof(float));
constexpr size_t kDvLds = 2 * ((size_t)(kDvQs * kKp + kHd * ColTile<kDvQs>::P) * sizeof(uint16_t) + 2 * kDvQs * sizeof(float));
static_assert(kDkLds <= 160 * 1024 && kDvLds <= 160 * 1024 && kDqLds <= 160 * 1024, "the tiles fit the LDS of a compute unit");

static f8_status check_attn(const void* q, int64_t ldq, const void* k, int64_t ldk, int64_t B, int64_t S, int64_t Hq,
                            int64_t Hkv, int64_t hd)
{
    if (!q || !k) return F8_ERR_NULL;
    if (hd != kHd || B < 0 || S < 0 || (S % 8) || Hq < 1 || Hkv < 1 || (Hq % Hkv)) return F8_ERR_SHAPE;
    if (S >= (1 << 24) || Hq >= (1 << 16) || B * S >= ((int64_t)1 << 31)) return F8_ERR_SHAPE;
    if (ldq < Hq * hd || ldk < Hkv * hd || (ldq % 8) || (ldk % 8)) return F8_ERR_SHAPE;
    if (!aligned16(q) || !aligned16(k)) return F8_ERR_ALIGN;
    return F8_OK;
}

}  // namespace f8

using namespace f8;

extern "C" {

f8_status f8_sdpa_fwd(const void* q_bf16, int64_t ldq, const void* k_bf16, int64_t ldk, const void* vt_bf16, int64_t B,
                      int64_t S, int64_t Hq, int64_t Hkv, int64_t hd, void* o_bf16, int64_t ldo, float* lse, float* amax_o,
                      void* stream)
{
    f8_status s = check_attn(q_bf16, ldq, k_bf16, ldk, B, S, Hq, Hkv, hd);
    if (s != F8_OK) return s;
    if (!vt_bf16 || !o_bf16 || !lse) return F8_ERR_NULL;
    if (ldo < Hq * hd || (ldo % 8)) return F8_ERR_SHAPE;
    if (!aligned16(vt_bf16) || !aligned16(o_bf16)) return F8_ERR_ALIGN;
    if (amax_o) zero_amax_kernel<<<1, 1, 0, (hipStream_t)stream>>>(reinterpret_cast<uint32_t*>(amax_o));
    if (B == 0 || S == 0) return last_launch_status();
    constexpr int kFwdWaves = 8;  // 256 queries per block, one block per compute unit
    const int64_t nqt = (S + 32 * kFwdWaves - 1) / (32 * kFwdWaves), nb = nqt * Hq * B;
    if (nb > (int64_t)0x7FFFFFFF) return F8_ERR_SHAPE;
    const float scale_log2e = (float)(1.4426950408889634074 / sqrt((double)hd));
    sdpa_fwd_kernel<kFwdWaves><<<(unsigned)nb, 64 * kFwdWaves, 0, (hipStream_t)stream>>>(
        (const uint16_t*)q_bf16, ldq, (const uint16_t*)k_bf16, ldk, (const uint16_t*)vt_bf16, B * S, (int)S, (int)Hq,
        (int)(Hq / Hkv), scale_log2e, (uint16_t*)o_bf16, ldo, lse, (int)nqt, reinterpret_cast<uint32_t*>(amax_o));
    return last_launch_status();
}

size_t f8_sdpa_bwd_workspace_bytes(int64_t B, int64_t S, int64_t Hq, int64_t Hkv, int64_t hd)
{
    if (B <= 0 || S <= 0 || Hq <= 0 || Hkv <= 0 || hd <= 0 || (Hq % Hkv) || Hq == Hkv) return 0;
    return (size_t)2 * (size_t)(B * S) * (size_t)(Hq * hd) * sizeof(float);  // dk and dv shares of every query head
}

f8_status f8_sdpa_bwd(const void* q_bf16, int64_t ldq, const void* qt_bf16, const void* k_bf16, int64_t ldk,
                      const void* kt_bf16, const void* v_bf16, int64_t ldv, const void* o_bf16, int64_t ldo,
                      const void* do_bf16, int64_t lddo, const void* dot_bf16, const float* lse, int64_t B, int64_t S,
                      int64_t Hq, int64_t Hkv, int64_t hd, void* dq_bf16, int64_t lddq, void* dk_bf16, int64_t lddk,
                      void* dv_bf16, int64_t lddv, float* delta, float* amax_dv_inout, void* workspace, size_t workspace_bytes_,
                      void* stream)
{
    f8_status s = check_attn(q_bf16, ldq, k_bf16, ldk, B, S, Hq, Hkv, hd);
    if (s != F8_OK) return s;
    if (!qt_bf16 || !kt_bf16 || !v_bf16 || !o_bf16 || !do_bf16 || !dot_bf16 || !lse || !dq_bf16 || !dk_bf16 || !dv_bf16 || !delta)
        return F8_ERR_NULL;
    const int64_t wq = Hq * hd, wk = Hkv * hd;
    if (ldv < wk || ldo < wq || lddo < wq || lddq < wq || lddk < wk || lddv < wk || (ldv % 8) || (ldo % 8) || (lddo % 8) ||
        (lddq % 8) || (lddk % 8) || (lddv % 8))
        return F8_ERR_SHAPE;
    if (!aligned16(qt_bf16) || !aligned16(kt_bf16) || !aligned16(v_bf16) || !aligned16(o_bf16) || !aligned16(do_bf16) ||
        !aligned16(dot_bf16) || !aligned16(dq_bf16) || !aligned16(dk_bf16) || !aligned16(dv_bf16))
        return F8_ERR_ALIGN;
    const int64_t group = Hq / Hkv;
    if (amax_dv_inout && group == 1) return F8_ERR_ENUM;  // the amax of dv is taken where the heads' shares are summed
    if (group > 1 && (!workspace || workspace_bytes_ < f8_sdpa_bwd_workspace_bytes(B, S, Hq, Hkv, hd))) return F8_ERR_WORKSPACE;
    if (group > 1 && !aligned16(workspace)) return F8_ERR_ALIGN;
    if (B == 0 || S == 0) return F8_OK;
    // More dynamic LDS than the default limit of a launch: raised once per process.  Only success
    // is remembered, so that a failure (a call made while the stream is being captured, a
    // transient error) is tried again by the next call instead of being final.
    static std::atomic<bool> configured{false};
    if (!configured.load(std::memory_order_acquire)) {
        const bool ok =
            hipFuncSetAttribute((const void*)sdpa_bwd_dq_kernel<kDqWaves>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kDqLds) == hipSuccess &&
            hipFuncSetAttribute((const void*)sdpa_bwd_dkv_kernel<true, kDkQs, kDkvWaves>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kDkLds) == hipSuccess &&
            hipFuncSetAttribute((const void*)sdpa_bwd_dkv_kernel<false, kDvQs, kDkvWaves>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kDvLds) == hipSuccess;
        if (!ok) {
            (void)hipGetLastError();
            return F8_ERR_LAUNCH;
        }
        configured.store(true, std::memory_order_release);
    }
    hipStream_t st = (hipStream_t)stream;
    const int64_t M = B * S;
    if ((S + 255) / 256 * Hq * B > (int64_t)0x7FFFFFFF) return F8_ERR_SHAPE;  // one block per 256 tokens and head
    const double sc = 1.0 / sqrt((double)hd);
    const float scale = (float)sc, scale_log2e = (float)(sc * 1.4426950408889634074);
    const int64_t nqt = (S + 32 * kDqWaves - 1) / (32 * kDqWaves);
    sdpa_bwd_dq_kernel<kDqWaves><<<(unsigned)(nqt * Hq * B), 64 * kDqWaves, kDqLds, st>>>(
        (const uint16_t*)q_bf16, ldq, (const uint16_t*)k_bf16, ldk, (const uint16_t*)kt_bf16, (const uint16_t*)v_bf16, ldv,
        (const uint16_t*)o_bf16, ldo, (const uint16_t*)do_bf16, lddo, lse, M, (int)S, (int)Hq, (int)(Hq / Hkv), scale_log2e, scale,
        (uint16_t*)dq_bf16, lddq, delta, (int)nqt);
    float* part_k = group > 1 ? (float*)workspace : nullptr;
    float* part_v = group > 1 ? part_k + group * M * wk : nullptr;
    const int64_t nkt = (S + 32 * kDkvWaves - 1) / (32 * kDkvWaves);
    sdpa_bwd_dkv_kernel<true, kDkQs, kDkvWaves><<<(unsigned)(nkt * Hq * B), 64 * kDkvWaves, kDkLds, st>>>(
        (const uint16_t*)q_bf16, ldq, (const uint16_t*)qt_bf16, (const uint16_t*)k_bf16, ldk, (const uint16_t*)v_bf16, ldv,
        (const uint16_t*)do_bf16, lddo, (const uint16_t*)dot_bf16, lse, delta, M, (int)S, (int)Hq, (int)group, scale_log2e,
        scale, (uint16_t*)dk_bf16, lddk, part_k);
    sdpa_bwd_dkv_kernel<false, kDvQs, kDkvWaves><<<(unsigned)(nkt * Hq * B), 64 * kDkvWaves, kDvLds, st>>>(
        (const uint16_t*)q_bf16, ldq, (const uint16_t*)qt_bf16, (const uint16_t*)k_bf16, ldk, (const uint16_t*)v_bf16, ldv,
        (const uint16_t*)do_bf16, lddo, (const uint16_t*)dot_bf16, lse, delta, M, (int)S, (int)Hq, (int)group, scale_log2e,
        scale, (uint16_t*)dv_bf16, lddv, part_v);
    if (group > 1) {
        int64_t nb = (2 * M * (wk / 8) + kAttnThreads - 1) / kAttnThreads;
        if (nb > 8192) nb = 8192;
        sdpa_group_sum_kernel<<<(unsigned)nb, kAttnThreads, 0, st>>>(part_k, part_v, M, wk, (int)group, (uint16_t*)dk_bf16, lddk,
                                                                   (uint16_t*)dv_bf16, lddv, reinterpret_cast<uint32_t*>(amax_dv_inout));
    }
    return last_launch_status();
}

}  // extern "C"
