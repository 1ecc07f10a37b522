// The bf16 glue between the two Float8 linears of a Llama feed-forward block,
//   Y = W2 ( silu(W1 x) * (W3 x) ),
// with W1 and W3 stacked into one linear whose output row is [a | b]:
//   forward   h = silu(a) * b                       silu(t) = t / (1 + e^-t)
//   backward  da = dh * b * silu'(a),  db = dh * silu(a)
// Both are elementwise and HBM-bound.  Each also leaves the amax of what it wrote, taken while
// the values are in registers, so that the Float8 linear that consumes the result casts it in
// one pass (f8_linear_fwd_chained / f8_linear_bwd_chained) instead of reading it twice.
#include "f8_device.hpp"
#include "f8_host.hpp"

namespace f8 {

constexpr int kGlueThreads = 256;
constexpr int kGlueWaves = kGlueThreads / kWave;
constexpr int kGlueMaxBlocks = 2048;
static_assert((size_t)kGlueMaxBlocks * sizeof(uint32_t) <= kMinWorkspaceBytes, "one partial per block fits the minimum workspace");

// ab [M, 2H] as 16-byte chunks: row m has 2 * hc chunks, a first; h [M, H]: hc chunks per row.
__global__ __launch_bounds__(kGlueThreads) void silu_mul_kernel(const uint4* __restrict__ ab, int64_t M, int64_t hc,
                                                               uint4* __restrict__ h, uint32_t* __restrict__ partial)
{
    __shared__ uint32_t red[kGlueWaves];
    const int64_t n = M * hc, stride = (int64_t)gridDim.x * kGlueThreads;
    uint32_t acc = 0;
    for (int64_t c = (int64_t)blockIdx.x * kGlueThreads + threadIdx.x; c < n; c += stride) {
        const int64_t m = c / hc, j = c - m * hc;
        const uint4 a = ab[m * 2 * hc + j], b = ab[m * 2 * hc + hc + j];
        uint4 o;
        o.x = silu_mul2(a.x, b.x), o.y = silu_mul2(a.y, b.y), o.z = silu_mul2(a.z, b.z), o.w = silu_mul2(a.w, b.w);
        h[c] = o;
        acc = absmax_acc(acc, o);
    }
    if (partial) {
        const uint32_t mx = block_max_u32<kGlueWaves>(pk_collapse(acc), red);
        if (threadIdx.x == 0) partial[blockIdx.x] = mx;
    }
}

__global__ __launch_bounds__(kGlueThreads) void silu_mul_bwd_kernel(const uint4* __restrict__ ab, const uint4* __restrict__ dh,
                                                                   int64_t M, int64_t hc, uint4* __restrict__ dab,
                                                                   uint32_t* __restrict__ partial)
{
    __shared__ uint32_t red[kGlueWaves];
    const int64_t n = M * hc, stride = (int64_t)gridDim.x * kGlueThreads;
    uint32_t acc = 0;
    for (int64_t c = (int64_t)blockIdx.x * kGlueThreads + threadIdx.x; c < n; c += stride) {
        const int64_t m = c / hc, j = c - m * hc;
        const uint4 a = ab[m * 2 * hc + j], b = ab[m * 2 * hc + hc + j], g = dh[c];
        uint4 da, db;
        silu_mul_bwd2(a.x, b.x, g.x, &da.x, &db.x);
        silu_mul_bwd2(a.y, b.y, g.y, &da.y, &db.y);
        silu_mul_bwd2(a.z, b.z, g.z, &da.z, &db.z);
        silu_mul_bwd2(a.w, b.w, g.w, &da.w, &db.w);
        dab[m * 2 * hc + j] = da;
        dab[m * 2 * hc + hc + j] = db;
        acc = absmax_acc(absmax_acc(acc, da), db);
    }
    if (partial) {
        const uint32_t mx = block_max_u32<kGlueWaves>(pk_collapse(acc), red);
        if (threadIdx.x == 0) partial[blockIdx.x] = mx;
    }
}

__global__ __launch_bounds__(kGlueThreads) void glue_amax_final_kernel(const uint32_t* __restrict__ partial, int n,
                                                                      float* __restrict__ amax_out)
{
    __shared__ uint32_t red[kGlueWaves];
    uint32_t m = 0;
    for (int i = threadIdx.x; i < n; i += kGlueThreads) m = partial[i] > m ? partial[i] : m;
    m = block_max_u32<kGlueWaves>(m, red);
    if (threadIdx.x == 0) amax_out[0] = mag_to_float(m);
}

// RMS normalisation, forward: y[m, :] = x[m, :] * rstd[m] * g, rstd[m] = 1 / sqrt(mean x[m, :]^2 + eps).
// One wavefront per row, rows strided over the grid; the row is read twice (the second time
// from the caches it has just been loaded into): once for the sum of squares, once to scale.
__device__ inline float sumsq_word(uint32_t w)
{
    const float a = bf16_lo(w), b = bf16_hi(w);
    return a * a + b * b;
}
__device__ inline uint32_t scale_word(uint32_t x, uint32_t g, float r)
{
    return pack_bf16((bf16_lo(x) * r) * bf16_lo(g), (bf16_hi(x) * r) * bf16_hi(g));
}

// NC > 0: a row has at most NC 16-byte chunks per lane and is kept in registers between the two
// passes; NC = 0: any row length, the second pass reads the row again (from the caches).
template <int NC>
__global__ __launch_bounds__(kGlueThreads) void rmsnorm_kernel(const uint4* __restrict__ x, const uint4* __restrict__ g,
                                                              int64_t M, int64_t dc /* 16-byte chunks per row */,
                                                              float inv_d, float eps, uint4* __restrict__ y,
                                                              float* __restrict__ rstd, uint32_t* __restrict__ partial)
{
    __shared__ uint32_t red[kGlueWaves];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    uint32_t acc = 0;
    for (int64_t m = (int64_t)blockIdx.x * kGlueWaves + wave; m < M; m += (int64_t)gridDim.x * kGlueWaves) {
        const uint4* row = x + m * dc;
        float ss = 0.0f;
        uint4 keep[NC > 0 ? NC : 1];
        if constexpr (NC > 0) {
#pragma unroll
            for (int i = 0; i < NC; ++i) {
                const int64_t c = lane + (int64_t)kWave * i;
                keep[i] = c < dc ? row[c] : make_uint4(0, 0, 0, 0);
                ss += (sumsq_word(keep[i].x) + sumsq_word(keep[i].y)) + (sumsq_word(keep[i].z) + sumsq_word(keep[i].w));
            }
        } else {
            for (int64_t c = lane; c < dc; c += kWave) {
                const uint4 v = row[c];
                ss += (sumsq_word(v.x) + sumsq_word(v.y)) + (sumsq_word(v.z) + sumsq_word(v.w));
            }
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) ss += __shfl_xor(ss, off, kWave);
        const float r = 1.0f / sqrtf(ss * inv_d + eps);
        if (lane == 0 && rstd) rstd[m] = r;
        auto emit = [&](int64_t c, uint4 v) {
            const uint4 w = g[c];
            uint4 o;
            o.x = scale_word(v.x, w.x, r), o.y = scale_word(v.y, w.y, r);
            o.z = scale_word(v.z, w.z, r), o.w = scale_word(v.w, w.w, r);
            y[m * dc + c] = o;
            acc = absmax_acc(acc, o);
        };
        if constexpr (NC > 0) {
#pragma unroll
            for (int i = 0; i < NC; ++i) {
                const int64_t c = lane + (int64_t)kWave * i;
                if (c < dc) emit(c, keep[i]);
            }
        } else {
            for (int64_t c = lane; c < dc; c += kWave) emit(c, row[c]);
        }
    }
    if (partial) {
        const uint32_t mx = block_max_u32<kGlueWaves>(pk_collapse(acc), red);
        if (threadIdx.x == 0) partial[blockIdx.x] = mx;
    }
}

static int glue_blocks(int64_t chunks)
{
    int64_t b = (chunks + kGlueThreads * 2 - 1) / (kGlueThreads * 2);
    if (b < 1) b = 1;
    if (b > kGlueMaxBlocks) b = kGlueMaxBlocks;
    return (int)b;
}

static f8_status check_glue(const void* ab, const void* other, void* out, int64_t M, int64_t H, const float* amax,
                            const void* ws, size_t ws_bytes)
{
    if (!ab || !other || !out) return F8_ERR_NULL;
    if (M < 0 || H < 0 || (M % 16) || (H % 16)) return F8_ERR_SHAPE;
    if (!aligned16(ab) || !aligned16(other) || !aligned16(out)) return F8_ERR_ALIGN;
    if (amax && (!ws || ws_bytes < (size_t)kGlueMaxBlocks * sizeof(uint32_t))) return F8_ERR_WORKSPACE;
    return F8_OK;
}

}  // namespace f8

using namespace f8;

extern "C" {

f8_status f8_silu_mul(const void* ab_bf16, int64_t M, int64_t H, void* h_bf16, float* amax_h, void* workspace,
                      size_t workspace_bytes_, void* stream)
{
    f8_status s = check_glue(ab_bf16, h_bf16, h_bf16, M, H, amax_h, workspace, workspace_bytes_);
    if (s != F8_OK) return s;
    hipStream_t st = (hipStream_t)stream;
    const int64_t hc = H / 8;
    int nb = 0;
    if (M > 0 && H > 0) {
        nb = glue_blocks(M * hc);
        silu_mul_kernel<<<nb, kGlueThreads, 0, st>>>((const uint4*)ab_bf16, M, hc, (uint4*)h_bf16,
                                                     amax_h ? (uint32_t*)workspace : nullptr);
    }
    if (amax_h) glue_amax_final_kernel<<<1, kGlueThreads, 0, st>>>((const uint32_t*)workspace, nb, amax_h);
    return last_launch_status();
}

f8_status f8_silu_mul_bwd(const void* ab_bf16, const void* dh_bf16, int64_t M, int64_t H, void* dab_bf16,
                          float* amax_dab, void* workspace, size_t workspace_bytes_, void* stream)
{
    f8_status s = check_glue(ab_bf16, dh_bf16, dab_bf16, M, H, amax_dab, workspace, workspace_bytes_);
    if (s != F8_OK) return s;
    hipStream_t st = (hipStream_t)stream;
    const int64_t hc = H / 8;
    int nb = 0;
    if (M > 0 && H > 0) {
        nb = glue_blocks(M * hc);
        silu_mul_bwd_kernel<<<nb, kGlueThreads, 0, st>>>((const uint4*)ab_bf16, (const uint4*)dh_bf16, M, hc,
                                                         (uint4*)dab_bf16, amax_dab ? (uint32_t*)workspace : nullptr);
    }
    if (amax_dab) glue_amax_final_kernel<<<1, kGlueThreads, 0, st>>>((const uint32_t*)workspace, nb, amax_dab);
    return last_launch_status();
}

f8_status f8_rmsnorm(const void* x_bf16, const void* g_bf16, int64_t M, int64_t D, float eps, void* y_bf16,
                     float* rstd, float* amax_y, void* workspace, size_t workspace_bytes_, void* stream)
{
    if (!x_bf16 || !g_bf16 || !y_bf16) return F8_ERR_NULL;
    if (M < 0 || D < 0 || (M % 16) || (D % 16) || !(eps >= 0.0f)) return F8_ERR_SHAPE;
    if (!aligned16(x_bf16) || !aligned16(g_bf16) || !aligned16(y_bf16)) return F8_ERR_ALIGN;
    if (amax_y && (!workspace || workspace_bytes_ < (size_t)kGlueMaxBlocks * sizeof(uint32_t))) return F8_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    int nb = 0;
    if (M > 0 && D > 0) {
        int64_t b = (M + kGlueWaves - 1) / kGlueWaves;
        nb = (int)(b > kGlueMaxBlocks ? kGlueMaxBlocks : b);
#define F8_RMSNORM_LAUNCH(NC)                                                                                         \
    rmsnorm_kernel<NC><<<nb, kGlueThreads, 0, st>>>((const uint4*)x_bf16, (const uint4*)g_bf16, M, D / 8, 1.0f / (float)D, eps, \
                                                    (uint4*)y_bf16, rstd, amax_y ? (uint32_t*)workspace : nullptr)
        if (D <= 8 * kWave * 8) F8_RMSNORM_LAUNCH(8);         // rows up to 4096 elements stay in registers
        else if (D <= 8 * kWave * 16) F8_RMSNORM_LAUNCH(16);  // up to 8192
        else F8_RMSNORM_LAUNCH(0);
#undef F8_RMSNORM_LAUNCH
    }
    if (amax_y) glue_amax_final_kernel<<<1, kGlueThreads, 0, st>>>((const uint32_t*)workspace, nb, amax_y);
    return last_launch_status();
}

}  // extern "C"
