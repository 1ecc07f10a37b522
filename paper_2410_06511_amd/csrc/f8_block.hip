// The bf16 operations that join the Float8 linears of one transformer block (Section 2.2.4
// applies Float8 to the linear layers only; everything between them stays in bf16): rotary
// position embedding (also writing the transposed copy that the attention backward contracts
// over tokens), a plain bf16 transposition, the residual addition and the backward of RMSNorm.
// All HBM-bound: 16-byte accesses, fp32 arithmetic, one rounding to bf16.
#include "f8_device.hpp"
#include "f8_host.hpp"

#include <math.h>

namespace f8 {

constexpr int kBlkThreads = 256;
constexpr int kBlkWaves = kBlkThreads / kWave;
constexpr int kRt = 64;            // tile edge of the rotating / transposing kernel
constexpr int kRtStride = kRt + 2; // LDS row pitch in bf16: odd number of words

struct RopeFreq {
    double f[128];  // theta^(-2 i / hd), i < hd / 2 <= 128
};

__device__ inline uint32_t add_word(uint32_t a, uint32_t b)
{
    return pack_bf16(bf16_lo(a) + bf16_lo(b), bf16_hi(a) + bf16_hi(b));
}

// rotate the pair (lo, hi) of one word by (c, s)
__device__ inline uint32_t rotate_word(uint32_t w, float c, float s)
{
    const float x0 = bf16_lo(w), x1 = bf16_hi(w);
    return pack_bf16(x0 * c - x1 * s, x0 * s + x1 * c);
}

// x [rows, nh * hd] (row pitch ldx) -> out (row pitch ldo; ROTATE: pairs of adjacent columns turned
// by pos * freq) and out_t [nh * hd, rows] (packed).  One block: a 64x64 tile at the same place of
// `hpb` consecutive heads, one head after the other: the sines and cosines depend on the row and
// on the column inside the head only, so they are taken once and used for every head.  rows, hd
// and the pitches are multiples of 8.  (The plain transposition is the case of one head of width
// cols.)
template <bool ROTATE, bool OUT, bool OUT_T>
__global__ __launch_bounds__(kBlkThreads) void rope_tile_kernel(const uint16_t* __restrict__ x, int64_t rows, int nh, int hd,
                                                                int hpb, int64_t ldx, int64_t ldo, int64_t S, float sign, RopeFreq fr,
                                                                uint16_t* __restrict__ out, uint16_t* __restrict__ out_t,
                                                                int tiles_c /* per row of tiles: tiles per head x head groups */,
                                                                uint32_t* __restrict__ amax_bits /* nullable: max-updated */)
{
    __shared__ uint16_t tile[kRt * kRtStride];
    uint32_t mag = 0;  // packed pair of the largest 15-bit magnitudes written
    const int tph = (hd + kRt - 1) / kRt;  // tiles per head
    const int tc = blockIdx.x % tiles_c;
    const int64_t r0 = (int64_t)(blockIdx.x / tiles_c) * kRt;
    const int c0 = (tc % tph) * kRt, h0 = (tc / tph) * hpb;  // column inside the head, first head
    const int cc = threadIdx.x & 7, rr = threadIdx.x >> 3;
    const int cih = c0 + cc * 8;            // this thread's column inside the head
    const bool col_ok = cih < hd;
    float cs[2][4], sn[2][4];
    if constexpr (ROTATE) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int64_t r = r0 + rr + 32 * i;
            const double pos = (double)(r % S);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                // the angle reaches thousands of radians: product and reduction to
                // [-pi, pi] in fp64, sine and cosine of the remainder in fp32
                const double a = pos * fr.f[col_ok ? (cih >> 1) + j : 0];
                const double red = a - 6.283185307179586476925286766559 * rint(a * 0.15915494309189533576888376337251);
                sincosf((float)red, &sn[i][j], &cs[i][j]);
                sn[i][j] *= sign;
            }
        }
    }
    const int h_end = h0 + hpb < nh ? h0 + hpb : nh;
    for (int h = h0; h < h_end; ++h) {
        const int64_t col = (int64_t)h * hd + cih;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int rl = rr + 32 * i;
            const int64_t r = r0 + rl;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (col_ok && r < rows) {
                v = *reinterpret_cast<const uint4*>(x + r * ldx + col);
                if constexpr (ROTATE)
                    v = make_uint4(rotate_word(v.x, cs[i][0], sn[i][0]), rotate_word(v.y, cs[i][1], sn[i][1]),
                                   rotate_word(v.z, cs[i][2], sn[i][2]), rotate_word(v.w, cs[i][3], sn[i][3]));
                if constexpr (OUT) *reinterpret_cast<uint4*>(out + r * ldo + col) = v;
                mag = absmax_acc(mag, v);
            }
            if constexpr (OUT_T) {
                uint32_t* t32 = reinterpret_cast<uint32_t*>(tile + rl * kRtStride + cc * 8);  // 4-byte aligned: pitch and cc*8 are even
                t32[0] = v.x, t32[1] = v.y, t32[2] = v.z, t32[3] = v.w;
            }
        }
        if constexpr (OUT_T) {
            __syncthreads();
            const int rb = threadIdx.x & 7, cb = threadIdx.x >> 3;
            const int64_t rbase = r0 + 8 * rb;
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int c = cb + 32 * i;
                uint32_t o[4];
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    o[j] = (uint32_t)tile[(8 * rb + 2 * j) * kRtStride + c] | ((uint32_t)tile[(8 * rb + 2 * j + 1) * kRtStride + c] << 16);
                if (rbase < rows && c0 + c < hd)  // rows is a multiple of 8: the piece is all in or all out
                    *reinterpret_cast<uint4*>(out_t + ((int64_t)h * hd + c0 + c) * rows + rbase) = make_uint4(o[0], o[1], o[2], o[3]);
            }
            __syncthreads();  // the tile is free for the next head
        }
    }
    if (amax_bits) {  // a maximum of non-negative floats is a maximum of their bit patterns: order-independent
        const uint32_t m = wave_max_u32(pk_collapse(mag)) << 16;
        if ((threadIdx.x & (kWave - 1)) == 0 && m > __atomic_load_n(amax_bits, __ATOMIC_RELAXED)) atomicMax(amax_bits, m);
    }
}


__global__ __launch_bounds__(kBlkThreads) void add_kernel(const uint4* __restrict__ a, const uint4* __restrict__ b, int64_t n,
                                                          uint4* __restrict__ out)
{
    for (int64_t c = (int64_t)blockIdx.x * kBlkThreads + threadIdx.x; c < n; c += (int64_t)gridDim.x * kBlkThreads) {
        const uint4 u = a[c], v = b[c];
        out[c] = make_uint4(add_word(u.x, v.x), add_word(u.y, v.y), add_word(u.z, v.z), add_word(u.w, v.w));
    }
}

// ---- RMSNorm backward ---------------------------------------------------------------------
//   y = x * r * g, r = rsqrt(mean(x^2) + eps):
//   dx = r * (g . dy) - x * r^3 * mean(x . g . dy),   dg = sum over rows of dy . x * r

__device__ inline float xgd_word(uint32_t x, uint32_t g, uint32_t d)
{
    return bf16_lo(x) * (bf16_lo(g) * bf16_lo(d)) + bf16_hi(x) * (bf16_hi(g) * bf16_hi(d));
}
__device__ inline uint32_t dx_word(uint32_t x, uint32_t g, uint32_t d, float r, float k)
{
    return pack_bf16(r * (bf16_lo(g) * bf16_lo(d)) - bf16_lo(x) * k, r * (bf16_hi(g) * bf16_hi(d)) - bf16_hi(x) * k);
}

// one wave per row.  NC > 0: at most NC 16-byte chunks per lane, x and dy are kept in registers
// between the two passes; NC = 0: any row length, the rows are read twice (second time from the caches)
template <int NC>
__global__ __launch_bounds__(kBlkThreads) void rmsnorm_dx_kernel(const uint4* __restrict__ x, const uint4* __restrict__ g,
                                                                 const float* __restrict__ rstd, const uint4* __restrict__ dy,
                                                                 int64_t M, int64_t dc, float inv_d, uint4* __restrict__ dx,
                                                                 const uint4* __restrict__ res /* nullable: added to dx */,
                                                                 uint32_t* __restrict__ amax_bits /* nullable: max-updated */)
{
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    uint32_t mag = 0;
    for (int64_t m = (int64_t)blockIdx.x * kBlkWaves + wave; m < M; m += (int64_t)gridDim.x * kBlkWaves) {
        const uint4 *xr = x + m * dc, *dr = dy + m * dc;
        float t = 0.0f;
        uint4 kx[NC > 0 ? NC : 1], kd[NC > 0 ? NC : 1];
        auto term = [&](uint4 v, uint4 w, uint4 d) {
            return (xgd_word(v.x, w.x, d.x) + xgd_word(v.y, w.y, d.y)) + (xgd_word(v.z, w.z, d.z) + xgd_word(v.w, w.w, d.w));
        };
        if constexpr (NC > 0) {
#pragma unroll
            for (int i = 0; i < NC; ++i) {
                const int64_t c = lane + (int64_t)kWave * i;
                kx[i] = c < dc ? xr[c] : make_uint4(0, 0, 0, 0);
                kd[i] = c < dc ? dr[c] : make_uint4(0, 0, 0, 0);
                if (c < dc) t += term(kx[i], g[c], kd[i]);
            }
        } else {
            for (int64_t c = lane; c < dc; c += kWave) t += term(xr[c], g[c], dr[c]);
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) t += __shfl_xor(t, off, kWave);
        const float r = rstd[m];
        const float k = ((r * r) * r) * (t * inv_d);
        auto emit = [&](int64_t c, uint4 v, uint4 d) {
            const uint4 w = g[c];
            uint4 o = make_uint4(dx_word(v.x, w.x, d.x, r, k), dx_word(v.y, w.y, d.y, r, k),
                                 dx_word(v.z, w.z, d.z, r, k), dx_word(v.w, w.w, d.w, r, k));
            if (res) {  // the residual branch's gradient: the same two roundings as f8_add after this call
                const uint4 a = res[m * dc + c];
                o = make_uint4(add_word(a.x, o.x), add_word(a.y, o.y), add_word(a.z, o.z), add_word(a.w, o.w));
            }
            dx[m * dc + c] = o;
            mag = absmax_acc(mag, o);
        };
        if constexpr (NC > 0) {
#pragma unroll
            for (int i = 0; i < NC; ++i) {
                const int64_t c = lane + (int64_t)kWave * i;
                if (c < dc) emit(c, kx[i], kd[i]);
            }
        } else {
            for (int64_t c = lane; c < dc; c += kWave) emit(c, xr[c], dr[c]);
        }
    }
    if (amax_bits) {
        const uint32_t m = wave_max_u32(pk_collapse(mag)) << 16;
        if (lane == 0 && m > __atomic_load_n(amax_bits, __ATOMIC_RELAXED)) atomicMax(amax_bits, m);
    }
}

// partial[strip][col] = sum over the strip's rows of dy * x * rstd.  Block: 64 columns x one strip
// of rows; thread (cc, rr) owns 8 columns and every 32nd row.
__global__ __launch_bounds__(kBlkThreads) void rmsnorm_dg_partial_kernel(const uint16_t* __restrict__ x,
                                                                         const float* __restrict__ rstd,
                                                                         const uint16_t* __restrict__ dy, int64_t M,
                                                                         int64_t D, int64_t strip_rows,
                                                                         float* __restrict__ partial, int tiles_c)
{
    __shared__ float red[32][65];
    const int64_t strip = blockIdx.x / tiles_c, c0 = (int64_t)(blockIdx.x % tiles_c) * 64;
    const int cc = threadIdx.x & 7, rr = threadIdx.x >> 3;
    const int64_t col = c0 + cc * 8;
    const int64_t rbeg = strip * strip_rows, rend = rbeg + strip_rows < M ? rbeg + strip_rows : M;
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (col < D) {
        for (int64_t r = rbeg + rr; r < rend; r += 32) {
            const uint4 v = *reinterpret_cast<const uint4*>(x + r * D + col);
            const uint4 d = *reinterpret_cast<const uint4*>(dy + r * D + col);
            const float rs = rstd[r];
            const uint32_t vw[4] = {v.x, v.y, v.z, v.w}, dw[4] = {d.x, d.y, d.z, d.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                acc[2 * j] += bf16_lo(dw[j]) * (bf16_lo(vw[j]) * rs);
                acc[2 * j + 1] += bf16_hi(dw[j]) * (bf16_hi(vw[j]) * rs);
            }
        }
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) red[rr][cc * 8 + j] = acc[j];
    __syncthreads();
    if (threadIdx.x < 64 && c0 + threadIdx.x < D) {
        float s = 0.0f;
        for (int i = 0; i < 32; ++i) s += red[i][threadIdx.x];  // fixed order: the result is reproducible
        partial[strip * D + c0 + threadIdx.x] = s;
    }
}

// dg[c] = sum over the strips, always in the same order: 64 columns per block, four groups of
// threads take every fourth strip each, their four sums are added in group order.
__global__ __launch_bounds__(kBlkThreads) void rmsnorm_dg_final_kernel(const float* __restrict__ partial, int strips, int64_t D,
                                                                       float* __restrict__ dg)
{
    __shared__ float red[4][64];
    const int cl = threadIdx.x & 63, part = threadIdx.x >> 6;
    const int64_t c = (int64_t)blockIdx.x * 64 + cl;
    float s = 0.0f;
    if (c < D)
        for (int i = part; i < strips; i += 4) s += partial[(int64_t)i * D + c];
    red[part][cl] = s;
    __syncthreads();
    if (part == 0 && c < D) dg[c] = ((red[0][cl] + red[1][cl]) + red[2][cl]) + red[3][cl];
}

static int elementwise_blocks(int64_t chunks)
{
    int64_t b = (chunks + kBlkThreads * 2 - 1) / (kBlkThreads * 2);
    if (b < 1) b = 1;
    if (b > 4096) b = 4096;
    return (int)b;
}

template <bool ROTATE>
static f8_status launch_rope_tiles(const void* x, int64_t rows, int64_t nh, int64_t hd, int64_t ldx, int64_t ldo, int64_t S,
                                   float sign, const RopeFreq& fr, void* out, void* out_t, float* amax, hipStream_t st)
{
    // heads per block: as many as leave about four blocks per compute unit
    const int64_t tiles_r = (rows + kRt - 1) / kRt, tph = (hd + kRt - 1) / kRt;
    int64_t hpb = (tiles_r * tph * nh) / 1024;
    if (hpb < 1) hpb = 1;
    if (hpb > 8) hpb = 8;
    if (hpb > nh) hpb = nh;
    const int64_t tiles_c = tph * ((nh + hpb - 1) / hpb);
    const int64_t nb = tiles_r * tiles_c;
    if (nb == 0) return F8_OK;
    if (nb > (int64_t)0x7FFFFFFF) return F8_ERR_SHAPE;
#define F8_ROPE_LAUNCH(O, T)                                                                                              \
    rope_tile_kernel<ROTATE, O, T><<<(unsigned)nb, kBlkThreads, 0, st>>>((const uint16_t*)x, rows, (int)nh, (int)hd, (int)hpb, ldx, \
                                                                         ldo, S, sign, fr, (uint16_t*)out, (uint16_t*)out_t, (int)tiles_c, \
                                                                         reinterpret_cast<uint32_t*>(amax))
    if (out && out_t) F8_ROPE_LAUNCH(true, true);
    else if (out) F8_ROPE_LAUNCH(true, false);
    else F8_ROPE_LAUNCH(false, true);
#undef F8_ROPE_LAUNCH
    return last_launch_status();
}

}  // namespace f8

using namespace f8;

extern "C" {

f8_status f8_rope(const void* x_bf16, int64_t ldx, int64_t M, int64_t S, int64_t n_heads, int64_t hd, double theta,
                  int inverse, void* out_bf16, int64_t ldo, void* out_t_bf16, float* amax_inout, void* stream)
{
    if (!x_bf16 || (!out_bf16 && !out_t_bf16)) return F8_ERR_NULL;
    if (M < 0 || S < 1 || n_heads < 1 || hd < 2 || hd > 256 || (hd % 8) || (M % 8) || !(theta > 0.0)) return F8_ERR_SHAPE;
    if (n_heads * hd >= (1 << 23) || ldx < n_heads * hd || (ldx % 8) || (out_bf16 && (ldo < n_heads * hd || (ldo % 8))))
        return F8_ERR_SHAPE;
    if (!aligned16(x_bf16) || (out_bf16 && !aligned16(out_bf16)) || (out_t_bf16 && !aligned16(out_t_bf16))) return F8_ERR_ALIGN;
    RopeFreq fr;
    for (int i = 0; i < 128; ++i) fr.f[i] = i < hd / 2 ? pow(theta, -2.0 * (double)i / (double)hd) : 0.0;
    return launch_rope_tiles<true>(x_bf16, M, n_heads, hd, ldx, ldo, S, inverse ? -1.0f : 1.0f, fr, out_bf16, out_t_bf16,
                                   amax_inout, (hipStream_t)stream);
}

f8_status f8_transpose_bf16(const void* x_bf16, int64_t ldx, int64_t rows, int64_t cols, void* out_t_bf16, void* stream)
{
    if (!x_bf16 || !out_t_bf16) return F8_ERR_NULL;
    if (rows < 0 || cols < 0 || (rows % 8) || (cols % 8) || ldx < cols || (ldx % 8)) return F8_ERR_SHAPE;
    if (!aligned16(x_bf16) || !aligned16(out_t_bf16)) return F8_ERR_ALIGN;
    RopeFreq fr = {};
    if (cols >= ((int64_t)1 << 31)) return F8_ERR_SHAPE;
    return launch_rope_tiles<false>(x_bf16, rows, 1, cols, ldx, cols, 1, 1.0f, fr, nullptr, out_t_bf16, nullptr, (hipStream_t)stream);
}

f8_status f8_add(const void* a_bf16, const void* b_bf16, int64_t n, void* out_bf16, void* stream)
{
    if (!a_bf16 || !b_bf16 || !out_bf16) return F8_ERR_NULL;
    if (n < 0 || (n % 8)) return F8_ERR_SHAPE;
    if (!aligned16(a_bf16) || !aligned16(b_bf16) || !aligned16(out_bf16)) return F8_ERR_ALIGN;
    if (n == 0) return F8_OK;
    add_kernel<<<elementwise_blocks(n / 8), kBlkThreads, 0, (hipStream_t)stream>>>((const uint4*)a_bf16, (const uint4*)b_bf16,
                                                                                   n / 8, (uint4*)out_bf16);
    return last_launch_status();
}

static f8_status rmsnorm_bwd(const void* x_bf16, const void* g_bf16, const float* rstd, const void* dy_bf16, const void* add_bf16,
                             int64_t M, int64_t D, void* dx_bf16, float* dg, float* amax_dx, void* workspace,
                             size_t workspace_bytes_, void* stream)
{
    if (!x_bf16 || !g_bf16 || !rstd || !dy_bf16 || (!dx_bf16 && !dg)) return F8_ERR_NULL;
    if (M < 0 || D < 0 || (M % 16) || (D % 16)) return F8_ERR_SHAPE;
    if (!aligned16(x_bf16) || !aligned16(g_bf16) || !aligned16(dy_bf16) || (dx_bf16 && !aligned16(dx_bf16))) return F8_ERR_ALIGN;
    // at most 64 strips of rows, each a multiple of 32 rows
    int64_t strip_rows = ((M + 63) / 64 + 31) / 32 * 32;
    if (strip_rows < 32) strip_rows = 32;
    const int64_t strips = M ? (M + strip_rows - 1) / strip_rows : 0;
    if (dg && (!workspace || workspace_bytes_ < (size_t)(strips * D) * sizeof(float))) return F8_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    if (D == 0) return F8_OK;
    if (dx_bf16 && M) {
        int64_t nb = (M + kBlkWaves - 1) / kBlkWaves;
        if (nb > 8192) nb = 8192;
#define F8_DX_LAUNCH(NC)                                                                                      \
    rmsnorm_dx_kernel<NC><<<(unsigned)nb, kBlkThreads, 0, st>>>((const uint4*)x_bf16, (const uint4*)g_bf16, rstd, \
                                                                (const uint4*)dy_bf16, M, D / 8, 1.0f / (float)D, (uint4*)dx_bf16, \
                                                                (const uint4*)add_bf16, reinterpret_cast<uint32_t*>(amax_dx))
        if (D <= 8 * kWave * 8) F8_DX_LAUNCH(8);  // rows up to 4096 elements stay in registers
        else F8_DX_LAUNCH(0);
#undef F8_DX_LAUNCH
    }
    if (dg) {
        const int64_t tiles_c = (D + 63) / 64;
        if (strips * tiles_c > (int64_t)0x7FFFFFFF) return F8_ERR_SHAPE;
        if (strips)
            rmsnorm_dg_partial_kernel<<<(unsigned)(strips * tiles_c), kBlkThreads, 0, st>>>(
                (const uint16_t*)x_bf16, rstd, (const uint16_t*)dy_bf16, M, D, strip_rows, (float*)workspace, (int)tiles_c);
        rmsnorm_dg_final_kernel<<<(unsigned)((D + 63) / 64), kBlkThreads, 0, st>>>(
            (const float*)workspace, (int)strips, D, dg);
    }
    return last_launch_status();
}

f8_status f8_rmsnorm_bwd(const void* x_bf16, const void* g_bf16, const float* rstd, const void* dy_bf16, int64_t M,
                         int64_t D, void* dx_bf16, float* dg, void* workspace, size_t workspace_bytes_, void* stream)
{
    return rmsnorm_bwd(x_bf16, g_bf16, rstd, dy_bf16, nullptr, M, D, dx_bf16, dg, nullptr, workspace, workspace_bytes_, stream);
}

f8_status f8_rmsnorm_bwd_add(const void* x_bf16, const void* g_bf16, const float* rstd, const void* dy_bf16,
                             const void* add_bf16, int64_t M, int64_t D, void* dx_bf16, float* dg, float* amax_dx_inout,
                             void* workspace, size_t workspace_bytes_, void* stream)
{
    if (!add_bf16 || !dx_bf16) return F8_ERR_NULL;
    if (!aligned16(add_bf16)) return F8_ERR_ALIGN;
    return rmsnorm_bwd(x_bf16, g_bf16, rstd, dy_bf16, add_bf16, M, D, dx_bf16, dg, amax_dx_inout, workspace, workspace_bytes_,
                       stream);
}

}  // extern "C"
