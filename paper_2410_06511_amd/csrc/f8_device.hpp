// Device-side helpers shared by the gfx950 kernels: bf16 unpacking, the fp8
// rounding step, wavefront / block max reductions.  wave64 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/f8.h"

namespace f8 {

constexpr int kWave = 64;
constexpr float kEps = 1e-12f;  // floor of amax in the scale formula

template <int FMT>
struct Fmt;
template <>
struct Fmt<F8_E4M3> {
    static constexpr int mant = 3, bias = 7;
    static constexpr float fmax = 448.0f;
};
template <>
struct Fmt<F8_E5M2> {
    static constexpr int mant = 2, bias = 15;
    static constexpr float fmax = 57344.0f;
};

__host__ __device__ inline float fmax_of(int fmt) { return fmt == F8_E4M3 ? 448.0f : 57344.0f; }

// ---- bf16 -------------------------------------------------------------------

// A 32-bit word holds two bf16; widening to fp32 is a shift / mask.
__device__ inline float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ inline float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// fp32 -> bf16 bits, round to nearest even (finite inputs; NaN stays NaN).
__device__ inline uint32_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x40u;
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// ---- fp8 rounding -----------------------------------------------------------

// Round y (already clamped to [-FMAX, FMAX], or NaN) to the fp8 grid, nearest
// with ties to even, using integer arithmetic on the fp32 bits.
//   normal results: add half a target ulp (minus one, plus the kept lsb) to the
//     fp32 magnitude bits and drop the low mantissa bits; a mantissa carry
//     walks into the exponent field by itself.  Re-bias.
//   subnormal results: adding 2^(23 + e_step) makes the fp32 adder do the
//     round-to-nearest-even onto multiples of the subnormal step 2^e_step; the
//     low mantissa bits of the sum are the code.
template <int FMT>
__device__ inline uint32_t encode_sw(float y)
{
    constexpr int MB = Fmt<FMT>::mant, BIAS = Fmt<FMT>::bias;
    constexpr uint32_t kMinNormalBits = (uint32_t)(1 - BIAS + 127) << 23;
    constexpr int SH = 23 - MB;
    const uint32_t u = __float_as_uint(y);
    const uint32_t sign = (u >> 24) & 0x80u;
    const uint32_t a = u & 0x7FFFFFFFu;
    uint32_t code;
    if (a > 0x7F800000u) {
        code = 0x7Fu;
    } else if (a >= kMinNormalBits) {
        const uint32_t r = a + ((1u << (SH - 1)) - 1u) + ((a >> SH) & 1u);
        code = (r >> SH) - ((uint32_t)(127 - BIAS) << MB);
    } else {
        const float magic = __uint_as_float((uint32_t)(127 + 23 + (1 - BIAS - MB)) << 23);
        const float t = __uint_as_float(a) + magic;
        code = __float_as_uint(t) - __float_as_uint(magic);
    }
    return sign | code;
}

// The same rounding by the gfx950 conversion instruction (OCP encodings on this
// chip).  Two values at a time; returns the two codes in the low 16 bits.
template <int FMT>
__device__ inline uint32_t encode_hw2(float y0, float y1)
{
    int r = 0;
    if constexpr (FMT == F8_E4M3)
        r = __builtin_amdgcn_cvt_pk_fp8_f32(y0, y1, r, false);
    else
        r = __builtin_amdgcn_cvt_pk_bf8_f32(y0, y1, r, false);
    return (uint32_t)r & 0xFFFFu;
}

// The casts use the conversion instruction (encode_hw2): the integer rounding (encode_sw) costs
// about a dozen operations per element, which would make the cast ALU-bound instead of HBM-bound.
// The GPU tests compare the two encoders over every fp32 bit pattern (f8_encode_f32).

// scale, saturate, round: two bf16 (one 32-bit word) -> two codes in bits 0..15.
template <int FMT>
__device__ inline uint32_t cast2(uint32_t w, float s0, float s1)
{
    constexpr float FM = Fmt<FMT>::fmax;
    // One rounded fp32 multiply each (no FMA can form: there is no add).  fminf /
    // fmaxf would drop a NaN operand, so clamp with compares that keep it.
    float y0 = bf16_lo(w) * s0;
    float y1 = bf16_hi(w) * s1;
    y0 = y0 > FM ? FM : y0;
    y0 = y0 < -FM ? -FM : y0;
    y1 = y1 > FM ? FM : y1;
    y1 = y1 < -FM ? -FM : y1;
    return encode_hw2<FMT>(y0, y1);
}

// Eight bf16 (a 16-byte chunk) with one scale -> eight codes (two words).
template <int FMT>
__device__ inline uint2 cast8(uint4 v, float s)
{
    uint2 o;
    o.x = cast2<FMT>(v.x, s, s) | (cast2<FMT>(v.y, s, s) << 16);
    o.y = cast2<FMT>(v.z, s, s) | (cast2<FMT>(v.w, s, s) << 16);
    return o;
}

// Eight bf16 with eight scales (per-column scaling).
template <int FMT>
__device__ inline uint2 cast8v(uint4 v, const float* s)
{
    uint2 o;
    o.x = cast2<FMT>(v.x, s[0], s[1]) | (cast2<FMT>(v.y, s[2], s[3]) << 16);
    o.y = cast2<FMT>(v.z, s[4], s[5]) | (cast2<FMT>(v.w, s[6], s[7]) << 16);
    return o;
}

// ---- abs-max on bf16 bit patterns --------------------------------------------

// For finite bf16 the magnitude order is the integer order of the low 15 bits,
// so the running maximum is kept as packed 16-bit integers, two per word.
typedef unsigned short us2 __attribute__((ext_vector_type(2)));

__device__ inline uint32_t pkmax(uint32_t a, uint32_t b)
{
    us2 x = __builtin_bit_cast(us2, a), y = __builtin_bit_cast(us2, b);
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(x, y));
}
__device__ inline uint32_t absmax_acc(uint32_t acc, uint4 v)
{
    acc = pkmax(acc, v.x & 0x7FFF7FFFu);
    acc = pkmax(acc, v.y & 0x7FFF7FFFu);
    acc = pkmax(acc, v.z & 0x7FFF7FFFu);
    acc = pkmax(acc, v.w & 0x7FFF7FFFu);
    return acc;
}
// packed pair -> the larger 15-bit magnitude
__device__ inline uint32_t pk_collapse(uint32_t acc)
{
    uint32_t lo = acc & 0xFFFFu, hi = acc >> 16;
    return lo > hi ? lo : hi;
}
__device__ inline float mag_to_float(uint32_t mag15) { return __uint_as_float(mag15 << 16); }

__device__ inline uint32_t wave_max_u32(uint32_t v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        uint32_t o = (uint32_t)__shfl_xor((int)v, off, kWave);
        v = o > v ? o : v;
    }
    return v;
}

// Max over a block of NW wavefronts; every thread gets the result.  `red` is
// NW words of LDS.  Ends with a barrier, so `red` may be reused afterwards.
template <int NW>
__device__ inline uint32_t block_max_u32(uint32_t v, uint32_t* red)
{
    v = wave_max_u32(v);
    const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
    if (lane == 0) red[w] = v;
    __syncthreads();
    uint32_t r = red[0];
#pragma unroll
    for (int i = 1; i < NW; ++i) r = red[i] > r ? red[i] : r;
    __syncthreads();
    return r;
}

// scale = FMAX / max(amax, eps); IEEE fp32 division (hipcc's default for '/').
__device__ inline float scale_from_amax(float amax, float fm)
{
    return fm / (amax > kEps ? amax : kEps);
}

// ---- feed-forward glue arithmetic (shared by the glue kernels and the cast that fuses it) ----

__device__ inline float sigmoidf_fast(float t) { return 1.0f / (1.0f + __expf(-t)); }

__device__ inline uint32_t pack_bf16(float lo, float hi) { return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16); }

// one 32-bit word = two bf16: h = bf16(silu(a) * b), silu(t) = t / (1 + e^-t)
__device__ inline uint32_t silu_mul2(uint32_t a, uint32_t b)
{
    const float a0 = bf16_lo(a), a1 = bf16_hi(a);
    return pack_bf16((a0 * sigmoidf_fast(a0)) * bf16_lo(b), (a1 * sigmoidf_fast(a1)) * bf16_hi(b));
}

// backward of h = silu(a) * b for one word (two bf16): da = g * b * silu'(a), db = g * silu(a)
__device__ inline void silu_mul_bwd2(uint32_t a, uint32_t b, uint32_t g, uint32_t* da, uint32_t* db)
{
    const float a0 = bf16_lo(a), a1 = bf16_hi(a), g0 = bf16_lo(g), g1 = bf16_hi(g);
    const float s0 = sigmoidf_fast(a0), s1 = sigmoidf_fast(a1);
    *da = pack_bf16((g0 * bf16_lo(b)) * (s0 * (1.0f + a0 * (1.0f - s0))), (g1 * bf16_hi(b)) * (s1 * (1.0f + a1 * (1.0f - s1))));
    *db = pack_bf16(g0 * (a0 * s0), g1 * (a1 * s1));
}

}  // namespace f8
