// Measuring kernels: what the chip delivers with nothing else in the way, so that the library's
// kernels can be reported against measured ceilings beside the nominal peaks (a matrix-pipe-only
// loop, a device copy, a device read), and the shader clock of a timed region.  Not on the hot path.
#include "f8_device.hpp"
#include "f8_host.hpp"

namespace f8 {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

typedef float v4f __attribute__((ext_vector_type(4)));

// The GEMM kernel's matrix-pipe work with no LDS and no memory traffic: every wave reads its
// operand fragments once from `operands` (32 bytes per lane each) and then only issues MFMAs, in
// the operand pairing of a 128 x 128 wave tile.
//   SHAPE 0: v_mfma_f32_16x16x128_f8f6f4, eight A and eight B fragments, 64 accumulators of four
//            registers: the instruction and the tile of gemm_tile_kernel; iters x 64 MFMAs.
//   SHAPE 1: v_mfma_f32_32x32x64_f8f6f4, four and four fragments, 16 accumulators of sixteen
//            registers: the other fp8 instruction of the same nominal rate; iters x 32 MFMAs
//            (two passes over the pairs), so that both shapes do the same work per iteration.
// Block 0 records the shader-clock and the 100 MHz counters around its loop.
template <int SHAPE>
__global__ __launch_bounds__(256) void probe_mfma_kernel(const uint8_t* __restrict__ operands, uint32_t operand_mask,
                                                         int iters, uint64_t* __restrict__ ticks,
                                                         float* __restrict__ sink)
{
    constexpr int F = SHAPE == 0 ? 8 : 4;
    v8i a[F], b[F];
    const uint32_t t = blockIdx.x * 256u + threadIdx.x;
#pragma unroll
    for (int i = 0; i < F; ++i) {
        a[i] = *reinterpret_cast<const v8i*>(operands + (((t * 16u + i) * 32u) & operand_mask));
        b[i] = *reinterpret_cast<const v8i*>(operands + (((t * 16u + 8 + i) * 32u) & operand_mask));
    }
    float s = 0.f;
    uint64_t c0, r0, c1, r1;
    if constexpr (SHAPE == 0) {
        v4f acc[8][8];
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[i][j] = v4f{0.f, 0.f, 0.f, 0.f};
        c0 = __builtin_readcyclecounter(), r0 = __builtin_amdgcn_s_memrealtime();
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(b[j], a[i], acc[i][j], 0, 0, 0, 0, 0, 0);
        }
        c1 = __builtin_readcyclecounter(), r1 = __builtin_amdgcn_s_memrealtime();
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int j = 0; j < 8; ++j) s += acc[i][j][(i + j) & 3];
    } else {
        v16f acc[4][4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
        c0 = __builtin_readcyclecounter(), r0 = __builtin_amdgcn_s_memrealtime();
        for (int it = 0; it < 2 * iters; ++it) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(b[j], a[i], acc[i][j], 0, 0, 0, 0, 0, 0);
        }
        c1 = __builtin_readcyclecounter(), r1 = __builtin_amdgcn_s_memrealtime();
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) s += acc[i][j][(i * 4 + j) & 15];
    }
    if (s == 1.2345678e-30f) sink[0] = s;  // keeps the loop alive; practically never true
    if (ticks && blockIdx.x == 0 && threadIdx.x == 0) {
        ticks[0] = c1 - c0;
        ticks[1] = r1 - r0;
    }
}

// grid-stride 16-byte copy / read, four loads in flight per thread
typedef unsigned int u4v __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void probe_copy_kernel(const u4v* __restrict__ src, u4v* __restrict__ dst, int64_t n)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    for (; i + 3 * stride < n; i += 4 * stride) {
        const u4v a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
        dst[i] = a, dst[i + stride] = b, dst[i + 2 * stride] = c, dst[i + 3 * stride] = d;
    }
    for (; i < n; i += stride) dst[i] = src[i];
}

__global__ __launch_bounds__(256) void probe_read_kernel(const u4v* __restrict__ src, int64_t n, uint32_t* __restrict__ sink)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    u4v acc = {0, 0, 0, 0};
    for (; i + 3 * stride < n; i += 4 * stride) {
        const u4v a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
        acc |= a | b | c | d;
    }
    for (; i < n; i += stride) acc |= src[i];
    if ((acc.x | acc.y | acc.z | acc.w) == 0x9E3779B9u) sink[0] = acc.x;  // practically never true
}

// The shader-clock counters of different compute units need not agree (they are not one chip-wide
// counter), so every workgroup files its reading under the compute unit it runs on: the die
// (XCC_ID, hardware register 20, bits 3:0) and the shader-engine / array / CU fields of HW_ID
// (hardware register 4, bits 15:8).  Two samples are then compared unit by unit.  Workgroups that
// land on the same unit write nearly the same values to the same slot; whichever lands last stays.
static_assert(F8_PROBE_CLOCK_SLOTS == 8 * 256, "one slot per die and value of HW_ID[15:8]");

__global__ void probe_clock_kernel(uint64_t* __restrict__ out)
{
    const uint32_t xcc = __builtin_amdgcn_s_getreg(20 | (0 << 6) | ((4 - 1) << 11)) & 7u;
    const uint32_t cu = __builtin_amdgcn_s_getreg(4 | (8 << 6) | ((8 - 1) << 11)) & 255u;
    const uint64_t c = __builtin_readcyclecounter();      // shader clock cycles
    const uint64_t r = __builtin_amdgcn_s_memrealtime();  // constant 100 MHz
    uint64_t* slot = out + 4 * (xcc * 256 + cu);
    slot[1] = c;
    slot[2] = r;
    slot[0] = 1;  // this unit's slot is filled
}

static int probe_cu_count()
{
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
        n = 256;
    return n;
}

}  // namespace f8

using namespace f8;

extern "C" {

f8_status f8_probe_mfma(int shape, const uint8_t* operands, int64_t operand_bytes, int iters, uint64_t* ticks, float* sink,
                        int64_t* flops_out, void* stream)
{
    if (shape != 0 && shape != 1) return F8_ERR_ENUM;
    if (!operands || !sink) return F8_ERR_NULL;
    // a power of two of at least one block's worth of fragments, so that offsets wrap with a mask
    if (operand_bytes < 131072 || (operand_bytes & (operand_bytes - 1)) || operand_bytes > (int64_t)1 << 30 || iters < 0 ||
        iters > (1 << 19))
        return F8_ERR_SHAPE;
    if (!aligned16(operands) || (reinterpret_cast<uintptr_t>(operands) & 31u)) return F8_ERR_ALIGN;
    const int blocks = probe_cu_count();  // one wave per SIMD, as the GEMM kernel runs
    // per wave and iteration: 64 x (2 * 16 * 16 * 128) = 32 x (2 * 32 * 32 * 64) flop
    if (flops_out) *flops_out = (int64_t)blocks * 4 * iters * 64 * (2LL * 16 * 16 * 128);
    const uint32_t mask = (uint32_t)(operand_bytes - 1);
    if (shape == 0) probe_mfma_kernel<0><<<blocks, 256, 0, (hipStream_t)stream>>>(operands, mask, iters, ticks, sink);
    else probe_mfma_kernel<1><<<blocks, 256, 0, (hipStream_t)stream>>>(operands, mask, iters, ticks, sink);
    return last_launch_status();
}

f8_status f8_probe_copy(const void* src, void* dst, int64_t bytes, void* stream)
{
    if (!src || !dst) return F8_ERR_NULL;
    if (bytes < 0 || (bytes % 16)) return F8_ERR_SHAPE;
    if (!aligned16(src) || !aligned16(dst)) return F8_ERR_ALIGN;
    if (bytes == 0) return F8_OK;
    probe_copy_kernel<<<2048, 256, 0, (hipStream_t)stream>>>((const u4v*)src, (u4v*)dst, bytes / 16);
    return last_launch_status();
}

f8_status f8_probe_read(const void* src, int64_t bytes, uint32_t* sink, void* stream)
{
    if (!src || !sink) return F8_ERR_NULL;
    if (bytes < 0 || (bytes % 16)) return F8_ERR_SHAPE;
    if (!aligned16(src)) return F8_ERR_ALIGN;
    if (bytes == 0) return F8_OK;
    probe_read_kernel<<<2048, 256, 0, (hipStream_t)stream>>>((const u4v*)src, bytes / 16, sink);
    return last_launch_status();
}

f8_status f8_probe_clock(uint64_t* out, void* stream)
{
    if (!out) return F8_ERR_NULL;
    probe_clock_kernel<<<4096, 64, 0, (hipStream_t)stream>>>(out);  // enough workgroups to visit most compute units
    return last_launch_status();
}

}  // extern "C"
