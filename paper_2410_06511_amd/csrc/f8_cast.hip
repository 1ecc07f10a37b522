// amax, scale and cast kernels (steps 1-3 of dynamic Float8 scaling) and their
// C entry points.  All of them are HBM-bandwidth bound: 16-byte loads, one pass
// per step, partial maxima combined without atomics.
#include "f8_device.hpp"
#include "f8_host.hpp"

namespace f8 {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
// Blocks of the tensorwise amax kernel (upper bound).  Every block of the following cast reduces
// all partials itself, so fewer is cheaper there: 512 measured best on the 8B step (256 about
// equal, 2048 one percent of the step slower).
constexpr int kMaxPartials = 512;
constexpr int kColChunksMax = 64;   // row chunks of the per-column amax kernel (upper bound)

// ---------------------------------------------------------------------------
// tensorwise amax: each block writes one partial maximum (a 15-bit magnitude)
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void amax_tensor_partial_kernel(
    const uint4* __restrict__ x, int64_t rows, int64_t chunks_per_row, int64_t ld_chunks,
    uint32_t* __restrict__ partial)
{
    __shared__ uint32_t red[kWaves];
    uint32_t acc = 0;
    if (ld_chunks == chunks_per_row) {
        const int64_t n = rows * chunks_per_row;
        const int64_t stride = (int64_t)gridDim.x * kThreads;
        int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
        // four independent 16-byte loads in flight per thread
        for (; i + 3 * stride < n; i += 4 * stride) {
            uint4 a = x[i], b = x[i + stride], c = x[i + 2 * stride], d = x[i + 3 * stride];
            acc = absmax_acc(acc, a);
            acc = absmax_acc(acc, b);
            acc = absmax_acc(acc, c);
            acc = absmax_acc(acc, d);
        }
        for (; i < n; i += stride) acc = absmax_acc(acc, x[i]);
    } else {
        for (int64_t r = blockIdx.x; r < rows; r += gridDim.x)
            for (int64_t c = threadIdx.x; c < chunks_per_row; c += kThreads)
                acc = absmax_acc(acc, x[r * ld_chunks + c]);
    }
    uint32_t m = block_max_u32<kWaves>(pk_collapse(acc), red);
    if (threadIdx.x == 0) partial[blockIdx.x] = m;
}

// Every thread of the calling block gets max(partial[0..n)).
__device__ inline uint32_t reduce_partials(const uint32_t* __restrict__ partial, int n, uint32_t* red)
{
    uint32_t m = 0;
    for (int i = threadIdx.x; i < n; i += kThreads) {
        uint32_t p = partial[i];
        m = p > m ? p : m;
    }
    return block_max_u32<kWaves>(m, red);
}

__global__ __launch_bounds__(kThreads) void amax_tensor_final_kernel(
    const uint32_t* __restrict__ partial, int n, float fm, float* __restrict__ amax_out,
    float* __restrict__ scale_out, float* __restrict__ inv_out)
{
    __shared__ uint32_t red[kWaves];
    uint32_t m = reduce_partials(partial, n, red);
    if (threadIdx.x == 0) {
        float a = mag_to_float(m);
        amax_out[0] = a;
        if (scale_out) {
            float s = scale_from_amax(a, fm);
            scale_out[0] = s;
            if (inv_out) inv_out[0] = 1.0f / s;
        }
    }
}

// ---------------------------------------------------------------------------
// per-row amax: one wavefront per row; optionally writes scale and 1/scale too
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void amax_rows_kernel(
    const uint4* __restrict__ x, int64_t rows, int64_t chunks_per_row, int64_t ld_chunks, float fm,
    float* __restrict__ amax_out, float* __restrict__ scale_out, float* __restrict__ inv_out)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t r = (int64_t)blockIdx.x * kWaves + threadIdx.x / kWave;
    if (r >= rows) return;
    const uint4* row = x + r * ld_chunks;
    uint32_t acc = 0;
    int64_t c = lane;
    for (; c + 3 * kWave < chunks_per_row; c += 4 * kWave) {
        uint4 a = row[c], b = row[c + kWave], d = row[c + 2 * kWave], e = row[c + 3 * kWave];
        acc = absmax_acc(acc, a);
        acc = absmax_acc(acc, b);
        acc = absmax_acc(acc, d);
        acc = absmax_acc(acc, e);
    }
    for (; c < chunks_per_row; c += kWave) acc = absmax_acc(acc, row[c]);
    uint32_t m = wave_max_u32(pk_collapse(acc));
    if (lane == 0) {
        float a = mag_to_float(m);
        amax_out[r] = a;
        if (scale_out) {
            float s = scale_from_amax(a, fm);
            scale_out[r] = s;
            if (inv_out) inv_out[r] = 1.0f / s;
        }
    }
}

// ---------------------------------------------------------------------------
// per-column amax: grid (column strips of 128, row chunks); partial[chunk][col]
// ---------------------------------------------------------------------------
// ROWS: the same pass also leaves, for every row, the maximum over this block's 128 columns in
// row_partial[strip][row] (both amax sets of rowwise scaling from one read of x).
__device__ inline uint32_t row_piece_max(uint4 v)
{
    // largest magnitude of the eight bf16 of a chunk, then of the 16 lanes that share the row
    uint32_t m = pk_collapse(pkmax(pkmax(v.x & 0x7FFF7FFFu, v.y & 0x7FFF7FFFu), pkmax(v.z & 0x7FFF7FFFu, v.w & 0x7FFF7FFFu)));
#pragma unroll
    for (int off = 8; off >= 1; off >>= 1) {
        const uint32_t o = (uint32_t)__shfl_xor((int)m, off, kWave);
        m = o > m ? o : m;
    }
    return m;
}

template <bool ROWS>
__global__ __launch_bounds__(kThreads) void amax_cols_partial_kernel(
    const uint4* __restrict__ x, int64_t rows, int64_t cols, int64_t ld_chunks, int64_t rows_per_chunk,
    uint32_t* __restrict__ partial /* [gridDim.y][cols] */, uint32_t* __restrict__ row_partial /* [gridDim.x][rows] */)
{
    __shared__ uint32_t red[16][64 + 1];  // [row lane][word of the strip: 64 words = 128 columns]
    const int cc = threadIdx.x & 15;      // which 16-byte chunk (8 columns) of the strip
    const int rl = threadIdx.x >> 4;      // row lane 0..15
    const int64_t col0 = (int64_t)blockIdx.x * 128 + cc * 8;
    const int64_t r_begin = (int64_t)blockIdx.y * rows_per_chunk;
    int64_t r_end = r_begin + rows_per_chunk;
    if (r_end > rows) r_end = rows;
    uint32_t a0 = 0, a1 = 0, a2 = 0, a3 = 0;
    if constexpr (!ROWS) {
        if (col0 < cols) {
            const uint4* p = x + (col0 >> 3);
            int64_t r = r_begin + rl;
            for (; r + 16 < r_end; r += 32) {
                uint4 v = p[r * ld_chunks], w = p[(r + 16) * ld_chunks];
                a0 = pkmax(a0, pkmax(v.x & 0x7FFF7FFFu, w.x & 0x7FFF7FFFu));
                a1 = pkmax(a1, pkmax(v.y & 0x7FFF7FFFu, w.y & 0x7FFF7FFFu));
                a2 = pkmax(a2, pkmax(v.z & 0x7FFF7FFFu, w.z & 0x7FFF7FFFu));
                a3 = pkmax(a3, pkmax(v.w & 0x7FFF7FFFu, w.w & 0x7FFF7FFFu));
            }
            for (; r < r_end; r += 16) {
                uint4 v = p[r * ld_chunks];
                a0 = pkmax(a0, v.x & 0x7FFF7FFFu);
                a1 = pkmax(a1, v.y & 0x7FFF7FFFu);
                a2 = pkmax(a2, v.z & 0x7FFF7FFFu);
                a3 = pkmax(a3, v.w & 0x7FFF7FFFu);
            }
        }
    } else {
        // Every lane takes part in the row reduction (the 16 lanes of a row form one shuffle
        // group); lanes past the last column contribute zeros.  rows_per_chunk is a multiple of
        // 16 and so is rows, hence all 16 row lanes of the block run the same number of steps.
        const bool col_ok = col0 < cols;
        const uint4* p = x + (col_ok ? (col0 >> 3) : 0);
        uint32_t* rp = row_partial + (int64_t)blockIdx.x * rows;
        // four rows (16 apart) in flight per thread
        for (int64_t r = r_begin + rl; r < r_end; r += 64) {
            uint4 v[4];
            bool in[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                in[k] = r + 16 * k < r_end;
                v[k] = make_uint4(0, 0, 0, 0);
                if (col_ok && in[k]) v[k] = p[(r + 16 * k) * ld_chunks];
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                a0 = pkmax(a0, v[k].x & 0x7FFF7FFFu);
                a1 = pkmax(a1, v[k].y & 0x7FFF7FFFu);
                a2 = pkmax(a2, v[k].z & 0x7FFF7FFFu);
                a3 = pkmax(a3, v[k].w & 0x7FFF7FFFu);
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const uint32_t mk = row_piece_max(v[k]);  // every lane takes part, also for rows past the end
                if (cc == 0 && in[k]) rp[r + 16 * k] = mk;
            }
        }
    }
    red[rl][cc * 4 + 0] = a0;
    red[rl][cc * 4 + 1] = a1;
    red[rl][cc * 4 + 2] = a2;
    red[rl][cc * 4 + 3] = a3;
    __syncthreads();
    if (threadIdx.x < 64) {
        uint32_t m = red[0][threadIdx.x];
#pragma unroll
        for (int i = 1; i < 16; ++i) m = pkmax(m, red[i][threadIdx.x]);
        const int64_t c = (int64_t)blockIdx.x * 128 + threadIdx.x * 2;
        if (c < cols) {
            uint32_t* out = partial + (int64_t)blockIdx.y * cols + c;
            out[0] = m & 0xFFFFu;
            out[1] = m >> 16;
        }
    }
}

// out[j] = max over i < n_outer of partial[i * n_inner + j], with scale and 1/scale: the second
// stage of the per-column maxima (n_outer row chunks, n_inner = cols) and of the per-row maxima
// (n_outer column strips, n_inner = rows).  A block owns 64 consecutive j (coalesced reads)
// and splits the outer index over its four wavefronts, which meet in LDS.
// With blocks0 > 0 a second vector is finished by the blocks from blocks0 on (the per-row maxima
// beside the per-column maxima of rowwise scaling: one launch for both).
__global__ __launch_bounds__(kThreads) void amax_vector_final_kernel(
    const uint32_t* __restrict__ partial, int n_outer, int64_t n_inner, float fm,
    float* __restrict__ amax_out, float* __restrict__ scale_out, float* __restrict__ inv_out,
    int blocks0 = 0, const uint32_t* __restrict__ partial1 = nullptr, int n_outer1 = 0, int64_t n_inner1 = 0,
    float* __restrict__ amax_out1 = nullptr, float* __restrict__ scale_out1 = nullptr, float* __restrict__ inv_out1 = nullptr)
{
    __shared__ uint32_t red[kWaves][kWave];
    const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
    int64_t block = blockIdx.x;
    if (blocks0 > 0 && block >= blocks0) {
        block -= blocks0;
        partial = partial1, n_outer = n_outer1, n_inner = n_inner1;
        amax_out = amax_out1, scale_out = scale_out1, inv_out = inv_out1;
    }
    const int64_t j = block * kWave + lane;
    uint32_t m = 0;
    if (j < n_inner) {
        int i = w;
        for (; i + 3 * kWaves < n_outer; i += 4 * kWaves) {
            const uint32_t p0 = partial[(int64_t)i * n_inner + j], p1 = partial[(int64_t)(i + kWaves) * n_inner + j];
            const uint32_t p2 = partial[(int64_t)(i + 2 * kWaves) * n_inner + j];
            const uint32_t p3 = partial[(int64_t)(i + 3 * kWaves) * n_inner + j];
            const uint32_t a = p0 > p1 ? p0 : p1, b = p2 > p3 ? p2 : p3;
            m = a > m ? a : m;
            m = b > m ? b : m;
        }
        for (; i < n_outer; i += kWaves) {
            const uint32_t p = partial[(int64_t)i * n_inner + j];
            m = p > m ? p : m;
        }
    }
    red[w][lane] = m;
    __syncthreads();
    if (w != 0 || j >= n_inner) return;
#pragma unroll
    for (int k = 1; k < kWaves; ++k) m = red[k][lane] > m ? red[k][lane] : m;
    const float a = mag_to_float(m);
    amax_out[j] = a;
    if (scale_out) {
        const float s = scale_from_amax(a, fm);
        scale_out[j] = s;
        if (inv_out) inv_out[j] = 1.0f / s;
    }
}

// ---------------------------------------------------------------------------
// scale
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void scale_kernel(const float* __restrict__ amax, int64_t n,
                                                          float fm, float* __restrict__ scale_out,
                                                          float* __restrict__ inv_out)
{
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= n) return;
    float s = scale_from_amax(amax[i], fm);
    scale_out[i] = s;
    if (inv_out) inv_out[i] = 1.0f / s;
}

// ---------------------------------------------------------------------------
// delayed scaling: amax history (one block)
// ---------------------------------------------------------------------------
// The step's amax is max(partial[0..npartial)) if partial is given, else amax_in[0].
//   used_scale (nullable): the scale this step's cast used; it and its reciprocal are
//     copied to saved_scale / saved_inv for the GEMM epilogues of this step.
//   history[0..len): newest first; shifted by one, the step's amax enters at [0].
//   next_scale / next_inv (nullable inv): FMAX / max(max(history), eps) for the next step.
// used_scale and next_scale may be the same address: it is read before it is written.
__global__ __launch_bounds__(kThreads) void history_push_kernel(
    const uint32_t* __restrict__ partial, int npartial, const float* __restrict__ amax_in,
    float* __restrict__ history, int len, float fm, float* __restrict__ amax_out,
    const float* used_scale, float* __restrict__ saved_scale, float* __restrict__ saved_inv,
    float* next_scale, float* __restrict__ next_inv)
{
    __shared__ uint32_t red[kWaves];
    float a;
    if (partial) a = mag_to_float(reduce_partials(partial, npartial, red));
    else a = amax_in[0];
    if (threadIdx.x != 0) return;
    if (amax_out) amax_out[0] = a;
    if (used_scale) {
        const float s = used_scale[0];
        saved_scale[0] = s;
        saved_inv[0] = 1.0f / s;
    }
    float m = a;
    for (int i = len - 1; i >= 1; --i) {
        const float h = history[i - 1];
        history[i] = h;
        m = h > m ? h : m;
    }
    if (len > 0) history[0] = a;
    if (next_scale) {
        const float s = scale_from_amax(m, fm);
        next_scale[0] = s;
        if (next_inv) next_inv[0] = 1.0f / s;
    }
}

// dynamic scaling with the amax already known: amax -> scale, 1/scale
__global__ void known_amax_kernel(const float* __restrict__ amax_in, float fm, float* __restrict__ amax_out,
                                  float* __restrict__ scale_out, float* __restrict__ inv_out)
{
    const float a = amax_in[0];
    const float s = scale_from_amax(a, fm);
    amax_out[0] = a;
    scale_out[0] = s;
    inv_out[0] = 1.0f / s;
}

// copies a given scale and its reciprocal (static scaling: the GEMM epilogue reads 1/scale)
__global__ void publish_scale_kernel(const float* __restrict__ s_in, float* __restrict__ s_out,
                                     float* __restrict__ inv_out)
{
    const float s = s_in[0];
    s_out[0] = s;
    inv_out[0] = 1.0f / s;
}

// ---------------------------------------------------------------------------
// cast, streaming form (no transposed output): tensorwise or per-row scales
// ---------------------------------------------------------------------------
// DYN: the scale is derived here from the partial maxima of the amax kernel
// (tensorwise dynamic scaling); block 0 also publishes amax, scale, 1/scale.
template <int FMT, int GRAN, bool DYN>
__global__ __launch_bounds__(kThreads) void cast_stream_kernel(
    const uint4* __restrict__ x, int64_t rows, int64_t chunks_per_row, int64_t ld_chunks,
    const float* __restrict__ scale, const uint32_t* __restrict__ partial, int npartial,
    float* __restrict__ amax_out, float* __restrict__ scale_out, float* __restrict__ inv_out,
    uint2* __restrict__ out, int64_t ldo_chunks)
{
    __shared__ uint32_t red[kWaves];
    float s = 0.0f;
    if constexpr (DYN) {
        float a = mag_to_float(reduce_partials(partial, npartial, red));
        s = scale_from_amax(a, Fmt<FMT>::fmax);
        if (blockIdx.x == 0 && threadIdx.x == 0) {
            amax_out[0] = a;
            scale_out[0] = s;
            inv_out[0] = 1.0f / s;
        }
    } else if constexpr (GRAN == F8_TENSORWISE) {
        s = scale[0];
    }
    if constexpr (GRAN == F8_TENSORWISE) {
        if (ld_chunks == chunks_per_row && ldo_chunks == chunks_per_row) {
            const int64_t n = rows * chunks_per_row;
            const int64_t stride = (int64_t)gridDim.x * kThreads;
            int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
            for (; i + 3 * stride < n; i += 4 * stride) {
                uint4 a = x[i], b = x[i + stride], c = x[i + 2 * stride], d = x[i + 3 * stride];
                out[i] = cast8<FMT>(a, s);
                out[i + stride] = cast8<FMT>(b, s);
                out[i + 2 * stride] = cast8<FMT>(c, s);
                out[i + 3 * stride] = cast8<FMT>(d, s);
            }
            for (; i < n; i += stride) out[i] = cast8<FMT>(x[i], s);
            return;
        }
    }
    for (int64_t r = blockIdx.x; r < rows; r += gridDim.x) {
        if constexpr (GRAN == F8_ROWWISE) s = scale[r];
        for (int64_t c = threadIdx.x; c < chunks_per_row; c += kThreads)
            out[r * ldo_chunks + c] = cast8<FMT>(x[r * ld_chunks + c], s);
    }
}

// ---------------------------------------------------------------------------
// tensorwise dynamic quantisation of one or two contiguous tensors per launch
// ---------------------------------------------------------------------------
// A linear's forward quantises X and W: with one launch per tensor and step the small tensor's
// two launches cost more in launch and drain than in memory time.  Here the grid of the amax
// launch and of the cast launch is split between the tensors in proportion to their sizes, so
// that both parts end together.  Each tensor has its own range of partial maxima.
struct StreamJob {
    const uint4* x;      // n chunks of eight bf16
    uint2* out;          // n chunks of eight codes
    int64_t n;
    uint32_t* partial;   // amax_blocks partial maxima
    float *amax, *scale, *inv;
    int amax_blocks, cast_blocks;
};
struct StreamJobs {
    StreamJob j[2];  // blocks [0, j[0].blocks) work on j[0], the rest on j[1]
};

// Measured on the 8B block's tensors (16384 tokens): four loads in flight per thread beat two and
// eight; 512 partial maxima in all beat 256 and 1024 (every cast block reduces them again); the
// cast is fastest when a block makes one pass of four chunks per thread (32768 blocks cover 268 M
// elements that way; 8192 blocks were 4 % slower, 4096 9 %).
constexpr int kJobPartials = 512;
constexpr int kJobCastBlocks = 32768;
static_assert((size_t)2 * kJobPartials * sizeof(uint32_t) <= kMinWorkspaceBytes, "two ranges of partials fit the minimum");

__global__ __launch_bounds__(kThreads) void amax_jobs_kernel(const StreamJobs jobs)
{
    __shared__ uint32_t red[kWaves];
    const bool second = (int)blockIdx.x >= jobs.j[0].amax_blocks;
    const StreamJob J = second ? jobs.j[1] : jobs.j[0];
    const int b = (int)blockIdx.x - (second ? jobs.j[0].amax_blocks : 0);
    const uint4* __restrict__ x = J.x;
    const int64_t n = J.n, stride = (int64_t)J.amax_blocks * kThreads;
    int64_t i = (int64_t)b * kThreads + threadIdx.x;
    uint32_t acc = 0;
    // four independent 16-byte loads in flight per thread
    for (; i + 3 * stride < n; i += 4 * stride) {
        const uint4 v0 = x[i], v1 = x[i + stride], v2 = x[i + 2 * stride], v3 = x[i + 3 * stride];
        acc = absmax_acc(absmax_acc(absmax_acc(absmax_acc(acc, v0), v1), v2), v3);
    }
    for (; i < n; i += stride) acc = absmax_acc(acc, x[i]);
    const uint32_t m = block_max_u32<kWaves>(pk_collapse(acc), red);
    if (threadIdx.x == 0) J.partial[b] = m;
}

// Every block derives its tensor's scale from that tensor's partial maxima; the first block of
// each tensor also publishes amax, scale and 1/scale.  A block's first four chunks are requested
// before the partial maxima are reduced, so that the reduction's latency (a load, a wave
// reduction, two barriers) passes while they are on their way.
template <int FMT>
__global__ __launch_bounds__(kThreads) void cast_jobs_kernel(const StreamJobs jobs)
{
    __shared__ uint32_t red[kWaves];
    const bool second = (int)blockIdx.x >= jobs.j[0].cast_blocks;
    const StreamJob J = second ? jobs.j[1] : jobs.j[0];
    const int b = (int)blockIdx.x - (second ? jobs.j[0].cast_blocks : 0);
    const uint4* __restrict__ x = J.x;
    uint2* __restrict__ out = J.out;
    const int64_t n = J.n, stride = (int64_t)J.cast_blocks * kThreads;
    int64_t i = (int64_t)b * kThreads + threadIdx.x;

    constexpr int PER_THREAD = (kJobPartials + kThreads - 1) / kThreads;
    uint32_t p[PER_THREAD];
#pragma unroll
    for (int k = 0; k < PER_THREAD; ++k) {
        const int idx = k * kThreads + (int)threadIdx.x;
        p[k] = idx < J.amax_blocks ? J.partial[idx] : 0u;
    }
    const bool first_full = i + 3 * stride < n;
    uint4 v0 = {}, v1 = {}, v2 = {}, v3 = {};
    if (first_full) v0 = x[i], v1 = x[i + stride], v2 = x[i + 2 * stride], v3 = x[i + 3 * stride];
    uint32_t m = p[0];
#pragma unroll
    for (int k = 1; k < PER_THREAD; ++k) m = p[k] > m ? p[k] : m;
    const float a = mag_to_float(block_max_u32<kWaves>(m, red));
    const float s = scale_from_amax(a, Fmt<FMT>::fmax);
    if (b == 0 && threadIdx.x == 0) {
        J.amax[0] = a;
        J.scale[0] = s;
        J.inv[0] = 1.0f / s;
    }
    if (first_full) {
        out[i] = cast8<FMT>(v0, s);
        out[i + stride] = cast8<FMT>(v1, s);
        out[i + 2 * stride] = cast8<FMT>(v2, s);
        out[i + 3 * stride] = cast8<FMT>(v3, s);
        i += 4 * stride;
    }
    for (; i + 3 * stride < n; i += 4 * stride) {
        const uint4 w0 = x[i], w1 = x[i + stride], w2 = x[i + 2 * stride], w3 = x[i + 3 * stride];
        out[i] = cast8<FMT>(w0, s);
        out[i + stride] = cast8<FMT>(w1, s);
        out[i + 2 * stride] = cast8<FMT>(w2, s);
        out[i + 3 * stride] = cast8<FMT>(w3, s);
    }
    for (; i < n; i += stride) out[i] = cast8<FMT>(x[i], s);
}

// Delayed scaling without a transposed copy: the scale is given, so one streaming pass casts the
// tensor and takes its amax on the way; block b leaves the largest magnitude it read in
// partial_out[b].  Contiguous tensors only (n chunks of eight elements).
template <int FMT>
__global__ __launch_bounds__(kThreads) void cast_measure_stream_kernel(
    const uint4* __restrict__ x, int64_t n, const float* __restrict__ scale, uint2* __restrict__ out,
    uint32_t* __restrict__ partial_out)
{
    __shared__ uint32_t red[kWaves];
    const float s = scale[0];
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    uint32_t acc = 0;
    for (; i + 3 * stride < n; i += 4 * stride) {
        const uint4 v0 = x[i], v1 = x[i + stride], v2 = x[i + 2 * stride], v3 = x[i + 3 * stride];
        out[i] = cast8<FMT>(v0, s);
        out[i + stride] = cast8<FMT>(v1, s);
        out[i + 2 * stride] = cast8<FMT>(v2, s);
        out[i + 3 * stride] = cast8<FMT>(v3, s);
        acc = absmax_acc(absmax_acc(absmax_acc(absmax_acc(acc, v0), v1), v2), v3);
    }
    for (; i < n; i += stride) {
        const uint4 v = x[i];
        out[i] = cast8<FMT>(v, s);
        acc = absmax_acc(acc, v);
    }
    const uint32_t m = block_max_u32<kWaves>(pk_collapse(acc), red);
    if (threadIdx.x == 0) partial_out[blockIdx.x] = m;
}

// ---------------------------------------------------------------------------
// cast, tiled form: 128 x 128 tile per block, writes out and/or out_t.
// The transposed copy goes through LDS so that both global writes are made of
// full 128-byte row segments.
// ---------------------------------------------------------------------------
constexpr int kTile = 128;
// Internal granularity of the tiled cast: `out` with one scale per row (scale[rows]) and, from
// the same read of x, `out_t` with one scale per column (scale_col[cols]): different codes.
constexpr int kGranBoth = 3;
constexpr int kLdsStride = 33;  // words per LDS tile row (32 data + 1 pad)

// 4x4 byte transpose: in r[j] byte i = element (row j, col i); out c[i] byte j.
__device__ inline void transpose4x4(const uint32_t r[4], uint32_t c[4])
{
    // interleave rows 0/1 and 2/3 bytewise, then gather 16-bit pairs
    uint32_t t0 = __builtin_amdgcn_perm(r[1], r[0], 0x05010400u);  // r0b0 r1b0 r0b1 r1b1
    uint32_t t1 = __builtin_amdgcn_perm(r[1], r[0], 0x07030602u);  // r0b2 r1b2 r0b3 r1b3
    uint32_t t2 = __builtin_amdgcn_perm(r[3], r[2], 0x05010400u);
    uint32_t t3 = __builtin_amdgcn_perm(r[3], r[2], 0x07030602u);
    c[0] = (t0 & 0xFFFFu) | (t2 << 16);
    c[1] = (t0 >> 16) | (t2 & 0xFFFF0000u);
    c[2] = (t1 & 0xFFFFu) | (t3 << 16);
    c[3] = (t1 >> 16) | (t3 & 0xFFFF0000u);
}

// MEASURE (delayed scaling): the scale is given, and the block also writes the largest
// magnitude of its own tile to partial_out[blockIdx.x], so that the tensor's amax of this step
// comes out of the same single pass over x.
// GLUE (with MEASURE): the tensor that is cast is formed in registers from the feed-forward glue's
// inputs and never written itself.
//   GLUE = 1: x = [a | b], [rows, 2 * cols] with ld = its row length; cast h = bf16(silu(a) * b).
//   GLUE = 2: x = [a | b] as above, x2 = dh [rows, cols]; cast dab = [bf16(dh * b * silu'(a)) |
//             bf16(dh * silu(a))], [rows, 2 * cols]: a block reads its tile of a, b and dh once and
//             emits the matching tiles of both halves (out, out_t have 2 * cols columns / rows).
template <int FMT, int GRAN, bool DYN, bool OUT, bool OUT_T, bool MEASURE = false, int GLUE = 0>
__global__ __launch_bounds__(kThreads) void cast_tile_kernel(
    const uint16_t* __restrict__ x, int64_t rows, int64_t cols, int64_t ld,
    const float* __restrict__ scale, const uint32_t* __restrict__ partial, int npartial,
    float* __restrict__ amax_out, float* __restrict__ scale_out, float* __restrict__ inv_out,
    uint8_t* __restrict__ out, int64_t ld_out, uint8_t* __restrict__ out_t, int64_t ld_out_t,
    int tiles_c, uint32_t* __restrict__ partial_out = nullptr, const float* __restrict__ scale_col = nullptr,
    const uint16_t* __restrict__ x2 = nullptr)
{
    __shared__ uint32_t red[kWaves];
    __shared__ uint32_t tile[kTile * kLdsStride];

    float s = 0.0f;
    if constexpr (!DYN && GRAN == F8_TENSORWISE) s = scale[0];

    // After an amax pass (which sweeps the tensor front to back) the tiles are taken back to front:
    // what the sweep read last is what the memory-side cache still holds.
    const unsigned tile_id = DYN ? gridDim.x - 1 - blockIdx.x : blockIdx.x;
    const int64_t r0 = (int64_t)(tile_id / tiles_c) * kTile;
    const int64_t c0 = (int64_t)(tile_id % tiles_c) * kTile;

    // phase 1: thread (rr, cc) converts the 16-byte chunk cc of rows rr, rr+16, ...
    const int cc = threadIdx.x & 15, rr = threadIdx.x >> 4;
    const int64_t col = c0 + cc * 8;
    const bool col_ok = col < cols;  // cols is a multiple of 8: the chunk is all in or all out
    float sc[8];
    if constexpr (GRAN == F8_COLWISE || GRAN == kGranBoth) {
        const float* cs = GRAN == kGranBoth ? scale_col : scale;
        if (col_ok) {
            const float4 s0 = *reinterpret_cast<const float4*>(cs + col);
            const float4 s1 = *reinterpret_cast<const float4*>(cs + col + 4);
            sc[0] = s0.x, sc[1] = s0.y, sc[2] = s0.z, sc[3] = s0.w;
            sc[4] = s1.x, sc[5] = s1.y, sc[6] = s1.z, sc[7] = s1.w;
        }
    }
    uint4 v[8];
    uint4 v2[GLUE == 2 ? 8 : 1];  // second half of dab
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int64_t r = r0 + rr + 16 * i;
        v[i] = make_uint4(0, 0, 0, 0);
        if constexpr (GLUE == 2) v2[i] = make_uint4(0, 0, 0, 0);
        // Streaming load: this is the last read of x by the quantisation; lines it would leave in
        // the caches only push out the codes that the GEMM reads next.
        typedef unsigned int u4v __attribute__((ext_vector_type(4)));
        if (col_ok && r < rows) {
            if constexpr (GLUE == 1) {
                const uint4 a = *reinterpret_cast<const uint4*>(x + r * ld + col);   // read again by the backward
                const uint4 b = *reinterpret_cast<const uint4*>(x + r * ld + cols + col);
                v[i] = make_uint4(silu_mul2(a.x, b.x), silu_mul2(a.y, b.y), silu_mul2(a.z, b.z), silu_mul2(a.w, b.w));
            } else if constexpr (GLUE == 2) {
                const uint4 a = *reinterpret_cast<const uint4*>(x + r * ld + col);
                const uint4 b = *reinterpret_cast<const uint4*>(x + r * ld + cols + col);
                const uint4 g = *reinterpret_cast<const uint4*>(x2 + r * cols + col);
                silu_mul_bwd2(a.x, b.x, g.x, &v[i].x, &v2[i].x);
                silu_mul_bwd2(a.y, b.y, g.y, &v[i].y, &v2[i].y);
                silu_mul_bwd2(a.z, b.z, g.z, &v[i].z, &v2[i].z);
                silu_mul_bwd2(a.w, b.w, g.w, &v[i].w, &v2[i].w);
            } else {
                const u4v t = __builtin_nontemporal_load(reinterpret_cast<const u4v*>(x + r * ld + col));
                v[i] = make_uint4(t.x, t.y, t.z, t.w);
            }
        }
    }
    if constexpr (DYN) {
        // After the loads of x have been issued: the reduction of the partial maxima (an L2 read
        // and two barriers) then overlaps their latency instead of preceding it.
        float a = mag_to_float(reduce_partials(partial, npartial, red));
        s = scale_from_amax(a, Fmt<FMT>::fmax);
        if (blockIdx.x == 0 && threadIdx.x == 0) {
            amax_out[0] = a;
            scale_out[0] = s;
            inv_out[0] = 1.0f / s;
        }
    }
    uint32_t macc = 0;
    if constexpr (MEASURE) {
#pragma unroll
        for (int i = 0; i < 8; ++i) macc = absmax_acc(macc, v[i]);  // out-of-range chunks are zero
        if constexpr (GLUE == 2) {
#pragma unroll
            for (int i = 0; i < 8; ++i) macc = absmax_acc(macc, v2[i]);
        }
    }
    // codes of one tile of values vv, written at column offset coff of out (row offset of out_t)
    auto emit = [&](const uint4* vv, int64_t coff) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int rl = rr + 16 * i;
            const int64_t r = r0 + rl;
            uint2 q, qt;
            if constexpr (GRAN == F8_COLWISE) {
                q = qt = cast8v<FMT>(vv[i], sc);
            } else if constexpr (GRAN == kGranBoth) {
                s = r < rows ? scale[r] : 0.0f;
                q = cast8<FMT>(vv[i], s);
                qt = cast8v<FMT>(vv[i], sc);
            } else {
                if constexpr (GRAN == F8_ROWWISE) s = r < rows ? scale[r] : 0.0f;
                q = qt = cast8<FMT>(vv[i], s);
            }
            if constexpr (OUT) {
                if (col_ok && r < rows) *reinterpret_cast<uint2*>(out + r * ld_out + coff + col) = q;
            }
            if constexpr (OUT_T) {
                tile[rl * kLdsStride + cc * 2] = qt.x;
                tile[rl * kLdsStride + cc * 2 + 1] = qt.y;
            }
        }
        if constexpr (OUT_T) {
            __syncthreads();
            // phase 2: thread (rb, cb) owns rows 16*rb.. +15 and columns 4*cb.. +3 of the tile and
            // writes four 16-byte pieces, one per column, into the transposed output.
            const int rb = threadIdx.x & 7, cb = threadIdx.x >> 3;
            uint32_t o[4][4];  // o[col i][row group g] = codes of rows 16rb+4g..+3, column 4cb+i
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                uint32_t rws[4], cls[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) rws[j] = tile[(16 * rb + 4 * g + j) * kLdsStride + cb];
                transpose4x4(rws, cls);
#pragma unroll
                for (int i = 0; i < 4; ++i) o[i][g] = cls[i];
            }
            const int64_t rbase = r0 + 16 * rb;
            if (rbase < rows) {  // rows is a multiple of 16: the piece is all in or all out
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int64_t c = c0 + 4 * cb + i;
                    if (c < cols)
                        *reinterpret_cast<uint4*>(out_t + (coff + c) * ld_out_t + rbase) =
                            make_uint4(o[i][0], o[i][1], o[i][2], o[i][3]);
                }
            }
        }
    };
    emit(v, 0);
    if constexpr (GLUE == 2) {
        if constexpr (OUT_T) __syncthreads();  // the tile in LDS has been read before it is rewritten
        emit(v2, cols);
    }
    if constexpr (MEASURE) {
        // after the stores are on their way: the reduction's barriers then stall nothing
        const uint32_t m = block_max_u32<kWaves>(pk_collapse(macc), red);
        if (threadIdx.x == 0) partial_out[blockIdx.x] = m;
    }
}

// ---------------------------------------------------------------------------
// the rounding step alone, for validation: fp32 -> code (clamp, then round)
// ---------------------------------------------------------------------------
template <int FMT, bool HW>
__global__ __launch_bounds__(kThreads) void encode_kernel(const float* __restrict__ y, int64_t n,
                                                           uint8_t* __restrict__ out)
{
    constexpr float FM = Fmt<FMT>::fmax;
    const int64_t i = ((int64_t)blockIdx.x * kThreads + threadIdx.x) * 2;
    if (i >= n) return;
    float a = y[i], b = (i + 1 < n) ? y[i + 1] : 0.0f;
    a = a > FM ? FM : a;
    a = a < -FM ? -FM : a;
    b = b > FM ? FM : b;
    b = b < -FM ? -FM : b;
    uint32_t c;
    if constexpr (HW)
        c = encode_hw2<FMT>(a, b);
    else
        c = encode_sw<FMT>(a) | (encode_sw<FMT>(b) << 8);
    out[i] = (uint8_t)(c & 0xFF);
    if (i + 1 < n) out[i + 1] = (uint8_t)(c >> 8);
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------

static int tensor_partial_blocks(int64_t rows, int64_t cols)
{
    const int64_t chunks = rows * (cols / 8);
    int64_t b = (chunks + kThreads * 4 - 1) / (kThreads * 4);  // >= 4 chunks per thread
    if (b < 1) b = 1;
    if (b > kMaxPartials) b = kMaxPartials;
    return (int)b;
}

static int col_chunks(int64_t rows, int64_t* rows_per_chunk)
{
    int64_t n = (rows + 255) / 256;
    if (n < 1) n = 1;
    if (n > kColChunksMax) n = kColChunksMax;
    int64_t rpc = (rows + n - 1) / n;
    rpc = (rpc + 15) / 16 * 16;
    if (rpc < 16) rpc = 16;
    *rows_per_chunk = rpc;
    return (int)((rows + rpc - 1) / rpc > 0 ? (rows + rpc - 1) / rpc : 1);
}

// what the amax / cast / glue kernels need for their partial maxima
size_t quantise_workspace_bytes(int64_t max_rows, int64_t max_cols)
{
    int64_t d = max_rows > max_cols ? max_rows : max_cols;
    if (d < 0) d = 0;
    static_assert((size_t)kMaxPartials * sizeof(uint32_t) <= kMinWorkspaceBytes, "tensorwise partials fit the minimum");
    size_t tensor = kMinWorkspaceBytes;
    size_t colw = (size_t)kColChunksMax * (size_t)d * sizeof(uint32_t);
    size_t n = tensor > colw ? tensor : colw;
    // per-column partials and per-row partials side by side (rowwise scaling, both from one pass)
    const size_t strips = (size_t)((max_cols > 0 ? max_cols : 0) + 127) / 128;
    const size_t both = colw + strips * (size_t)(max_rows > 0 ? max_rows : 0) * sizeof(uint32_t);
    n = both > n ? both : n;
    // one partial per 128x128 tile of the measuring cast (delayed scaling)
    const int64_t r = max_rows > 0 ? max_rows : 0, c = max_cols > 0 ? max_cols : 0;
    size_t tiles = (size_t)((r + kTile - 1) / kTile) * (size_t)((c + kTile - 1) / kTile) * sizeof(uint32_t);
    n = tiles > n ? tiles : n;
    return (n + 255) / 256 * 256;
}

// the public size: the above, and room for the fp32 partial results of a matrix product split
// along its contraction (up to 8 ranges of an output no larger than rows x cols, and never more
// than one 256x256 tile per compute unit in all)
size_t workspace_bytes(int64_t max_rows, int64_t max_cols)
{
    const size_t r = max_rows > 0 ? (size_t)max_rows : 0, c = max_cols > 0 ? (size_t)max_cols : 0;
    size_t split = (size_t)8 * r * c * sizeof(float);
    split = split < kSplitKMaxBytes ? split : kSplitKMaxBytes;
    const size_t q = quantise_workspace_bytes(max_rows, max_cols);
    const size_t n = split > q ? split : q;
    return (n + 255) / 256 * 256;
}

static f8_status check_matrix(const void* p, int64_t rows, int64_t cols, int64_t ld)
{
    if (!p) return F8_ERR_NULL;
    if (rows < 0 || cols < 0 || (rows % 16) || (cols % 16) || (ld % 16) || ld < cols) return F8_ERR_SHAPE;
    if (((rows + 127) / 128) * ((cols + 127) / 128) > (int64_t)0x7FFFFFFF) return F8_ERR_SHAPE;  // one block per 128x128 tile
    if (!aligned16(p)) return F8_ERR_ALIGN;
    return F8_OK;
}

static inline int nscales(int64_t rows, int64_t cols, int g) { return g == F8_TENSORWISE ? 1 : (g == F8_ROWWISE ? rows : cols); }

// amax (+ optionally scale and 1/scale) of a checked matrix.
static f8_status launch_amax(const void* x, int64_t rows, int64_t cols, int64_t ld, int g, float fm,
                             float* amax_out, float* scale_out, float* inv_out, void* ws,
                             hipStream_t st)
{
    const uint4* xc = static_cast<const uint4*>(x);
    if (g == F8_TENSORWISE) {
        int nb = 0;
        if (rows > 0 && cols > 0) {
            nb = tensor_partial_blocks(rows, cols);
            amax_tensor_partial_kernel<<<nb, kThreads, 0, st>>>(xc, rows, cols / 8, ld / 8, (uint32_t*)ws);
        }
        amax_tensor_final_kernel<<<1, kThreads, 0, st>>>((const uint32_t*)ws, nb, fm, amax_out, scale_out, inv_out);
    } else if (g == F8_ROWWISE) {
        if (rows > 0)
            amax_rows_kernel<<<(unsigned)((rows + kWaves - 1) / kWaves), kThreads, 0, st>>>(
                xc, rows, cols / 8, ld / 8, fm, amax_out, scale_out, inv_out);
    } else {
        if (cols > 0) {
            int64_t rpc = 16;
            int nch = 0;
            if (rows > 0) {
                nch = col_chunks(rows, &rpc);
                dim3 grid((unsigned)((cols + 127) / 128), (unsigned)nch);
                amax_cols_partial_kernel<false><<<grid, kThreads, 0, st>>>(xc, rows, cols, ld / 8, rpc, (uint32_t*)ws, nullptr);
            }
            amax_vector_final_kernel<<<(unsigned)((cols + kWave - 1) / kWave), kThreads, 0, st>>>(
                (const uint32_t*)ws, nch, cols, fm, amax_out, scale_out, inv_out);
        }
    }
    return last_launch_status();
}

template <int FMT, int GRAN, bool DYN>
static void launch_cast_t(const void* x, int64_t rows, int64_t cols, int64_t ld, const float* scale,
                          const uint32_t* partial, int npartial, float* amax_out, float* scale_out,
                          float* inv_out, uint8_t* out, int64_t ld_out, uint8_t* out_t,
                          int64_t ld_out_t, hipStream_t st)
{
    if (rows == 0 || cols == 0) return;
    if (!out_t && GRAN != F8_COLWISE) {
        int64_t chunks = rows * (cols / 8);
        int64_t nb = (chunks + kThreads * 4 - 1) / (kThreads * 4);
        if (nb > kJobCastBlocks) nb = kJobCastBlocks;
        if (GRAN == F8_ROWWISE && nb > rows) nb = rows;
        cast_stream_kernel<FMT, GRAN, DYN><<<(unsigned)nb, kThreads, 0, st>>>(
            (const uint4*)x, rows, cols / 8, ld / 8, scale, partial, npartial, amax_out, scale_out,
            inv_out, (uint2*)out, ld_out / 8);
        return;
    }
    const int tiles_r = (int)((rows + kTile - 1) / kTile), tiles_c = (int)((cols + kTile - 1) / kTile);
    const unsigned nb = (unsigned)tiles_r * (unsigned)tiles_c;
#define F8_LAUNCH_TILE(O, T)                                                                       \
    cast_tile_kernel<FMT, GRAN, DYN, O, T><<<nb, kThreads, 0, st>>>(                               \
        (const uint16_t*)x, rows, cols, ld, scale, partial, npartial, amax_out, scale_out, inv_out, \
        out, ld_out, out_t, ld_out_t, tiles_c)
    if (out && out_t)
        F8_LAUNCH_TILE(true, true);
    else if (out_t)
        F8_LAUNCH_TILE(false, true);
    else
        F8_LAUNCH_TILE(true, false);
#undef F8_LAUNCH_TILE
}

template <bool DYN>
static f8_status launch_cast(const void* x, int64_t rows, int64_t cols, int64_t ld, const float* scale,
                             int g, int fmt, const uint32_t* partial, int npartial, float* amax_out,
                             float* scale_out, float* inv_out, uint8_t* out, int64_t ld_out,
                             uint8_t* out_t, int64_t ld_out_t, hipStream_t st)
{
#define F8_CAST_CASE(F, G)                                                                        \
    launch_cast_t<F, G, DYN && (G == F8_TENSORWISE)>(x, rows, cols, ld, scale, partial, npartial, \
                                                     amax_out, scale_out, inv_out, out, ld_out,   \
                                                     out_t, ld_out_t, st)
    if (fmt == F8_E4M3) {
        if (g == F8_TENSORWISE) F8_CAST_CASE(F8_E4M3, F8_TENSORWISE);
        else if (g == F8_ROWWISE) F8_CAST_CASE(F8_E4M3, F8_ROWWISE);
        else F8_CAST_CASE(F8_E4M3, F8_COLWISE);
    } else {
        if (g == F8_TENSORWISE) F8_CAST_CASE(F8_E5M2, F8_TENSORWISE);
        else if (g == F8_ROWWISE) F8_CAST_CASE(F8_E5M2, F8_ROWWISE);
        else F8_CAST_CASE(F8_E5M2, F8_COLWISE);
    }
#undef F8_CAST_CASE
    return last_launch_status();
}

static f8_status check_cast_outputs(int64_t rows, int64_t cols, const uint8_t* out, int64_t ld_out,
                                    const uint8_t* out_t, int64_t ld_out_t)
{
    if (!out && !out_t) return F8_ERR_NULL;
    if (out) {
        if ((ld_out % 16) || ld_out < cols) return F8_ERR_SHAPE;
        if (!aligned16(out)) return F8_ERR_ALIGN;
    }
    if (out_t) {
        if ((ld_out_t % 16) || ld_out_t < rows) return F8_ERR_SHAPE;
        if (!aligned16(out_t)) return F8_ERR_ALIGN;
    }
    return F8_OK;
}

// Grid shares of the job launches.  The amax launch has at most kJobPartials blocks in all, the
// cast launch at most kJobCastBlocks; a tensor's share is proportional to its size, and a thread
// has at least four chunks to work on.
static void job_shares(int64_t n0, int64_t n1, int total, int* b0, int* b1)
{
    const int64_t per_block = (int64_t)kThreads * 4;
    const int64_t want0 = (n0 + per_block - 1) / per_block, want1 = (n1 + per_block - 1) / per_block;
    if (want0 + want1 <= total) {
        *b0 = (int)want0, *b1 = (int)want1;
        return;
    }
    int64_t s1 = n1 > 0 ? (int64_t)((double)total * (double)n1 / (double)(n0 + n1)) : 0;
    if (n1 > 0 && s1 < 1) s1 = 1;
    if (s1 > want1) s1 = want1;
    int64_t s0 = total - s1;
    if (s0 > want0) s0 = want0;
    *b0 = (int)s0, *b1 = (int)s1;
}

// Tensorwise dynamic quantisation of one or two checked, contiguous, non-empty tensors (n1 = 0:
// one) without transposed copies: two launches in all.  ws: kMinWorkspaceBytes.
struct StreamTensor {
    const void* x;
    int64_t n;  // elements, a multiple of 8
    float *amax, *scale, *inv;
    uint8_t* out;
};
static f8_status quantise_stream(const StreamTensor& t0, const StreamTensor* t1, int fmt, void* ws, hipStream_t st)
{
    StreamJobs jobs{};
    const StreamTensor* t[2] = {&t0, t1};
    const int64_t n0 = t0.n / 8, n1 = t1 ? t1->n / 8 : 0;
    int ab[2], cb[2];
    job_shares(n0, n1, kJobPartials, &ab[0], &ab[1]);
    job_shares(n0, n1, kJobCastBlocks, &cb[0], &cb[1]);
    for (int k = 0; k < 2; ++k) {
        StreamJob& J = jobs.j[k];
        if (!t[k]) continue;
        J.x = (const uint4*)t[k]->x, J.out = (uint2*)t[k]->out, J.n = t[k]->n / 8;
        J.partial = (uint32_t*)ws + k * kJobPartials;
        J.amax = t[k]->amax, J.scale = t[k]->scale, J.inv = t[k]->inv;
        J.amax_blocks = ab[k], J.cast_blocks = cb[k];
    }
    amax_jobs_kernel<<<(unsigned)(ab[0] + ab[1]), kThreads, 0, st>>>(jobs);
    if (fmt == F8_E4M3) cast_jobs_kernel<F8_E4M3><<<(unsigned)(cb[0] + cb[1]), kThreads, 0, st>>>(jobs);
    else cast_jobs_kernel<F8_E5M2><<<(unsigned)(cb[0] + cb[1]), kThreads, 0, st>>>(jobs);
    return last_launch_status();
}

static inline bool streamable(int64_t rows, int64_t cols, int64_t ld, int64_t ld_out, const uint8_t* out, const uint8_t* out_t)
{
    return rows > 0 && cols > 0 && ld == cols && ld_out == cols && out && !out_t;
}

// X and W of a linear's forward (tensorwise, same format, contiguous): both in two launches when
// neither wants a transposed copy, else one after the other.
f8_status quantise_pair(const void* x0, int64_t rows0, int64_t cols0, float* amax0, float* scale0, float* inv0,
                        uint8_t* out0, uint8_t* out_t0, const void* x1, int64_t rows1, int64_t cols1, float* amax1,
                        float* scale1, float* inv1, uint8_t* out1, uint8_t* out_t1, int fmt, void* ws, hipStream_t st)
{
    if (streamable(rows0, cols0, cols0, cols0, out0, out_t0) && streamable(rows1, cols1, cols1, cols1, out1, out_t1)) {
        const StreamTensor a{x0, rows0 * cols0, amax0, scale0, inv0, out0}, b{x1, rows1 * cols1, amax1, scale1, inv1, out1};
        // the larger tensor's blocks first, the smaller one's fill the tail
        return a.n >= b.n ? quantise_stream(a, &b, fmt, ws, st) : quantise_stream(b, &a, fmt, ws, st);
    }
    f8_status s = quantise(x0, rows0, cols0, cols0, F8_TENSORWISE, fmt, amax0, scale0, inv0, out0, cols0, out_t0, rows0, ws, st);
    if (s != F8_OK) return s;
    return quantise(x1, rows1, cols1, cols1, F8_TENSORWISE, fmt, amax1, scale1, inv1, out1, cols1, out_t1, rows1, ws, st);
}

// Dynamic-scaling quantisation of one checked tensor (used by f8_amax_cast and the linear).
f8_status quantise(const void* x, int64_t rows, int64_t cols, int64_t ld, int g, int fmt,
                   float* amax_out, float* scale_out, float* inv_out, uint8_t* out, int64_t ld_out,
                   uint8_t* out_t, int64_t ld_out_t, void* ws, hipStream_t st)
{
    const float fm = fmax_of(fmt);
    if (g == F8_TENSORWISE && streamable(rows, cols, ld, ld_out, out, out_t))
        return quantise_stream(StreamTensor{x, rows * cols, amax_out, scale_out, inv_out, out}, nullptr, fmt, ws, st);
    if (g == F8_TENSORWISE && rows > 0 && cols > 0) {
        // partial maxima, then the cast derives the scale from them itself: two launches
        const int nb = tensor_partial_blocks(rows, cols);
        amax_tensor_partial_kernel<<<nb, kThreads, 0, st>>>((const uint4*)x, rows, cols / 8, ld / 8, (uint32_t*)ws);
        return launch_cast<true>(x, rows, cols, ld, nullptr, g, fmt, (const uint32_t*)ws, nb, amax_out,
                                 scale_out, inv_out, out, ld_out, out_t, ld_out_t, st);
    }
    f8_status s = launch_amax(x, rows, cols, ld, g, fm, amax_out, scale_out, inv_out, ws, st);
    if (s != F8_OK) return s;
    return launch_cast<false>(x, rows, cols, ld, scale_out, g, fmt, nullptr, 0, nullptr, nullptr, nullptr,
                              out, ld_out, out_t, ld_out_t, st);
}

// Tensorwise cast with a given scale that also leaves one partial maximum per 128x128 tile in
// ws (checked tensor).  *npartial = number of partials written (0 for an empty tensor).
f8_status cast_measure(const void* x, int64_t rows, int64_t cols, int64_t ld, const float* scale, int fmt,
                       uint8_t* out, int64_t ld_out, uint8_t* out_t, int64_t ld_out_t, void* ws,
                       size_t ws_bytes, int* npartial, hipStream_t st, int glue, const void* x2)
{
    *npartial = 0;
    if (rows == 0 || cols == 0) return F8_OK;
    const int64_t kcols = glue == 2 ? cols / 2 : cols;  // the kernel's tile grid covers one half of dab
    const int64_t tiles_r = (rows + kTile - 1) / kTile, tiles_c = (kcols + kTile - 1) / kTile;
    const int64_t nb = tiles_r * tiles_c;
    if (nb > (int64_t)0x7FFFFFFF || (size_t)nb * sizeof(uint32_t) > ws_bytes) return F8_ERR_WORKSPACE;
    if (glue == 0 && streamable(rows, cols, ld, ld_out, out, out_t)) {
        // one partial per block, never more blocks than the tiled form has tiles (the workspace
        // is sized for those) and at least four chunks per thread
        const int64_t chunks = rows * (cols / 8);
        int64_t sb = (chunks + kThreads * 4 - 1) / (kThreads * 4);
        sb = sb < nb ? sb : nb;
        sb = sb < kJobCastBlocks ? sb : kJobCastBlocks;
        if (fmt == F8_E4M3)
            cast_measure_stream_kernel<F8_E4M3><<<(unsigned)sb, kThreads, 0, st>>>((const uint4*)x, chunks, scale, (uint2*)out, (uint32_t*)ws);
        else
            cast_measure_stream_kernel<F8_E5M2><<<(unsigned)sb, kThreads, 0, st>>>((const uint4*)x, chunks, scale, (uint2*)out, (uint32_t*)ws);
        *npartial = (int)sb;
        return last_launch_status();
    }
#define F8_LAUNCH_MEASURE_G(F, O, T, G)                                                                  \
    cast_tile_kernel<F, F8_TENSORWISE, false, O, T, true, G><<<(unsigned)nb, kThreads, 0, st>>>(         \
        (const uint16_t*)x, rows, kcols, ld, scale, nullptr, 0, nullptr, nullptr, nullptr, out, ld_out, out_t, \
        ld_out_t, (int)tiles_c, (uint32_t*)ws, nullptr, (const uint16_t*)x2)
#define F8_LAUNCH_MEASURE(F, O, T)                       \
    do {                                                 \
        if (glue == 1) F8_LAUNCH_MEASURE_G(F, O, T, 1);  \
        else if (glue == 2) F8_LAUNCH_MEASURE_G(F, O, T, 2); \
        else F8_LAUNCH_MEASURE_G(F, O, T, 0);            \
    } while (0)
#define F8_MEASURE_FMT(F)                               \
    do {                                                \
        if (out && out_t) F8_LAUNCH_MEASURE(F, true, true);  \
        else if (out_t) F8_LAUNCH_MEASURE(F, false, true);   \
        else F8_LAUNCH_MEASURE(F, true, false);              \
    } while (0)
    if (fmt == F8_E4M3) F8_MEASURE_FMT(F8_E4M3);
    else F8_MEASURE_FMT(F8_E5M2);
#undef F8_MEASURE_FMT
#undef F8_LAUNCH_MEASURE
#undef F8_LAUNCH_MEASURE_G
    *npartial = (int)nb;
    return last_launch_status();
}

f8_status history_push(const void* partial, int npartial, const float* amax_in, float* history, int64_t len,
                       int fmt, float* amax_out, const float* used_scale, float* saved_scale,
                       float* saved_inv, float* next_scale, float* next_inv, hipStream_t st)
{
    history_push_kernel<<<1, kThreads, 0, st>>>((const uint32_t*)partial, npartial, amax_in, history, (int)len,
                                                fmax_of(fmt), amax_out, used_scale, saved_scale, saved_inv,
                                                next_scale, next_inv);
    return last_launch_status();
}

f8_status publish_scale(const float* s_in, float* s_out, float* inv_out, hipStream_t st)
{
    publish_scale_kernel<<<1, 1, 0, st>>>(s_in, s_out, inv_out);
    return last_launch_status();
}

// Rowwise quantisation of both orientations from ONE read of x: out [rows, cols] with the
// per-row scales, out_t [cols, rows] with the per-column scales (checked arguments).
f8_status cast_rows_and_cols(const void* x, int64_t rows, int64_t cols, int64_t ld, int fmt,
                             const float* scale_rows, const float* scale_cols, uint8_t* out, int64_t ld_out,
                             uint8_t* out_t, int64_t ld_out_t, hipStream_t st)
{
    if (rows == 0 || cols == 0) return F8_OK;
    const int tiles_r = (int)((rows + kTile - 1) / kTile), tiles_c = (int)((cols + kTile - 1) / kTile);
    const unsigned nb = (unsigned)tiles_r * (unsigned)tiles_c;
    if (fmt == F8_E4M3)
        cast_tile_kernel<F8_E4M3, kGranBoth, false, true, true><<<nb, kThreads, 0, st>>>(
            (const uint16_t*)x, rows, cols, ld, scale_rows, nullptr, 0, nullptr, nullptr, nullptr, out, ld_out, out_t,
            ld_out_t, tiles_c, nullptr, scale_cols);
    else
        cast_tile_kernel<F8_E5M2, kGranBoth, false, true, true><<<nb, kThreads, 0, st>>>(
            (const uint16_t*)x, rows, cols, ld, scale_rows, nullptr, 0, nullptr, nullptr, nullptr, out, ld_out, out_t,
            ld_out_t, tiles_c, nullptr, scale_cols);
    return last_launch_status();
}

// Rowwise scaling: per-row and per-column amax, scale and 1/scale of x from ONE read (checked
// arguments, rows and cols > 0).  ws: workspace_bytes(rows, cols).
f8_status amax_rows_and_cols(const void* x, int64_t rows, int64_t cols, int64_t ld, int fmt, float* amax_r,
                             float* scale_r, float* inv_r, float* amax_c, float* scale_c, float* inv_c, void* ws,
                             hipStream_t st)
{
    const float fm = fmax_of(fmt);
    int64_t rpc = 16;
    const int nch = col_chunks(rows, &rpc);
    const unsigned strips = (unsigned)((cols + 127) / 128);
    uint32_t* colp = (uint32_t*)ws;
    uint32_t* rowp = colp + (size_t)kColChunksMax * (size_t)(rows > cols ? rows : cols);
    dim3 grid(strips, (unsigned)nch);
    amax_cols_partial_kernel<true><<<grid, kThreads, 0, st>>>((const uint4*)x, rows, cols, ld / 8, rpc, colp, rowp);
    const unsigned bc = (unsigned)((cols + kWave - 1) / kWave), br = (unsigned)((rows + kWave - 1) / kWave);
    amax_vector_final_kernel<<<bc + br, kThreads, 0, st>>>(colp, nch, cols, fm, amax_c, scale_c, inv_c, (int)bc, rowp,
                                                           (int)strips, rows, amax_r, scale_r, inv_r);
    return last_launch_status();
}

// per-row or per-column amax with scales (no cast), for callers that cast both orientations at once
f8_status amax_scales(const void* x, int64_t rows, int64_t cols, int64_t ld, int g, int fmt, float* amax_out,
                      float* scale_out, float* inv_out, void* ws, hipStream_t st)
{
    return launch_amax(x, rows, cols, ld, g, fmax_of(fmt), amax_out, scale_out, inv_out, ws, st);
}

// amax is known (taken by the producer of x): publish amax / scale / 1/scale, then one cast pass.
f8_status quantise_known_amax(const void* x, int64_t rows, int64_t cols, int64_t ld, int fmt, const float* amax_in,
                              float* amax_out, float* scale_out, float* inv_out, uint8_t* out, int64_t ld_out,
                              uint8_t* out_t, int64_t ld_out_t, hipStream_t st)
{
    known_amax_kernel<<<1, 1, 0, st>>>(amax_in, fmax_of(fmt), amax_out, scale_out, inv_out);
    f8_status s = last_launch_status();
    if (s != F8_OK) return s;
    return launch_cast<false>(x, rows, cols, ld, scale_out, F8_TENSORWISE, fmt, nullptr, 0, nullptr, nullptr, nullptr,
                              out, ld_out, out_t, ld_out_t, st);
}

f8_status cast_given(const void* x, int64_t rows, int64_t cols, int64_t ld, const float* scale, int fmt,
                     uint8_t* out, int64_t ld_out, uint8_t* out_t, int64_t ld_out_t, hipStream_t st)
{
    return launch_cast<false>(x, rows, cols, ld, scale, F8_TENSORWISE, fmt, nullptr, 0, nullptr, nullptr, nullptr,
                              out, ld_out, out_t, ld_out_t, st);
}

}  // namespace f8

using namespace f8;

extern "C" {

size_t f8_workspace_bytes(int64_t max_rows, int64_t max_cols) { return workspace_bytes(max_rows, max_cols); }

f8_status f8_amax(const void* x_bf16, int64_t rows, int64_t cols, int64_t ld, f8_granularity g,
                  float* amax_out, void* workspace, size_t workspace_bytes_, void* stream)
{
    if ((int)g < 0 || (int)g > F8_COLWISE) return F8_ERR_ENUM;
    f8_status s = check_matrix(x_bf16, rows, cols, ld);
    if (s != F8_OK) return s;
    if (!amax_out) return F8_ERR_NULL;
    if (g != F8_ROWWISE && (!workspace || workspace_bytes_ < quantise_workspace_bytes(rows, cols))) return F8_ERR_WORKSPACE;
    return launch_amax(x_bf16, rows, cols, ld, g, 0.0f, amax_out, nullptr, nullptr, workspace, (hipStream_t)stream);
}

f8_status f8_scale(const float* amax, int64_t n, f8_format fmt, float* scale_out, float* inv_scale_out,
                   void* stream)
{
    if ((int)fmt < 0 || (int)fmt > F8_E5M2) return F8_ERR_ENUM;
    if (!amax || !scale_out) return F8_ERR_NULL;
    if (n < 0) return F8_ERR_SHAPE;
    if (n == 0) return F8_OK;
    scale_kernel<<<(unsigned)((n + kThreads - 1) / kThreads), kThreads, 0, (hipStream_t)stream>>>(
        amax, n, fmax_of(fmt), scale_out, inv_scale_out);
    return last_launch_status();
}

f8_status f8_cast(const void* x_bf16, int64_t rows, int64_t cols, int64_t ld, const float* scale,
                  f8_granularity g, f8_format fmt, uint8_t* out, int64_t ld_out, uint8_t* out_t,
                  int64_t ld_out_t, void* stream)
{
    if ((int)g < 0 || (int)g > F8_COLWISE || (int)fmt < 0 || (int)fmt > F8_E5M2) return F8_ERR_ENUM;
    f8_status s = check_matrix(x_bf16, rows, cols, ld);
    if (s != F8_OK) return s;
    if (!scale) return F8_ERR_NULL;
    if (g == F8_COLWISE && !aligned16(scale)) return F8_ERR_ALIGN;
    s = check_cast_outputs(rows, cols, out, ld_out, out_t, ld_out_t);
    if (s != F8_OK) return s;
    return launch_cast<false>(x_bf16, rows, cols, ld, scale, g, fmt, nullptr, 0, nullptr, nullptr, nullptr,
                              out, ld_out, out_t, ld_out_t, (hipStream_t)stream);
}

f8_status f8_amax_cast(const void* x_bf16, int64_t rows, int64_t cols, int64_t ld, f8_granularity g,
                       f8_format fmt, float* amax_out, float* scale_out, float* inv_scale_out,
                       uint8_t* out, int64_t ld_out, uint8_t* out_t, int64_t ld_out_t, void* workspace,
                       size_t workspace_bytes_, void* stream)
{
    if ((int)g < 0 || (int)g > F8_COLWISE || (int)fmt < 0 || (int)fmt > F8_E5M2) return F8_ERR_ENUM;
    f8_status s = check_matrix(x_bf16, rows, cols, ld);
    if (s != F8_OK) return s;
    if (!amax_out || !scale_out || !inv_scale_out) return F8_ERR_NULL;
    if (g == F8_COLWISE && !aligned16(scale_out)) return F8_ERR_ALIGN;
    s = check_cast_outputs(rows, cols, out, ld_out, out_t, ld_out_t);
    if (s != F8_OK) return s;
    if (g != F8_ROWWISE && (!workspace || workspace_bytes_ < quantise_workspace_bytes(rows, cols))) return F8_ERR_WORKSPACE;
    return quantise(x_bf16, rows, cols, ld, g, fmt, amax_out, scale_out, inv_scale_out, out, ld_out, out_t,
                    ld_out_t, workspace, (hipStream_t)stream);
}

f8_status f8_cast_amax(const void* x_bf16, int64_t rows, int64_t cols, int64_t ld, const float* scale,
                       f8_format fmt, uint8_t* out, int64_t ld_out, uint8_t* out_t, int64_t ld_out_t,
                       float* amax_out, void* workspace, size_t workspace_bytes_, void* stream)
{
    if ((int)fmt < 0 || (int)fmt > F8_E5M2) return F8_ERR_ENUM;
    f8_status s = check_matrix(x_bf16, rows, cols, ld);
    if (s != F8_OK) return s;
    if (!scale || !amax_out) return F8_ERR_NULL;
    s = check_cast_outputs(rows, cols, out, ld_out, out_t, ld_out_t);
    if (s != F8_OK) return s;
    if (!workspace || workspace_bytes_ < quantise_workspace_bytes(rows, cols)) return F8_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    int np = 0;
    s = cast_measure(x_bf16, rows, cols, ld, scale, fmt, out, ld_out, out_t, ld_out_t, workspace,
                     workspace_bytes_, &np, st, 0, nullptr);
    if (s != F8_OK) return s;
    amax_tensor_final_kernel<<<1, kThreads, 0, st>>>((const uint32_t*)workspace, np, 0.0f, amax_out, nullptr, nullptr);
    return last_launch_status();
}

f8_status f8_amax_history_push(float* history, int64_t len, const float* amax_new, f8_format fmt,
                               float* scale_out, float* inv_scale_out, void* stream)
{
    if ((int)fmt < 0 || (int)fmt > F8_E5M2) return F8_ERR_ENUM;
    if (!history || !amax_new || !scale_out) return F8_ERR_NULL;
    if (len < 1 || len > F8_MAX_HISTORY) return F8_ERR_SHAPE;
    return history_push(nullptr, 0, amax_new, history, len, fmt, nullptr, nullptr, nullptr, nullptr, scale_out,
                        inv_scale_out, (hipStream_t)stream);
}

f8_status f8_encode_f32(const float* y, int64_t n, f8_format fmt, int use_hw_convert, uint8_t* out,
                        void* stream)
{
    if ((int)fmt < 0 || (int)fmt > F8_E5M2) return F8_ERR_ENUM;
    if (!y || !out) return F8_ERR_NULL;
    if (n < 0) return F8_ERR_SHAPE;
    if (n == 0) return F8_OK;
    const unsigned nb = (unsigned)(((n + 1) / 2 + kThreads - 1) / kThreads);
    hipStream_t st = (hipStream_t)stream;
    if (fmt == F8_E4M3) {
        if (use_hw_convert) encode_kernel<F8_E4M3, true><<<nb, kThreads, 0, st>>>(y, n, out);
        else encode_kernel<F8_E4M3, false><<<nb, kThreads, 0, st>>>(y, n, out);
    } else {
        if (use_hw_convert) encode_kernel<F8_E5M2, true><<<nb, kThreads, 0, st>>>(y, n, out);
        else encode_kernel<F8_E5M2, false><<<nb, kThreads, 0, st>>>(y, n, out);
    }
    return last_launch_status();
}

}  // extern "C"
