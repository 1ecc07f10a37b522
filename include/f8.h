/*
 * f8.h - C ABI of the MI355X (gfx950) Float8 linear-layer library.
 *
 * The operation: the Float8 linear layer of the paper's section "Boosting
 * throughput with mixed precision training and Float8 support": a linear
 * layer whose three matrix products (forward Y = X W^T, backward dX = dY W and
 * dW = dY^T X) run on fp8 operands with dynamic scaling, i.e. each bf16 tensor
 * is scaled by FMAX / amax(tensor) computed from the tensor itself right before
 * it is cast.  Number formats are the OCP FP8 formats the paper cites
 * (Micikevicius et al., "FP8 formats for deep learning"): E4M3 (max 448, no
 * infinity) and E5M2 (max 57344).  Products accumulate in fp32; outputs are
 * bf16 (the experiments section notes that FP8 and BF16 matrix units both take
 * part in a Float8 training step).
 *
 * Conventions that hold for every entry point
 *   - Every data pointer is DEVICE memory on the current HIP device, owned by
 *     the caller.  The library never allocates, frees or synchronises.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Every call only enqueues kernels on it and returns.
 *   - Matrices are row-major; a leading dimension `ld*` is in elements.
 *   - bf16 data is passed as `const void*` / `void*` (2 bytes per element),
 *     fp8 data as uint8_t codes, scales as fp32 in device memory (they never
 *     visit the host).
 *   - Data pointers must be 16-byte aligned; rows, cols, leading dimensions and
 *     M, N, K must be multiples of 16 (zero is allowed and is a no-op apart
 *     from writing amax = 0 and its scale).  Violations return F8_ERR_ALIGN /
 *     F8_ERR_SHAPE.
 *   - Arguments are checked on the host before anything is launched; on an
 *     error return nothing has been enqueued or written.  A failed launch
 *     returns F8_ERR_LAUNCH.  No exception or abort crosses this boundary.
 *   - No global mutable state (f8_linear_fwd_noalloc is the one exception, see
 *     there): calls on different streams with disjoint buffers (including
 *     disjoint workspaces) may run concurrently.
 *   - Inputs are expected to be finite.  With a caller-given finite scale,
 *     f8_cast maps NaN to one of the format's NaN codes and +-Inf to the
 *     +-FMAX code; amax over non-finite data is unspecified.
 */
#ifndef F8_H
#define F8_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    F8_OK = 0,
    F8_ERR_NULL = 1,      /* a required pointer is NULL                        */
    F8_ERR_SHAPE = 2,     /* negative size, size or ld not a multiple of 16, ld too small */
    F8_ERR_ALIGN = 3,     /* a data pointer is not 16-byte aligned             */
    F8_ERR_ENUM = 4,      /* an enum argument is out of range                  */
    F8_ERR_WORKSPACE = 5, /* workspace NULL or smaller than required           */
    F8_ERR_LAUNCH = 6     /* the HIP runtime refused a kernel launch           */
} f8_status;

/* OCP FP8 formats.  E4M3: 4 exponent bits, bias 7, NaN = S.1111.111 only, max
 * finite 0x7E = 448.  E5M2: 5 exponent bits, bias 15, IEEE-like, max finite
 * 0x7B = 57344. */
typedef enum { F8_E4M3 = 0, F8_E5M2 = 1 } f8_format;

/* How many scales a [rows, cols] tensor has: one, one per row, one per column. */
typedef enum { F8_TENSORWISE = 0, F8_ROWWISE = 1, F8_COLWISE = 2 } f8_granularity;

/* Operand layouts of f8_gemm; D is always [M, N].
 *   F8_NT: A[M,K], B[N,K]   (both contraction-contiguous)
 *   F8_NN: A[M,K], B[K,N]
 *   F8_TN: A[K,M], B[K,N]
 * All three run on the same tiled kernel when K is a multiple of 256 (operands
 * whose contraction index is the slow one are turned inside the kernel);
 * otherwise a slower generic kernel takes over. */
typedef enum { F8_NT = 0, F8_NN = 1, F8_TN = 2 } f8_layout;

/* Bytes of device workspace that is enough for any call of this library on
 * tensors of at most max_rows x max_cols (for a linear layer: the largest of
 * M, K, N in both arguments).  The workspace holds partial maxima of the
 * quantisation and, in the backward of a linear whose weight gradient has few
 * output tiles and a long contraction, fp32 partial sums of that product (at
 * most 64 MiB); it needs no initialisation and carries no state between calls.
 * The quantisation calls on their own (f8_amax, f8_cast_amax, f8_amax_cast,
 * f8_quantise, the fused glue casts) accept less: 64 * max(rows, cols) * 4 +
 * ceil(cols / 128) * rows * 4 bytes, at least 8 KiB. */
size_t f8_workspace_bytes(int64_t max_rows, int64_t max_cols);

const char* f8_status_string(f8_status s);

/*
 * Step 1 of dynamic scaling: amax = max |x| of a bf16 matrix [rows, cols].
 *   g = F8_TENSORWISE: amax_out[0];  F8_ROWWISE: amax_out[rows] (max over the
 *   columns of each row);  F8_COLWISE: amax_out[cols] (max over the rows of
 *   each column).  Exact (it is one of the inputs' magnitudes).
 * workspace: f8_workspace_bytes(rows, cols) bytes (unused for F8_ROWWISE; may be NULL then).
 */
f8_status f8_amax(const void* x_bf16, int64_t rows, int64_t cols, int64_t ld, f8_granularity g,
                  float* amax_out, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Step 2: scale[i] = FMAX(fmt) / max(amax[i], 1e-12f) and inv_scale[i] =
 * 1.0f / scale[i], both single correctly rounded fp32 divisions.  n >= 0
 * entries; inv_scale_out may be NULL.
 */
f8_status f8_scale(const float* amax, int64_t n, f8_format fmt, float* scale_out,
                   float* inv_scale_out, void* stream);

/*
 * Step 3: code = fp8_rne( clamp( fp32(x) * scale, -FMAX, +FMAX ) ): one fp32
 * multiply (rounded), saturation, then round-to-nearest-even to the fp8 grid.
 *   scale: 1, rows or cols entries according to g.
 *   out   [rows, cols] (ld_out >= cols) and/or
 *   out_t [cols, rows] (ld_out_t >= rows), the same codes transposed.
 * At least one of out / out_t must be non-NULL.
 */
f8_status f8_cast(const void* x_bf16, int64_t rows, int64_t cols, int64_t ld, const float* scale,
                  f8_granularity g, f8_format fmt, uint8_t* out, int64_t ld_out, uint8_t* out_t,
                  int64_t ld_out_t, void* stream);

/*
 * The rounding of step 3 alone, on fp32 inputs that are already scaled:
 * out[i] = fp8_rne( clamp( y[i], -FMAX, +FMAX ) ), n >= 0 elements, no
 * alignment requirement.  use_hw_convert = 0 rounds with integer arithmetic,
 * 1 with the chip's packed fp32->fp8 conversion instruction; the two must
 * agree (this entry point exists so that tests can show they do).
 */
f8_status f8_encode_f32(const float* y, int64_t n, f8_format fmt, int use_hw_convert, uint8_t* out,
                        void* stream);

/*
 * Steps 1-3 fused as the hot path uses them (dynamic scaling): writes
 * amax_out, scale_out, inv_scale_out (1, rows or cols entries; all required)
 * and the codes.  Results are identical to f8_amax -> f8_scale -> f8_cast.
 * workspace: f8_workspace_bytes(rows, cols) bytes (may be NULL for F8_ROWWISE).
 */
f8_status f8_amax_cast(const void* x_bf16, int64_t rows, int64_t cols, int64_t ld,
                       f8_granularity g, f8_format fmt, float* amax_out, float* scale_out,
                       float* inv_scale_out, uint8_t* out, int64_t ld_out, uint8_t* out_t,
                       int64_t ld_out_t, void* workspace, size_t workspace_bytes, void* stream);

/*
 * The other two per-tensor scaling strategies the paper's Float8 section names
 * beside dynamic scaling: DELAYED (the scale comes from the amax values of
 * earlier steps) and STATIC (the scale is a constant the caller chose).  In
 * both the scale is known before the tensor is read, so the cast is a single
 * pass over x (2 B read + 1 B written per element and orientation) instead of
 * dynamic scaling's two.  Tensorwise only.
 *
 * f8_cast_amax: f8_cast with a tensorwise scale[0] that also measures
 * amax_out[0] = max |x| in the same pass (the value delayed scaling records for
 * later steps).  Codes are identical to f8_cast with the same scale; values
 * beyond the scale's range saturate to +-FMAX.
 * workspace: f8_workspace_bytes(rows, cols) bytes.
 */
f8_status f8_cast_amax(const void* x_bf16, int64_t rows, int64_t cols, int64_t ld, const float* scale,
                       f8_format fmt, uint8_t* out, int64_t ld_out, uint8_t* out_t, int64_t ld_out_t,
                       float* amax_out, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Delayed scaling's amax history: history[0] is the newest entry,
 * history[len-1] the oldest, 1 <= len <= F8_MAX_HISTORY.  The call drops the
 * oldest entry, shifts the rest by one, stores amax_new[0] at history[0], then
 * writes scale_out[0] = FMAX(fmt) / max(max(history), 1e-12f) and
 * inv_scale_out[0] = 1 / scale_out[0] (inv_scale_out may be NULL).  A fresh
 * history is all zeros; an all-zero history gives the scale of an all-zero
 * tensor (FMAX / 1e-12f), so seed it with one measured amax before the first
 * delayed cast.
 */
#define F8_MAX_HISTORY 1024
f8_status f8_amax_history_push(float* history, int64_t len, const float* amax_new, f8_format fmt,
                               float* scale_out, float* inv_scale_out, void* stream);

/*
 * fp8 GEMM with fp32 accumulation and bf16 output:
 *   D[m,n] = bf16_rne( (sum_k dec(A)[m,k] * dec(B)[n,k]) * inv_scale_a * inv_scale_b )
 * fa / fb: format of A / B codes (mixed E5M2 x E4M3 is allowed).
 * g = F8_TENSORWISE: inv_scale_a[0], inv_scale_b[0].
 * g = F8_ROWWISE:    inv_scale_a[M] (per output row), inv_scale_b[N] (per output column).
 * F8_COLWISE is not a GEMM mode (F8_ERR_ENUM).
 * M, N, K and the leading dimensions must be below 2^23 (F8_ERR_SHAPE); the
 * same bound holds for M, K, N of the linear-layer calls.
 * Summation order is unspecified (results agree with any fp32 order within
 * accumulation rounding).
 * amax_d (nullable, device, 1 float): if given, receives max |D[m,n]| over the
 * bf16 values stored by this call, taken in the epilogue while they are still
 * in registers: the amax a following Float8 linear (dynamic or delayed
 * scaling) needs of its input, without another pass over D.  It is the exact
 * maximum of the stored values (0 for an empty D).
 */
f8_status f8_gemm(f8_layout layout, int64_t M, int64_t N, int64_t K, const uint8_t* A, f8_format fa,
                  int64_t lda, const uint8_t* B, f8_format fb, int64_t ldb, const float* inv_scale_a,
                  const float* inv_scale_b, f8_granularity g, void* D_bf16, int64_t ldd,
                  float* amax_d, void* stream);

/*
 * f8_gemm with a workspace (nullable; any size, 16-byte aligned).  A product
 * with few output tiles and a long contraction (the weight gradient of a narrow
 * linear: 64 tiles of 256 x 256 for 256 compute units) is then computed in 2, 4
 * or 8 contraction ranges, one (tile, range) per compute unit, whose unscaled
 * fp32 sums go to the workspace and are added in range order by a second
 * kernel that applies the scales and rounds to bf16: reproducible, no atomics.
 * It happens when ranges * M * N * 4 bytes fit the workspace (at most 64 MiB;
 * f8_workspace_bytes(M, N) is always enough), amax_d is NULL and the estimated
 * time is lower; otherwise the call is f8_gemm.  Results of a split product
 * differ from the unsplit one within accumulation rounding.
 */
f8_status f8_gemm_ws(f8_layout layout, int64_t M, int64_t N, int64_t K, const uint8_t* A, f8_format fa,
                     int64_t lda, const uint8_t* B, f8_format fb, int64_t ldb, const float* inv_scale_a,
                     const float* inv_scale_b, f8_granularity g, void* D_bf16, int64_t ldd,
                     float* amax_d, void* workspace, size_t workspace_bytes, void* stream);

/*
 * One quantised tensor T[rows, cols] as the linear layer keeps it between
 * forward and backward.  All members are caller-allocated device memory.
 *   Tensorwise: q [rows, cols] holds the codes; amax / scale / inv_scale have 1
 *     entry; the *_t scale members are unused (may be NULL).  q_t may be NULL
 *     (the normal case): the backward products then read q in place, turning
 *     the operand inside the GEMM kernel.  If q_t [cols, rows] is given it
 *     receives the same codes transposed (+1 byte written per element) and
 *     the backward products run on the transposed copies instead; dW does so
 *     only if both dY's and X's q_t are given.
 *   Rowwise: q is scaled per row (amax, scale, inv_scale: rows entries); q_t is
 *     the transposed tensor scaled per ITS row, i.e. per column of T (amax_t,
 *     scale_t, inv_scale_t: cols entries).  The two hold different codes.
 */
typedef struct f8_qtensor {
    uint8_t* q;
    uint8_t* q_t;
    float* amax;
    float* scale;
    float* inv_scale;
    float* amax_t;
    float* scale_t;
    float* inv_scale_t;
} f8_qtensor;

/* X [M,K], W [N,K], dY [M,N]. */
typedef struct f8_saved {
    f8_qtensor x;
    f8_qtensor w;
    f8_qtensor dy;
} f8_saved;

/*
 * The quantisation the linear layer applies to one bf16 tensor T [rows, cols]
 * (leading dimension cols) under dynamic scaling:
 *   g = F8_TENSORWISE: q->amax / scale / inv_scale (1 entry), q->q [rows, cols]
 *     and, if q->q_t is not NULL, q->q_t [cols, rows] with the same codes.
 *   g = F8_ROWWISE: q->q with one scale per row (amax, scale, inv_scale: rows
 *     entries) and q->q_t with one scale per column of T (amax_t, scale_t,
 *     inv_scale_t: cols entries); T is read once for both casts.
 * workspace: f8_workspace_bytes(rows, cols) bytes.
 */
f8_status f8_quantise(const void* t_bf16, int64_t rows, int64_t cols, f8_granularity g, f8_format fmt,
                      const f8_qtensor* q, void* workspace, size_t workspace_bytes, void* stream);

typedef struct f8_linear_desc {
    int64_t M, K, N;
    int32_t granularity; /* F8_TENSORWISE or F8_ROWWISE */
    int32_t grad_format; /* f8_format of dY; X and W are always E4M3 */
} f8_linear_desc;

/*
 * Forward of the Float8 linear: quantise X [M,K] and W [N,K] (bf16) with
 * dynamic scaling into saved->x, saved->w (kept for the backward), then
 * Y [M,N] (bf16) = X8 W8^T with the scales folded into the epilogue.
 * Rowwise: Y uses X per row m and W per row n.
 */
f8_status f8_linear_fwd(const f8_linear_desc* d, const void* X, const void* W, void* Y,
                        f8_saved* saved, void* workspace, size_t workspace_bytes, void* stream);

/*
 * The quantisation half of f8_linear_fwd alone (steps 1-3 of dynamic scaling,
 * Section 2.2.4, for X and W; no product): fills saved->x and saved->w exactly
 * as f8_linear_fwd does and with the same launches - tensorwise without
 * transposed copies, ONE amax launch and ONE cast launch serve both tensors
 * (the grid is split between them by size).  f8_linear_fwd is this call
 * followed by f8_gemm(F8_NT) on the codes.  Same arguments, checks and
 * workspace as f8_linear_fwd, minus Y.
 */
f8_status f8_linear_fwd_quantise(const f8_linear_desc* d, const void* X, const void* W, f8_saved* saved,
                                 void* workspace, size_t workspace_bytes, void* stream);

/*
 * f8_linear_fwd with the weight already quantised: saved->w holds W's codes
 * and its scales from an earlier f8_linear_fwd (or f8_quantise) — weights
 * change once per optimizer step, not per micro-batch.  (Under dynamic scaling
 * as this library reads Section 2.2.4 the weight is recast on every forward;
 * keeping the codes is the caller's choice.)  Quantises X, computes
 * Y = X8 W8^T.
 */
f8_status f8_linear_fwd_wq(const f8_linear_desc* d, const void* X, void* Y, f8_saved* saved, void* workspace,
                           size_t workspace_bytes, void* stream);

/*
 * f8_linear_fwd for callers that cannot allocate and have no workspace to
 * pass: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments minus the workspace, same results bit for
 * bit.  The partial maxima that f8_linear_fwd keeps in the caller's workspace
 * live in a built-in device array of F8_NOALLOC_SCRATCH_BYTES (8 MiB) that each
 * GPU the library runs on holds until the process ends; the call allocates and
 * frees nothing and calls no allocating routine.  Its first call on a device
 * looks up the array's address there (hipGetSymbolAddress), so make that call
 * outside a stream capture.
 * Limits: tensorwise scaling fits for every shape; rowwise scaling needs the
 * partial maxima of its larger tensor T [rows, cols] (X [M,K] or W [N,K]):
 * 64 * max(rows, cols) * 4 + ceil(cols / 128) * rows * 4 bytes, and a shape
 * needing more than the array returns F8_ERR_WORKSPACE with nothing launched.
 * This is the library's only shared state: every call on a GPU uses that GPU's
 * one array (nothing in it has to be cleared between calls: each quantisation
 * writes its partial maxima before it reads them), so calls that overlap on one
 * GPU - on different streams, or from different threads - race; serialise them.
 */
#define F8_NOALLOC_SCRATCH_BYTES (8u << 20)
f8_status f8_linear_fwd_noalloc(const f8_linear_desc* d, const void* X, const void* W, void* Y,
                                f8_saved* saved, void* stream);

/*
 * Backward: quantise dY [M,N] into saved->dy, then
 *   dX [M,K] = dY8 W8      (rowwise: dY per row m, W per column k)
 *   dW [N,K] = dY8^T X8    (rowwise: dY per column n, X per column k)
 * using saved->x and saved->w from the forward call.
 */
f8_status f8_linear_bwd(const f8_linear_desc* d, const void* dY, f8_saved* saved, void* dX,
                        void* dW, void* workspace, size_t workspace_bytes, void* stream);

/*
 * The linear layer under delayed or static scaling (tensorwise; the
 * descriptor's granularity must be F8_TENSORWISE).
 *
 * state->mode = F8_DELAYED: every tensor T in {X, W, dY} is cast with the
 *   scale found in state->scale_T[0] when the call starts.  saved->T then
 *   holds the codes, that scale, its reciprocal, and the amax of THIS step's
 *   tensor; the amax is pushed into state->hist_T (f8_amax_history_push) and
 *   state->scale_T[0] becomes the scale for the next step.  Seed each
 *   scale_T / hist_T before the first step (e.g. f8_amax on a first batch, then
 *   f8_amax_history_push).
 * state->mode = F8_STATIC: every tensor is cast with state->scale_T[0], which
 *   is never modified; saved->T gets the codes, the scale and its reciprocal;
 *   saved->T.amax is not written and the hist_* members are unused.
 * state->mode = F8_DYNAMIC: same as f8_linear_fwd / f8_linear_bwd; the state's
 *   pointers are unused.
 * The forward call uses the x and w members of the state, the backward call
 * the dy members.  All state members are caller-owned device memory.
 */
typedef enum { F8_DYNAMIC = 0, F8_DELAYED = 1, F8_STATIC = 2 } f8_scaling;

typedef struct f8_scaling_state {
    int32_t mode;        /* f8_scaling */
    int32_t history_len; /* entries of each hist_* array (F8_DELAYED), 1 .. F8_MAX_HISTORY */
    float* hist_x;
    float* hist_w;
    float* hist_dy;
    float* scale_x; /* 1 entry each: the scale the next cast of that tensor uses */
    float* scale_w;
    float* scale_dy;
} f8_scaling_state;

f8_status f8_linear_fwd_scaled(const f8_linear_desc* d, const f8_scaling_state* state, const void* X,
                               const void* W, void* Y, f8_saved* saved, void* workspace,
                               size_t workspace_bytes, void* stream);

f8_status f8_linear_bwd_scaled(const f8_linear_desc* d, const f8_scaling_state* state, const void* dY,
                               f8_saved* saved, void* dX, void* dW, void* workspace,
                               size_t workspace_bytes, void* stream);

/*
 * The dynamic-scaling linear for a chain of Float8 linears, where one layer's
 * output is the next layer's input: the amax of a GEMM output is taken in that
 * GEMM's epilogue (see f8_gemm, amax_d) and handed to the consumer, whose
 * quantisation of that tensor then needs a single pass (cast only) instead of
 * two (amax, then cast).  Tensorwise only.
 *
 * f8_linear_fwd_chained: as f8_linear_fwd, but
 *   x_amax (nullable, device, 1 float): amax of X, e.g. the y_amax of the
 *     producing layer.  It must be exactly max |X| for the result to equal
 *     f8_linear_fwd's; NULL: the amax pass runs as usual.
 *   y_amax (nullable, device, 1 float): receives max |Y|.
 * f8_linear_bwd_chained: as f8_linear_bwd, with dy_amax given (nullable) and
 *   dx_amax (nullable) receiving max |dX| for the layer below.
 */
f8_status f8_linear_fwd_chained(const f8_linear_desc* d, const void* X, const float* x_amax,
                                const void* W, void* Y, float* y_amax, f8_saved* saved,
                                void* workspace, size_t workspace_bytes, void* stream);

f8_status f8_linear_bwd_chained(const f8_linear_desc* d, const void* dY, const float* dy_amax,
                                f8_saved* saved, void* dX, float* dx_amax, void* dW,
                                void* workspace, size_t workspace_bytes, void* stream);

/*
 * The bf16 glue between the two Float8 linears of a Llama feed-forward block
 * (the paper trains Llama 3.1 models; their feed-forward is
 * Y = W2 ( silu(W1 x) * (W3 x) ), silu(t) = t / (1 + e^-t)).  W1 and W3 are
 * stacked into one linear of width 2H whose output row is [a | b].
 *
 * f8_silu_mul:     ab [M, 2H] bf16 -> h [M, H] bf16, h = silu(a) * b.
 * f8_silu_mul_bwd: ab [M, 2H], dh [M, H] -> dab [M, 2H] = [dh * b * silu'(a) | dh * silu(a)].
 * Arithmetic is fp32 with one rounding to bf16 at the end; results agree with
 * the exact functions to within one bf16 unit in the last place.
 * amax_h / amax_dab (nullable, device, 1 float): receives the exact maximum
 * magnitude of the bf16 values written, for f8_linear_fwd_chained /
 * f8_linear_bwd_chained of the consuming linear.  workspace (needed only with
 * an amax output): f8_workspace_bytes(M, 2 * H) bytes.  M and H multiples of 16.
 */
f8_status f8_silu_mul(const void* ab_bf16, int64_t M, int64_t H, void* h_bf16, float* amax_h,
                      void* workspace, size_t workspace_bytes, void* stream);

f8_status f8_silu_mul_bwd(const void* ab_bf16, const void* dh_bf16, int64_t M, int64_t H,
                          void* dab_bf16, float* amax_dab, void* workspace, size_t workspace_bytes,
                          void* stream);

/*
 * RMS normalisation in front of a Llama block's attention and feed-forward
 * linears (the producer of a Float8 linear's input; f8_rmsnorm_bwd is its
 * backward):
 *   y[m, :] = x[m, :] * rstd[m] * g,   rstd[m] = 1 / sqrt(mean_d x[m, d]^2 + eps)
 * x, y [M, D] bf16, g [D] bf16; rstd (nullable) [M] fp32, kept for a backward
 * pass; amax_y (nullable, 1 float) receives the exact maximum magnitude of
 * the bf16 values written, for f8_linear_fwd_chained of the consuming linear.
 * fp32 arithmetic, one rounding to bf16: within one bf16 unit in the last
 * place of the exact result.  workspace (only with amax_y):
 * f8_workspace_bytes(M, D) bytes.  M and D multiples of 16, eps >= 0.
 */
f8_status f8_rmsnorm(const void* x_bf16, const void* g_bf16, int64_t M, int64_t D, float eps,
                     void* y_bf16, float* rstd, float* amax_y, void* workspace,
                     size_t workspace_bytes, void* stream);

/*
 * The feed-forward glue fused into the cast of its consumer, for delayed
 * scaling (where the scale is known before the tensor exists; this is the kind
 * of producer/cast fusion the paper gets from torch.compile): from ab [M, 2H]
 * = [a | b] it forms h = bf16(silu(a) * b) in registers and writes only its fp8
 * codes: q->q [M, H] (and q->q_t [H, M] if given), cast with scale[0]; q->scale / inv_scale
 * receive the scale used, q->amax the amax of h, which is then pushed into
 * history (f8_amax_history_push) and scale[0] becomes the next step's scale.
 * Same results as f8_silu_mul followed by the delayed-scaling quantisation of
 * h, without writing and re-reading h.  workspace: f8_workspace_bytes(M, H).
 */
f8_status f8_silu_mul_quantise_delayed(const void* ab_bf16, int64_t M, int64_t H, f8_format fmt,
                                       float* history, int64_t history_len, float* scale,
                                       const f8_qtensor* q, void* workspace, size_t workspace_bytes,
                                       void* stream);

/*
 * The same fusion for the backward of the glue: from ab [M, 2H] and dh [M, H]
 * it forms dab = [dh * b * silu'(a) | dh * silu(a)] in registers and writes
 * only its fp8 codes q->q [M, 2H] (and q->q_t [2H, M] if given; delayed scaling as above;
 * fmt is the gradient format).  Same results as f8_silu_mul_bwd followed by the
 * delayed-scaling quantisation of dab.  workspace: f8_workspace_bytes(M, 2H).
 */
f8_status f8_silu_mul_bwd_quantise_delayed(const void* ab_bf16, const void* dh_bf16, int64_t M, int64_t H,
                                           f8_format fmt, float* history, int64_t history_len,
                                           float* scale, const f8_qtensor* q, void* workspace,
                                           size_t workspace_bytes, void* stream);

/*
 * Backward of the linear whose output gradient is already quantised in
 * saved->dy (codes, inv_scale; in d->grad_format): the
 * two GEMMs dX = dY8 W8, dW = dY8^T X8 only.  Tensorwise only.
 */
f8_status f8_linear_bwd_dyq(const f8_linear_desc* d, f8_saved* saved, void* dX, void* dW, void* stream);

/*
 * The bf16 operations that join the Float8 linears of one transformer block
 * (Section 2.2.4 applies Float8 to the linear layers only; Section 2.1 names
 * the TransformerBlock as the unit that is wrapped, sharded and recomputed).
 *
 * f8_rope: rotary position embedding of x [M, n_heads * hd] bf16 (row pitch
 * ldx elements): row m is position m % S of its sequence; within each head
 * the adjacent pair (x[2i], x[2i+1]) is turned by the angle
 * pos * theta^(-2i/hd) (by its negative when inverse != 0: the backward).
 * out (nullable) [M, n_heads * hd], row pitch ldo; out_t (nullable) the same
 * values transposed, [n_heads * hd, M] packed: the copy that the attention
 * backward contracts over tokens.  Angle and its reduction in fp64, sine and
 * cosine and the rotation in fp32, one rounding to bf16.  hd a multiple of 8
 * and <= 256, M and the pitches multiples of 8.
 *
 * amax_inout (nullable, 1 float, also in f8_rmsnorm_bwd_add and f8_sdpa_bwd):
 * raised to the maximum magnitude of the bf16 values this call writes if that is
 * larger (the caller sets it to 0 before the first producer of a tensor that
 * several calls assemble, such as the gradient of a fused q|k|v output); exact
 * and independent of the order of the updates.
 *
 * f8_transpose_bf16: out_t [cols, rows] packed = x [rows, cols]^T (pitch ldx).
 * f8_add: out = bf16(a + b) over n elements (the residual), n multiple of 8.
 */
f8_status f8_rope(const void* x_bf16, int64_t ldx, int64_t M, int64_t S, int64_t n_heads, int64_t hd,
                  double theta, int inverse, void* out_bf16, int64_t ldo, void* out_t_bf16,
                  float* amax_inout, void* stream);
f8_status f8_transpose_bf16(const void* x_bf16, int64_t ldx, int64_t rows, int64_t cols, void* out_t_bf16,
                            void* stream);
f8_status f8_add(const void* a_bf16, const void* b_bf16, int64_t n, void* out_bf16, void* stream);

/*
 * Causal grouped-query attention of B sequences of S tokens (token m = b * S +
 * position), Hq query heads, Hkv key/value heads (query head h reads key/value
 * head h / (Hq / Hkv)), head dimension hd = 128:
 *   O[q, h] = sum_k P[q, k] v[k],  P = softmax over k <= q of (q . k) / sqrt(hd)
 * q [B*S, Hq*hd] (pitch ldq), k [B*S, Hkv*hd] (pitch ldk): bf16, after the
 * rotary embedding; vt [Hkv*hd, B*S] packed: the values TRANSPOSED
 * (f8_transpose_bf16 of v); o [B*S, Hq*hd] (pitch ldo) bf16; lse [Hq, B*S]
 * fp32: the log of the softmax denominator (natural log, scaled scores), kept
 * for the backward.  Scores and probabilities are never written: bf16 matrix
 * instructions with fp32 accumulation, online softmax, probabilities rounded to
 * bf16 before they multiply the values.  amax_o (nullable, 1 float) receives
 * the exact maximum magnitude of the bf16 values written to o, for
 * f8_linear_fwd_chained of the output projection.  S and the pitches
 * multiples of 8.
 */
f8_status f8_sdpa_fwd(const void* q_bf16, int64_t ldq, const void* k_bf16, int64_t ldk, const void* vt_bf16,
                      int64_t B, int64_t S, int64_t Hq, int64_t Hkv, int64_t hd, void* o_bf16,
                      int64_t ldo, float* lse, float* amax_o, void* stream);

/*
 * Backward of f8_sdpa_fwd.  With P recomputed from lse and delta[q] = sum_d dO O:
 *   dV = P^T dO,  dP = dO V^T,  dS = P (dP - delta),
 *   dQ = dS K / sqrt(hd),  dK = dS^T Q / sqrt(hd)
 * (the gradients of the query heads that share a key/value head are summed).
 * Token-major inputs: q, k, v, o, do (with their pitches); the copies that are
 * contiguous along tokens, packed with pitch B*S: qt [Hq*hd, B*S], kt
 * [Hkv*hd, B*S] (f8_rope's transposed outputs) and dot [Hq*hd, B*S]
 * (f8_transpose_bf16 of do); lse from the forward.  Outputs: dq [B*S, Hq*hd],
 * dk, dv [B*S, Hkv*hd] bf16 with their pitches (dq and dk are gradients of the
 * ROTATED q and k: f8_rope with inverse != 0 turns them back), and delta
 * [Hq, B*S] fp32, scratch that the call fills.  With grouped heads (Hq > Hkv)
 * every query head's share of dk and dv is kept in fp32 in the workspace
 * (f8_sdpa_bwd_workspace_bytes: 2 * B*S * Hq*hd * 4 bytes; 0 and no workspace
 * when Hq == Hkv) and the shares are summed in head order.  No atomics:
 * results are reproducible.  dS and P are rounded to bf16 before they enter a
 * product.  amax_dv_inout (nullable; grouped heads only, else F8_ERR_ENUM): see
 * f8_rope.
 */
f8_status f8_sdpa_bwd(const void* q_bf16, int64_t ldq, const void* qt_bf16, const void* k_bf16, int64_t ldk,
                      const void* kt_bf16, const void* v_bf16, int64_t ldv, const void* o_bf16,
                      int64_t ldo, const void* do_bf16, int64_t lddo, const void* dot_bf16,
                      const float* lse, int64_t B, int64_t S, int64_t Hq, int64_t Hkv, int64_t hd,
                      void* dq_bf16, int64_t lddq, void* dk_bf16, int64_t lddk, void* dv_bf16,
                      int64_t lddv, float* delta, float* amax_dv_inout, void* workspace,
                      size_t workspace_bytes, void* stream);
size_t f8_sdpa_bwd_workspace_bytes(int64_t B, int64_t S, int64_t Hq, int64_t Hkv, int64_t hd);

/*
 * Backward of f8_rmsnorm: with r = rstd[m] from the forward,
 *   dx[m, :] = r * (g . dy[m, :]) - x[m, :] * r^3 * mean_d(x . g . dy)[m]
 *   dg[d]    = sum_m dy[m, d] * x[m, d] * r[m]
 * x, dy, dx [M, D] bf16, g [D] bf16, rstd [M] fp32, dg [D] fp32.  dx or dg may
 * be NULL (not both).  fp32 arithmetic; the sums over rows are taken in a fixed
 * order (results are reproducible).  workspace (only with dg):
 * f8_workspace_bytes(M, D) bytes.  M and D multiples of 16.
 */
f8_status f8_rmsnorm_bwd(const void* x_bf16, const void* g_bf16, const float* rstd, const void* dy_bf16,
                         int64_t M, int64_t D, void* dx_bf16, float* dg, void* workspace,
                         size_t workspace_bytes, void* stream);
/* The same with the residual branch's gradient added: dx = bf16(add + bf16(dx above)), the bits
 * that f8_rmsnorm_bwd followed by f8_add gives, without writing and re-reading the first. */
f8_status f8_rmsnorm_bwd_add(const void* x_bf16, const void* g_bf16, const float* rstd, const void* dy_bf16,
                             const void* add_bf16, int64_t M, int64_t D, void* dx_bf16, float* dg,
                             float* amax_dx_inout, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Forward of the linear whose input is already quantised in saved->x (codes in
 * saved->x.q, scale, inv_scale; e.g. by f8_silu_mul_quantise_delayed):
 * quantises W [N,K] as state->mode says (the w members of the state; for
 * F8_DYNAMIC they are unused), then Y = X8 W8^T.  Tensorwise only.
 */
f8_status f8_linear_fwd_xq(const f8_linear_desc* d, const f8_scaling_state* state, const void* W,
                           void* Y, f8_saved* saved, void* workspace, size_t workspace_bytes,
                           void* stream);

/*
 * Measuring helpers (not part of the linear layer): what the chip delivers
 * with nothing else in the way, so that a benchmark can quote the kernels
 * above against measured ceilings beside the nominal peaks.
 *
 * f8_probe_mfma: one wavefront per SIMD on every compute unit issues fp8
 *   matrix instructions (E4M3 x E4M3) on register operands only, in the operand
 *   pairing of a 128 x 128 wavefront tile: the GEMM kernel's matrix work with no
 *   LDS and no memory traffic.  shape 0: iters x 64 of 16x16x128 (the
 *   instruction and tile of the GEMM kernel; eight A and eight B fragments);
 *   shape 1: iters x 32 of 32x32x64 (the other fp8 instruction of the same
 *   nominal rate; four and four fragments): the same work per iteration.  The
 *   fragments are read once from `operands` (operand_bytes: a power of two,
 *   128 KiB .. 1 GiB, 32-byte aligned; fill it with the codes whose switching
 *   activity is to be measured: constant, or a quantised tensor).  iters up to
 *   2^19.  flops_out (host, nullable) receives the floating-point operations of
 *   the launch; ticks (device, nullable, 2 words): shader-clock cycles and
 *   100 MHz ticks that workgroup 0 spent in its loop; sink: one float of device
 *   memory that is (practically) never written.
 * f8_probe_copy / f8_probe_read: grid-stride 16-byte copy of `bytes` bytes
 *   (read + write) / read of them; bytes a multiple of 16.  The copy is also
 *   the kernel of known size against which the HBM byte counters are scaled.
 * f8_probe_clock: many small workgroups each read the shader-clock cycle
 *   counter and the 100 MHz counter and file them under the compute unit they
 *   run on (the counters of different units need not agree): slot u of `out`
 *   (F8_PROBE_CLOCK_SLOTS slots of 4 words, device memory that the caller
 *   zeroes first) gets out[4 u + 0] = 1 (filled), out[4 u + 1] = cycles,
 *   out[4 u + 2] = 100 MHz ticks.  Compare two calls (before and after a region
 *   on one stream) slot by slot: mean shader clock = 0.1 GHz x d(cycles) /
 *   d(ticks), averaged over the slots filled in both.
 */
f8_status f8_probe_mfma(int shape, const uint8_t* operands, int64_t operand_bytes, int iters, uint64_t* ticks,
                        float* sink, int64_t* flops_out, void* stream);
f8_status f8_probe_copy(const void* src, void* dst, int64_t bytes, void* stream);
f8_status f8_probe_read(const void* src, int64_t bytes, uint32_t* sink, void* stream);
#define F8_PROBE_CLOCK_SLOTS 2048
f8_status f8_probe_clock(uint64_t* out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* F8_H */
