// The Float8 linear layer: forward and backward as compositions of the
// quantisation (amax -> scale -> cast) and the fp8 GEMM, all enqueued on one
// stream with no host synchronisation in between.
//
// Tensorwise scaling keeps ONE code tensor per operand; the backward products read them in
// the orientation they were written in (the GEMM kernel turns k-major operands on their way
// from LDS to the registers):
//   Y  [M,N] = X8  [M,K] . W8 [N,K]^T     F8_NT, contraction K
//   dX [M,K] = dY8 [M,N] . W8 [N,K]       F8_NN, contraction N
//   dW [N,K] = dY8 [M,N]^T . X8 [M,K]     F8_TN, contraction M
// A caller that also passes transposed code tensors (q_t) gets them filled, and the backward
// then runs as F8_NT products on them.  Rowwise scaling needs two differently scaled code sets
// per tensor anyway (per row for one product, per column for the other); the second is kept
// transposed in q_t.
#include <mutex>

#include "f8_host.hpp"

namespace f8 {

static f8_status check_desc(const f8_linear_desc* d)
{
    if (!d) return F8_ERR_NULL;
    if (d->granularity != F8_TENSORWISE && d->granularity != F8_ROWWISE) return F8_ERR_ENUM;
    if (d->grad_format != F8_E4M3 && d->grad_format != F8_E5M2) return F8_ERR_ENUM;
    if (d->M < 0 || d->K < 0 || d->N < 0 || (d->M % 16) || (d->K % 16) || (d->N % 16)) return F8_ERR_SHAPE;
    if (d->M >= (1 << 23) || d->K >= (1 << 23) || d->N >= (1 << 23)) return F8_ERR_SHAPE;
    return F8_OK;
}

static f8_status check_q(const f8_qtensor* q, bool rowwise)
{
    if (!q->q || !q->amax || !q->scale || !q->inv_scale) return F8_ERR_NULL;
    if (rowwise && (!q->q_t || !q->amax_t || !q->scale_t || !q->inv_scale_t)) return F8_ERR_NULL;
    if (!aligned16(q->q) || !aligned16(q->q_t)) return F8_ERR_ALIGN;  // a null q_t counts as aligned
    if (rowwise && (!aligned16(q->scale) || !aligned16(q->inv_scale) || !aligned16(q->scale_t) ||
                    !aligned16(q->inv_scale_t)))
        return F8_ERR_ALIGN;
    return F8_OK;
}

static size_t linear_workspace(const f8_linear_desc* d)
{
    int64_t m = d->M > d->K ? d->M : d->K;
    m = m > d->N ? m : d->N;
    return workspace_bytes(m, m);
}

// Quantise T[rows, cols] into q (and q_t).  Tensorwise: q, and the same codes transposed if the
// caller keeps a q_t.
// Rowwise: q with per-row scales, q_t with per-column scales (different codes): the two amax
// sets from one pass over T, then one cast pass that writes both.
static f8_status quantise_both(const void* T, int64_t rows, int64_t cols, bool rowwise, int fmt,
                               const f8_qtensor* q, void* ws, hipStream_t st)
{
    if (!rowwise)
        return quantise(T, rows, cols, cols, F8_TENSORWISE, fmt, q->amax, q->scale, q->inv_scale, q->q, cols,
                        q->q_t, rows, ws, st);
    f8_status s;
    if (rows > 0 && cols > 0) {
        s = amax_rows_and_cols(T, rows, cols, cols, fmt, q->amax, q->scale, q->inv_scale, q->amax_t, q->scale_t,
                               q->inv_scale_t, ws, st);
    } else {  // an empty tensor still publishes amax 0 and its scale along the non-empty axis
        s = amax_scales(T, rows, cols, cols, F8_ROWWISE, fmt, q->amax, q->scale, q->inv_scale, ws, st);
        if (s != F8_OK) return s;
        s = amax_scales(T, rows, cols, cols, F8_COLWISE, fmt, q->amax_t, q->scale_t, q->inv_scale_t, ws, st);
    }
    if (s != F8_OK) return s;
    return cast_rows_and_cols(T, rows, cols, cols, fmt, q->scale, q->scale_t, q->q, cols, q->q_t, rows, st);
}

// X and W of a forward under dynamic scaling.  Tensorwise: one amax launch and one cast launch
// for the two tensors together.
static f8_status quantise_xw(const f8_linear_desc* d, const void* X, const void* W, const f8_saved* saved, void* ws,
                             hipStream_t st)
{
    if (d->granularity != F8_ROWWISE) {
        const f8_qtensor *x = &saved->x, *w = &saved->w;
        return quantise_pair(X, d->M, d->K, x->amax, x->scale, x->inv_scale, x->q, x->q_t, W, d->N, d->K, w->amax,
                             w->scale, w->inv_scale, w->q, w->q_t, F8_E4M3, ws, st);
    }
    f8_status s = quantise_both(X, d->M, d->K, true, F8_E4M3, &saved->x, ws, st);
    if (s != F8_OK) return s;
    return quantise_both(W, d->N, d->K, true, F8_E4M3, &saved->w, ws, st);
}

// One tensor under delayed or static scaling: cast with the state's scale into both
// orientations; delayed also records the tensor's amax and derives the next scale.
static f8_status quantise_scaled(const void* T, int64_t rows, int64_t cols, int fmt, int mode, int64_t hist_len,
                                 float* hist, float* state_scale, const f8_qtensor* q, void* ws,
                                 size_t ws_bytes, hipStream_t st, int glue = 0, const void* T2 = nullptr)
{
    f8_status s;
    if (mode == F8_STATIC) {
        if ((s = cast_given(T, rows, cols, cols, state_scale, fmt, q->q, cols, q->q_t, rows, st)) != F8_OK) return s;
        return publish_scale(state_scale, q->scale, q->inv_scale, st);
    }
    int np = 0;
    if ((s = cast_measure(T, rows, cols, glue == 1 ? 2 * cols : cols, state_scale, fmt, q->q, cols, q->q_t, rows, ws,
                          ws_bytes, &np, st, glue, T2)) != F8_OK)
        return s;
    return history_push(ws, np, nullptr, hist, hist_len, fmt, q->amax, state_scale, q->scale, q->inv_scale,
                        state_scale, nullptr, st);
}

static f8_status check_state(const f8_scaling_state* st, bool fwd)
{
    if (!st) return F8_ERR_NULL;
    if (st->mode != F8_DYNAMIC && st->mode != F8_DELAYED && st->mode != F8_STATIC) return F8_ERR_ENUM;
    if (st->mode == F8_DYNAMIC) return F8_OK;
    if (fwd ? (!st->scale_x || !st->scale_w) : !st->scale_dy) return F8_ERR_NULL;
    if (st->mode == F8_DELAYED) {
        if (st->history_len < 1 || st->history_len > F8_MAX_HISTORY) return F8_ERR_SHAPE;
        if (fwd ? (!st->hist_x || !st->hist_w) : !st->hist_dy) return F8_ERR_NULL;
    }
    return F8_OK;
}

// Argument checks shared by the forward entry points (every check before any launch).
static f8_status check_fwd(const f8_linear_desc* d, bool tensorwise_only, const void* X, const void* W, const void* Y,
                           const f8_saved* saved, const void* ws, size_t ws_bytes, bool check_workspace = true)
{
    f8_status s = check_desc(d);
    if (s != F8_OK) return s;
    if (tensorwise_only && d->granularity != F8_TENSORWISE) return F8_ERR_ENUM;
    if (!X || !W || !Y || !saved) return F8_ERR_NULL;
    if (!aligned16(X) || !aligned16(W) || !aligned16(Y)) return F8_ERR_ALIGN;
    const bool rw = d->granularity == F8_ROWWISE;
    if ((s = check_q(&saved->x, rw)) != F8_OK) return s;
    if ((s = check_q(&saved->w, rw)) != F8_OK) return s;
    if (check_workspace && (!ws || ws_bytes < linear_workspace(d))) return F8_ERR_WORKSPACE;
    return F8_OK;
}

static f8_status check_bwd(const f8_linear_desc* d, bool tensorwise_only, const void* dY, const f8_saved* saved,
                           const void* dX, const void* dW, const void* ws, size_t ws_bytes)
{
    f8_status s = check_desc(d);
    if (s != F8_OK) return s;
    if (tensorwise_only && d->granularity != F8_TENSORWISE) return F8_ERR_ENUM;
    if (!dY || !dX || !dW || !saved) return F8_ERR_NULL;
    if (!aligned16(dY) || !aligned16(dX) || !aligned16(dW)) return F8_ERR_ALIGN;
    const bool rw = d->granularity == F8_ROWWISE;
    if ((s = check_q(&saved->x, rw)) != F8_OK) return s;
    if ((s = check_q(&saved->w, rw)) != F8_OK) return s;
    if ((s = check_q(&saved->dy, rw)) != F8_OK) return s;
    if (!ws || ws_bytes < linear_workspace(d)) return F8_ERR_WORKSPACE;
    return F8_OK;
}

// Y [M,N] = X8 [M,K] . (W8 [N,K])^T, scales in the epilogue; y_amax may be null.
static f8_status gemm_fwd(const f8_linear_desc* d, const f8_saved* sv, void* Y, float* y_amax, hipStream_t st)
{
    return gemm(F8_NT, d->M, d->N, d->K, sv->x.q, F8_E4M3, d->K, sv->w.q, F8_E4M3, d->K, sv->x.inv_scale,
                sv->w.inv_scale, d->granularity, Y, d->N, y_amax, st);
}

// dX [M,K] = dY8 [M,N] . W8 [N,K]: contraction N, W read k-major; with a transposed copy of W's
//   codes as dY8 . (W8t [K,N])^T.  Rowwise: dY per row m; W per column k = per row of W8t.
// dW [N,K] = dY8 [M,N]^T . X8 [M,K]: contraction M, both read k-major; with transposed copies of
//   both as dY8t [N,M] . (X8t [K,M])^T.  Rowwise: dY per column n, X per column k.
static f8_status gemms_bwd(const f8_linear_desc* d, const f8_saved* sv, void* dX, float* dx_amax, void* dW,
                           hipStream_t st, void* ws = nullptr, size_t ws_bytes = 0)
{
    const int64_t M = d->M, K = d->K, N = d->N;
    const int gf = d->grad_format;
    const bool rw = d->granularity == F8_ROWWISE;
    f8_status s;
    if (sv->w.q_t)
        s = gemm(F8_NT, M, K, N, sv->dy.q, gf, N, sv->w.q_t, F8_E4M3, N, sv->dy.inv_scale,
                 rw ? sv->w.inv_scale_t : sv->w.inv_scale, d->granularity, dX, K, dx_amax, st);
    else
        s = gemm(F8_NN, M, K, N, sv->dy.q, gf, N, sv->w.q, F8_E4M3, K, sv->dy.inv_scale, sv->w.inv_scale,
                 d->granularity, dX, K, dx_amax, st);
    if (s != F8_OK) return s;
    if (sv->dy.q_t && sv->x.q_t)
        return gemm(F8_NT, N, K, M, sv->dy.q_t, gf, M, sv->x.q_t, F8_E4M3, M, rw ? sv->dy.inv_scale_t : sv->dy.inv_scale,
                    rw ? sv->x.inv_scale_t : sv->x.inv_scale, d->granularity, dW, K, nullptr, st, ws, ws_bytes);
    return gemm(F8_TN, N, K, M, sv->dy.q, gf, N, sv->x.q, F8_E4M3, K, sv->dy.inv_scale, sv->x.inv_scale,
                d->granularity, dW, K, nullptr, st, ws, ws_bytes);
}

// ---- the forward that allocates nothing and takes no workspace ---------------------------
// Its partial maxima live in a file-scope device array instead of a caller's workspace.  In
// host code the array's name is only a handle for hipGetSymbolAddress; kernels get the device
// address that call returns, one per device (every GPU holds its own copy of the array).
constexpr size_t kScratchBytes = F8_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
static std::mutex scratch_mutex;
static void* scratch_ptr[kMaxDevices];  // device address of `scratch` per device; null = not asked yet

static f8_status scratch_of_current_device(void** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return F8_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();  // do not leave the error for a later, unrelated call
            return F8_ERR_LAUNCH;
        }
        scratch_ptr[dev] = p;
    }
    *out = scratch_ptr[dev];
    return F8_OK;
}

// What the forward's quantisations really need: the tensorwise partials fit the minimum; rowwise
// needs the per-column and per-row partials of its larger tensor.
static size_t fwd_scratch_need(const f8_linear_desc* d)
{
    if (d->granularity != F8_ROWWISE) return kMinWorkspaceBytes;
    const size_t x = quantise_workspace_bytes(d->M, d->K), w = quantise_workspace_bytes(d->N, d->K);
    return x > w ? x : w;
}

}  // namespace f8

using namespace f8;

extern "C" {

f8_status f8_linear_fwd_noalloc(const f8_linear_desc* d, const void* X, const void* W, void* Y, f8_saved* saved,
                                void* stream)
{
    f8_status s = check_fwd(d, false, X, W, Y, saved, nullptr, 0, false);
    if (s != F8_OK) return s;
    if (fwd_scratch_need(d) > kScratchBytes) return F8_ERR_WORKSPACE;  // beyond the built-in scratch
    void* ws = nullptr;
    if ((s = scratch_of_current_device(&ws)) != F8_OK) return s;
    hipStream_t st = (hipStream_t)stream;
    // the partial maxima are written before they are read within each quantisation: nothing in
    // the scratch has to start at zero
    if ((s = quantise_xw(d, X, W, saved, ws, st)) != F8_OK) return s;
    return gemm_fwd(d, saved, Y, nullptr, st);
}

const char* f8_status_string(f8_status s)
{
    switch (s) {
        case F8_OK: return "ok";
        case F8_ERR_NULL: return "a required pointer is NULL";
        case F8_ERR_SHAPE: return "bad shape: sizes and leading dimensions must be non-negative multiples of 16, ld >= cols";
        case F8_ERR_ALIGN: return "a data pointer is not 16-byte aligned";
        case F8_ERR_ENUM: return "an enum argument is out of range";
        case F8_ERR_WORKSPACE: return "workspace is NULL or too small (see f8_workspace_bytes), or the shape is beyond the built-in scratch of f8_linear_fwd_noalloc";
        case F8_ERR_LAUNCH: return "kernel launch failed";
    }
    return "unknown status";
}

f8_status f8_quantise(const void* t_bf16, int64_t rows, int64_t cols, f8_granularity g, f8_format fmt,
                      const f8_qtensor* q, void* workspace, size_t workspace_bytes_, void* stream)
{
    if (((int)g != F8_TENSORWISE && (int)g != F8_ROWWISE) || (int)fmt < 0 || (int)fmt > F8_E5M2) return F8_ERR_ENUM;
    if (!t_bf16 || !q) return F8_ERR_NULL;
    if (rows < 0 || cols < 0 || (rows % 16) || (cols % 16)) return F8_ERR_SHAPE;
    if (!aligned16(t_bf16)) return F8_ERR_ALIGN;
    f8_status s = check_q(q, g == F8_ROWWISE);
    if (s != F8_OK) return s;
    if (!workspace || workspace_bytes_ < quantise_workspace_bytes(rows, cols)) return F8_ERR_WORKSPACE;
    return quantise_both(t_bf16, rows, cols, g == F8_ROWWISE, fmt, q, workspace, (hipStream_t)stream);
}

f8_status f8_linear_fwd(const f8_linear_desc* d, const void* X, const void* W, void* Y, f8_saved* saved,
                        void* workspace, size_t workspace_bytes_, void* stream)
{
    f8_status s = check_fwd(d, false, X, W, Y, saved, workspace, workspace_bytes_);
    if (s != F8_OK) return s;
    hipStream_t st = (hipStream_t)stream;
    if ((s = quantise_xw(d, X, W, saved, workspace, st)) != F8_OK) return s;
    return gemm_fwd(d, saved, Y, nullptr, st);
}

f8_status f8_linear_fwd_quantise(const f8_linear_desc* d, const void* X, const void* W, f8_saved* saved,
                                 void* workspace, size_t workspace_bytes_, void* stream)
{
    // X stands in for Y in the shared checks, which only test it for NULL and alignment
    f8_status s = check_fwd(d, false, X, W, X, saved, workspace, workspace_bytes_);
    if (s != F8_OK) return s;
    return quantise_xw(d, X, W, saved, workspace, (hipStream_t)stream);
}

f8_status f8_linear_fwd_wq(const f8_linear_desc* d, const void* X, void* Y, f8_saved* saved, void* workspace,
                           size_t workspace_bytes_, void* stream)
{
    // the weight's codes and scales in saved->w are the caller's (kept from an earlier call): X is a
    // stand-in for W in the shared checks, which only test it for NULL and alignment
    f8_status s = check_fwd(d, false, X, X, Y, saved, workspace, workspace_bytes_);
    if (s != F8_OK) return s;
    hipStream_t st = (hipStream_t)stream;
    if ((s = quantise_both(X, d->M, d->K, d->granularity == F8_ROWWISE, F8_E4M3, &saved->x, workspace, st)) != F8_OK) return s;
    return gemm_fwd(d, saved, Y, nullptr, st);
}

f8_status f8_linear_bwd(const f8_linear_desc* d, const void* dY, f8_saved* saved, void* dX, void* dW,
                        void* workspace, size_t workspace_bytes_, void* stream)
{
    f8_status s = check_bwd(d, false, dY, saved, dX, dW, workspace, workspace_bytes_);
    if (s != F8_OK) return s;
    hipStream_t st = (hipStream_t)stream;
    if ((s = quantise_both(dY, d->M, d->N, d->granularity == F8_ROWWISE, d->grad_format, &saved->dy, workspace, st)) != F8_OK)
        return s;
    return gemms_bwd(d, saved, dX, nullptr, dW, st, workspace, workspace_bytes_);
}

f8_status f8_linear_fwd_scaled(const f8_linear_desc* d, const f8_scaling_state* state, const void* X,
                               const void* W, void* Y, f8_saved* saved, void* workspace,
                               size_t workspace_bytes_, void* stream)
{
    f8_status s = check_state(state, true);
    if (s != F8_OK) return s;
    if (state->mode == F8_DYNAMIC) return f8_linear_fwd(d, X, W, Y, saved, workspace, workspace_bytes_, stream);
    if ((s = check_fwd(d, true, X, W, Y, saved, workspace, workspace_bytes_)) != F8_OK) return s;
    hipStream_t st = (hipStream_t)stream;
    if ((s = quantise_scaled(X, d->M, d->K, F8_E4M3, state->mode, state->history_len, state->hist_x, state->scale_x,
                             &saved->x, workspace, workspace_bytes_, st)) != F8_OK)
        return s;
    if ((s = quantise_scaled(W, d->N, d->K, F8_E4M3, state->mode, state->history_len, state->hist_w, state->scale_w,
                             &saved->w, workspace, workspace_bytes_, st)) != F8_OK)
        return s;
    return gemm_fwd(d, saved, Y, nullptr, st);
}

f8_status f8_linear_bwd_scaled(const f8_linear_desc* d, const f8_scaling_state* state, const void* dY,
                               f8_saved* saved, void* dX, void* dW, void* workspace,
                               size_t workspace_bytes_, void* stream)
{
    f8_status s = check_state(state, false);
    if (s != F8_OK) return s;
    if (state->mode == F8_DYNAMIC) return f8_linear_bwd(d, dY, saved, dX, dW, workspace, workspace_bytes_, stream);
    if ((s = check_bwd(d, true, dY, saved, dX, dW, workspace, workspace_bytes_)) != F8_OK) return s;
    hipStream_t st = (hipStream_t)stream;
    if ((s = quantise_scaled(dY, d->M, d->N, d->grad_format, state->mode, state->history_len, state->hist_dy,
                             state->scale_dy, &saved->dy, workspace, workspace_bytes_, st)) != F8_OK)
        return s;
    return gemms_bwd(d, saved, dX, nullptr, dW, st, workspace, workspace_bytes_);
}

f8_status f8_linear_fwd_chained(const f8_linear_desc* d, const void* X, const float* x_amax, const void* W,
                                void* Y, float* y_amax, f8_saved* saved, void* workspace,
                                size_t workspace_bytes_, void* stream)
{
    f8_status s = check_fwd(d, true, X, W, Y, saved, workspace, workspace_bytes_);
    if (s != F8_OK) return s;
    hipStream_t st = (hipStream_t)stream;
    const int64_t M = d->M, K = d->K, N = d->N;
    if (x_amax) {
        s = quantise_known_amax(X, M, K, K, F8_E4M3, x_amax, saved->x.amax, saved->x.scale, saved->x.inv_scale,
                                saved->x.q, K, saved->x.q_t, M, st);
        if (s != F8_OK) return s;
        s = quantise_both(W, N, K, false, F8_E4M3, &saved->w, workspace, st);
    } else {
        s = quantise_xw(d, X, W, saved, workspace, st);
    }
    if (s != F8_OK) return s;
    return gemm_fwd(d, saved, Y, y_amax, st);
}

f8_status f8_linear_bwd_chained(const f8_linear_desc* d, const void* dY, const float* dy_amax, f8_saved* saved,
                                void* dX, float* dx_amax, void* dW, void* workspace, size_t workspace_bytes_,
                                void* stream)
{
    f8_status s = check_bwd(d, true, dY, saved, dX, dW, workspace, workspace_bytes_);
    if (s != F8_OK) return s;
    hipStream_t st = (hipStream_t)stream;
    const int64_t M = d->M, N = d->N;
    const int gf = d->grad_format;
    if (dy_amax)
        s = quantise_known_amax(dY, M, N, N, gf, dy_amax, saved->dy.amax, saved->dy.scale, saved->dy.inv_scale,
                                saved->dy.q, N, saved->dy.q_t, M, st);
    else
        s = quantise_both(dY, M, N, false, gf, &saved->dy, workspace, st);
    if (s != F8_OK) return s;
    return gemms_bwd(d, saved, dX, dx_amax, dW, st, workspace, workspace_bytes_);
}

f8_status f8_silu_mul_quantise_delayed(const void* ab_bf16, int64_t M, int64_t H, f8_format fmt, float* history,
                                       int64_t history_len, float* scale, const f8_qtensor* q, void* workspace,
                                       size_t workspace_bytes_, void* stream)
{
    if ((int)fmt < 0 || (int)fmt > F8_E5M2) return F8_ERR_ENUM;
    if (!ab_bf16 || !history || !scale || !q) return F8_ERR_NULL;
    if (M < 0 || H < 0 || (M % 16) || (H % 16) || history_len < 1 || history_len > F8_MAX_HISTORY) return F8_ERR_SHAPE;
    if (!aligned16(ab_bf16)) return F8_ERR_ALIGN;
    f8_status s = check_q(q, false);
    if (s != F8_OK) return s;
    if (!workspace || workspace_bytes_ < quantise_workspace_bytes(M, H)) return F8_ERR_WORKSPACE;
    return quantise_scaled(ab_bf16, M, H, fmt, F8_DELAYED, history_len, history, scale, q, workspace, workspace_bytes_,
                           (hipStream_t)stream, 1);
}

f8_status f8_silu_mul_bwd_quantise_delayed(const void* ab_bf16, const void* dh_bf16, int64_t M, int64_t H,
                                           f8_format fmt, float* history, int64_t history_len, float* scale,
                                           const f8_qtensor* q, void* workspace, size_t workspace_bytes_,
                                           void* stream)
{
    if ((int)fmt < 0 || (int)fmt > F8_E5M2) return F8_ERR_ENUM;
    if (!ab_bf16 || !dh_bf16 || !history || !scale || !q) return F8_ERR_NULL;
    if (M < 0 || H < 0 || (M % 16) || (H % 16) || history_len < 1 || history_len > F8_MAX_HISTORY) return F8_ERR_SHAPE;
    if (!aligned16(ab_bf16) || !aligned16(dh_bf16)) return F8_ERR_ALIGN;
    f8_status s = check_q(q, false);
    if (s != F8_OK) return s;
    if (!workspace || workspace_bytes_ < quantise_workspace_bytes(M, 2 * H)) return F8_ERR_WORKSPACE;
    return quantise_scaled(ab_bf16, M, 2 * H, fmt, F8_DELAYED, history_len, history, scale, q, workspace,
                           workspace_bytes_, (hipStream_t)stream, 2, dh_bf16);
}

f8_status f8_linear_bwd_dyq(const f8_linear_desc* d, f8_saved* saved, void* dX, void* dW, void* stream)
{
    f8_status s = check_desc(d);
    if (s != F8_OK) return s;
    if (d->granularity != F8_TENSORWISE) return F8_ERR_ENUM;
    if (!dX || !dW || !saved) return F8_ERR_NULL;
    if (!aligned16(dX) || !aligned16(dW)) return F8_ERR_ALIGN;
    if ((s = check_q(&saved->x, false)) != F8_OK) return s;
    if ((s = check_q(&saved->w, false)) != F8_OK) return s;
    if ((s = check_q(&saved->dy, false)) != F8_OK) return s;
    return gemms_bwd(d, saved, dX, nullptr, dW, (hipStream_t)stream);
}

f8_status f8_linear_fwd_xq(const f8_linear_desc* d, const f8_scaling_state* state, const void* W, void* Y,
                           f8_saved* saved, void* workspace, size_t workspace_bytes_, void* stream)
{
    if (!state) return F8_ERR_NULL;
    if (state->mode != F8_DYNAMIC && state->mode != F8_DELAYED && state->mode != F8_STATIC) return F8_ERR_ENUM;
    if (state->mode != F8_DYNAMIC) {
        if (!state->scale_w) return F8_ERR_NULL;
        if (state->mode == F8_DELAYED && (!state->hist_w || state->history_len < 1 || state->history_len > F8_MAX_HISTORY))
            return state->hist_w ? F8_ERR_SHAPE : F8_ERR_NULL;
    }
    f8_status s = check_fwd(d, true, W, W, Y, saved, workspace, workspace_bytes_);  // X is not an argument here
    if (s != F8_OK) return s;
    hipStream_t st = (hipStream_t)stream;
    if (state->mode == F8_DYNAMIC)
        s = quantise_both(W, d->N, d->K, false, F8_E4M3, &saved->w, workspace, st);
    else
        s = quantise_scaled(W, d->N, d->K, F8_E4M3, state->mode, state->history_len, state->hist_w, state->scale_w,
                            &saved->w, workspace, workspace_bytes_, st);
    if (s != F8_OK) return s;
    return gemm_fwd(d, saved, Y, nullptr, st);
}

}  // extern "C"
