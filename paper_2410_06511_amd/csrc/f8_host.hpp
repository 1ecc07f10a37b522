// Host-side helpers shared by the entry points.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/f8.h"

namespace f8 {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Launch errors are sticky in the HIP runtime until read; reading also clears them.
inline f8_status last_launch_status() { return hipGetLastError() == hipSuccess ? F8_OK : F8_ERR_LAUNCH; }

// Never less than kMinWorkspaceBytes: room for the per-block partial maxima of the kernels
// whose grid does not depend on the shape (tensorwise amax, feed-forward glue).
constexpr size_t kMinWorkspaceBytes = 8192;
size_t workspace_bytes(int64_t max_rows, int64_t max_cols);           // what f8_workspace_bytes returns
size_t quantise_workspace_bytes(int64_t max_rows, int64_t max_cols);  // the partial maxima alone

// amax -> scale -> cast of one validated tensor (dynamic scaling), any granularity.
f8_status quantise(const void* x, int64_t rows, int64_t cols, int64_t ld, int g, int fmt,
                   float* amax_out, float* scale_out, float* inv_out, uint8_t* out, int64_t ld_out,
                   uint8_t* out_t, int64_t ld_out_t, void* ws, hipStream_t st);

// Tensorwise dynamic quantisation of two validated contiguous tensors of one format (a forward's X
// and W; out_t nullable as in quantise): one amax launch and one cast launch for both when neither
// wants a transposed copy.  ws: kMinWorkspaceBytes at least.
f8_status quantise_pair(const void* x0, int64_t rows0, int64_t cols0, float* amax0, float* scale0, float* inv0,
                        uint8_t* out0, uint8_t* out_t0, const void* x1, int64_t rows1, int64_t cols1, float* amax1,
                        float* scale1, float* inv1, uint8_t* out1, uint8_t* out_t1, int fmt, void* ws, hipStream_t st);

// Delayed / static scaling pieces (tensorwise, validated arguments).
// cast with a given scale, leaving one partial maximum per 128x128 tile in ws
// glue = 1: x is [rows, 2 * cols] = [a | b] (ld = its row length), the tensor cast is bf16(silu(a) * b);
// glue = 2: x is [a | b] [rows, cols], x2 is dh [rows, cols / 2], the tensor cast is the glue's backward
f8_status cast_measure(const void* x, int64_t rows, int64_t cols, int64_t ld, const float* scale, int fmt,
                       uint8_t* out, int64_t ld_out, uint8_t* out_t, int64_t ld_out_t, void* ws,
                       size_t ws_bytes, int* npartial, hipStream_t st, int glue = 0, const void* x2 = nullptr);
// step amax (from partials, or amax_in) -> amax_out; used_scale -> saved_scale, 1/x -> saved_inv;
// history shifted and extended; FMAX / max(history) -> next_scale (, 1/x -> next_inv)
f8_status history_push(const void* partial, int npartial, const float* amax_in, float* history, int64_t len,
                       int fmt, float* amax_out, const float* used_scale, float* saved_scale,
                       float* saved_inv, float* next_scale, float* next_inv, hipStream_t st);
f8_status publish_scale(const float* s_in, float* s_out, float* inv_out, hipStream_t st);
f8_status cast_given(const void* x, int64_t rows, int64_t cols, int64_t ld, const float* scale, int fmt,
                     uint8_t* out, int64_t ld_out, uint8_t* out_t, int64_t ld_out_t, hipStream_t st);

// Rowwise scaling, both orientations: the two amax passes, then one cast that reads x once.
f8_status amax_scales(const void* x, int64_t rows, int64_t cols, int64_t ld, int g, int fmt, float* amax_out,
                      float* scale_out, float* inv_out, void* ws, hipStream_t st);
f8_status amax_rows_and_cols(const void* x, int64_t rows, int64_t cols, int64_t ld, int fmt, float* amax_r,
                             float* scale_r, float* inv_r, float* amax_c, float* scale_c, float* inv_c, void* ws,
                             hipStream_t st);
f8_status cast_rows_and_cols(const void* x, int64_t rows, int64_t cols, int64_t ld, int fmt,
                             const float* scale_rows, const float* scale_cols, uint8_t* out, int64_t ld_out,
                             uint8_t* out_t, int64_t ld_out_t, hipStream_t st);

// Dynamic scaling of a tensorwise tensor whose amax the producer already took: one cast pass.
f8_status quantise_known_amax(const void* x, int64_t rows, int64_t cols, int64_t ld, int fmt, const float* amax_in,
                              float* amax_out, float* scale_out, float* inv_out, uint8_t* out, int64_t ld_out,
                              uint8_t* out_t, int64_t ld_out_t, hipStream_t st);

// Validated GEMM launch (see f8_gemm); amax_d may be null.  ws (nullable): device scratch of
// ws_bytes for the fp32 partial results of a product that is better split along its
// contraction (few output tiles, long contraction); without it such a product runs unsplit.
f8_status gemm(int layout, int64_t M, int64_t N, int64_t K, const uint8_t* A, int fa, int64_t lda,
               const uint8_t* B, int fb, int64_t ldb, const float* isa, const float* isb, int g,
               void* D, int64_t ldd, float* amax_d, hipStream_t st, void* ws = nullptr, size_t ws_bytes = 0);
// Largest scratch a split product can use (ranges x output elements x 4 bytes, with ranges x tiles
// at most one per compute unit): part of what workspace_bytes returns.
constexpr size_t kSplitKMaxBytes = (size_t)256 * 256 * 256 * sizeof(float);

}  // namespace f8
