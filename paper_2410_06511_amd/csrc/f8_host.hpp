// Host-side helpers shared by the entry points.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/f8.h"

namespace f8 {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Launch errors are sticky in the HIP runtime until read; reading also clears them.
inline f8_status last_launch_status() { return hipGetLastError() == hipSuccess ? F8_OK : F8_ERR_LAUNCH; }

size_t workspace_bytes(int64_t max_rows, int64_t max_cols);

// amax -> scale -> cast of one validated tensor (dynamic scaling), any granularity.
f8_status quantise(const void* x, int64_t rows, int64_t cols, int64_t ld, int g, int fmt,
                   float* amax_out, float* scale_out, float* inv_out, uint8_t* out, int64_t ld_out,
                   uint8_t* out_t, int64_t ld_out_t, void* ws, hipStream_t st);

// Validated GEMM launch (see f8_gemm).
f8_status gemm(int layout, int64_t M, int64_t N, int64_t K, const uint8_t* A, int fa, int64_t lda,
               const uint8_t* B, int fb, int64_t ldb, const float* isa, const float* isb, int g,
               void* D, int64_t ldd, hipStream_t st);

}  // namespace f8
