// The f8_gemm entry point (steps 4-6 of the Float8 linear: Y = X W^T, dX = dY W, dW = dY^T X).
// The kernels live in f8_gemm_kernels.hpp and are instantiated per operand-format pair and layout
// by f8_gemm_inst.hip.
#include "f8_host.hpp"

namespace f8 {

// gemm_inst_<format of A>_<format of B>_<layout>: one object file each (f8_gemm_inst.hip)
typedef void (*gemm_fn)(int g, int M, int N, int K, const uint8_t* A, int64_t lda, const uint8_t* B, int64_t ldb,
                        const float* isa, const float* isb, uint16_t* D, int64_t ldd, uint32_t* amax_bits, void* ws,
                        size_t ws_bytes, hipStream_t st);
#define F8_DECLARE_GEMM(fa, fb, l)                                                                              \
    void gemm_inst_##fa##_##fb##_##l(int g, int M, int N, int K, const uint8_t* A, int64_t lda, const uint8_t* B, \
                                     int64_t ldb, const float* isa, const float* isb, uint16_t* D, int64_t ldd,  \
                                     uint32_t* amax_bits, void* ws, size_t ws_bytes, hipStream_t st);
#define F8_DECLARE_LAYOUTS(fa, fb) F8_DECLARE_GEMM(fa, fb, 0) F8_DECLARE_GEMM(fa, fb, 1) F8_DECLARE_GEMM(fa, fb, 2)
F8_DECLARE_LAYOUTS(0, 0)
F8_DECLARE_LAYOUTS(0, 1)
F8_DECLARE_LAYOUTS(1, 0)
F8_DECLARE_LAYOUTS(1, 1)
#undef F8_DECLARE_LAYOUTS
#undef F8_DECLARE_GEMM
static_assert(F8_E4M3 == 0 && F8_E5M2 == 1 && F8_NT == 0 && F8_NN == 1 && F8_TN == 2, "table order below");
#define F8_ROW(fa, fb) {gemm_inst_##fa##_##fb##_0, gemm_inst_##fa##_##fb##_1, gemm_inst_##fa##_##fb##_2}
static const gemm_fn kGemmTable[2][2][3] = {{F8_ROW(0, 0), F8_ROW(0, 1)}, {F8_ROW(1, 0), F8_ROW(1, 1)}};
#undef F8_ROW

__global__ void zero_word_kernel(uint32_t* p) { p[0] = 0; }

f8_status gemm(int layout, int64_t M, int64_t N, int64_t K, const uint8_t* A, int fa, int64_t lda,
               const uint8_t* B, int fb, int64_t ldb, const float* isa, const float* isb, int g, void* D,
               int64_t ldd, float* amax_d, hipStream_t st, void* ws, size_t ws_bytes)
{
    uint32_t* amax_bits = reinterpret_cast<uint32_t*>(amax_d);
    if (amax_bits) zero_word_kernel<<<1, 1, 0, st>>>(amax_bits);
    if (M == 0 || N == 0) return last_launch_status();
    uint16_t* d = static_cast<uint16_t*>(D);
    const int m = (int)M, n = (int)N, k = (int)K;
    kGemmTable[fa][fb][layout](g, m, n, k, A, lda, B, ldb, isa, isb, d, ldd, amax_bits, ws, ws_bytes, st);
    return last_launch_status();
}

}  // namespace f8

using namespace f8;

static f8_status gemm_checked(f8_layout layout, int64_t M, int64_t N, int64_t K, const uint8_t* A, f8_format fa,
                              int64_t lda, const uint8_t* B, f8_format fb, int64_t ldb, const float* inv_scale_a,
                              const float* inv_scale_b, f8_granularity g, void* D_bf16, int64_t ldd, float* amax_d,
                              void* workspace, size_t workspace_bytes_, void* stream)
{
    if ((int)layout < 0 || (int)layout > F8_TN || (int)fa < 0 || (int)fa > F8_E5M2 || (int)fb < 0 ||
        (int)fb > F8_E5M2 || ((int)g != F8_TENSORWISE && (int)g != F8_ROWWISE))
        return F8_ERR_ENUM;
    if (!A || !B || !D_bf16 || !inv_scale_a || !inv_scale_b) return F8_ERR_NULL;
    if (M < 0 || N < 0 || K < 0 || (M % 16) || (N % 16) || (K % 16) || (lda % 16) || (ldb % 16) || (ldd % 16))
        return F8_ERR_SHAPE;
    if (M >= (1 << 23) || N >= (1 << 23) || K >= (1 << 23) || lda >= (1 << 23) || ldb >= (1 << 23) || ldd >= (1 << 23))
        return F8_ERR_SHAPE;  // the kernels keep lane offsets inside a tile in 32 bits
    const int64_t a_cols = layout == F8_TN ? M : K, b_cols = layout == F8_NT ? K : N;
    if (lda < a_cols || ldb < b_cols || ldd < N) return F8_ERR_SHAPE;
    if (((M + 63) / 64) * ((N + 63) / 64) > (int64_t)0x7FFFFFFF) return F8_ERR_SHAPE;  // one block per 64x64 tile at most
    if (!aligned16(A) || !aligned16(B) || !aligned16(D_bf16)) return F8_ERR_ALIGN;
    if (g == F8_ROWWISE && !aligned16(inv_scale_b)) return F8_ERR_ALIGN;
    if (workspace && !aligned16(workspace)) return F8_ERR_ALIGN;
    // K == 0: the generic kernel's K loop does not run and it stores zeros
    return gemm(layout, M, N, K, A, fa, lda, B, fb, ldb, inv_scale_a, inv_scale_b, g, D_bf16, ldd, amax_d,
                (hipStream_t)stream, workspace, workspace ? workspace_bytes_ : 0);
}

extern "C" {

f8_status f8_gemm(f8_layout layout, int64_t M, int64_t N, int64_t K, const uint8_t* A, f8_format fa, int64_t lda,
                  const uint8_t* B, f8_format fb, int64_t ldb, const float* inv_scale_a, const float* inv_scale_b,
                  f8_granularity g, void* D_bf16, int64_t ldd, float* amax_d, void* stream)
{
    return gemm_checked(layout, M, N, K, A, fa, lda, B, fb, ldb, inv_scale_a, inv_scale_b, g, D_bf16, ldd, amax_d,
                        nullptr, 0, stream);
}

f8_status f8_gemm_ws(f8_layout layout, int64_t M, int64_t N, int64_t K, const uint8_t* A, f8_format fa, int64_t lda,
                     const uint8_t* B, f8_format fb, int64_t ldb, const float* inv_scale_a, const float* inv_scale_b,
                     f8_granularity g, void* D_bf16, int64_t ldd, float* amax_d, void* workspace,
                     size_t workspace_bytes_, void* stream)
{
    return gemm_checked(layout, M, N, K, A, fa, lda, B, fb, ldb, inv_scale_a, inv_scale_b, g, D_bf16, ldd, amax_d,
                        workspace, workspace_bytes_, stream);
}

}  // extern "C"
