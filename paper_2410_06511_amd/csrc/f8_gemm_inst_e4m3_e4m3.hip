// fp8 GEMM kernels instantiated for A codes in E4M3 and B codes in E4M3.
#include "f8_gemm_kernels.hpp"

namespace f8 {

void gemm_e4m3_e4m3(int layout, int g, int M, int N, int K, const uint8_t* A, int64_t lda, const uint8_t* B, int64_t ldb,
               const float* isa, const float* isb, uint16_t* D, int64_t ldd, uint32_t* amax_bits, hipStream_t st)
{
    gemm_formats<F8_E4M3, F8_E4M3>(layout, g, M, N, K, A, lda, B, ldb, isa, isb, D, ldd, amax_bits, st);
}

}  // namespace f8
