// The fp8 GEMM kernels instantiated for ONE operand-format pair and ONE layout, so that the
// twelve combinations compile in parallel.  The build compiles this file once per combination
// with -DF8_INST_FA=<0|1> -DF8_INST_FB=<0|1> -DF8_INST_LAYOUT=<0|1|2> (f8_format of the A and B
// codes, f8_layout); each object defines f8::gemm_inst_<FA>_<FB>_<LAYOUT>.
#if !defined(F8_INST_FA) || !defined(F8_INST_FB) || !defined(F8_INST_LAYOUT)
#error "compile with -DF8_INST_FA=, -DF8_INST_FB=, -DF8_INST_LAYOUT= (see build.py)"
#endif
#include "f8_gemm_kernels.hpp"

#define F8_INST_NAME_(fa, fb, l) gemm_inst_##fa##_##fb##_##l
#define F8_INST_NAME(fa, fb, l) F8_INST_NAME_(fa, fb, l)

namespace f8 {

void F8_INST_NAME(F8_INST_FA, F8_INST_FB, F8_INST_LAYOUT)(int g, int M, int N, int K, const uint8_t* A, int64_t lda,
                                                           const uint8_t* B, int64_t ldb, const float* isa,
                                                           const float* isb, uint16_t* D, int64_t ldd,
                                                           uint32_t* amax_bits, void* ws, size_t ws_bytes, hipStream_t st)
{
    gemm_formats<F8_INST_LAYOUT, F8_INST_FA, F8_INST_FB>(g, M, N, K, A, lda, B, ldb, isa, isb, D, ldd, amax_bits, ws,
                                                         ws_bytes, st);
}

}  // namespace f8
