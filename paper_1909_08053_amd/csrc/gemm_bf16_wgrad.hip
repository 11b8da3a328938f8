// bf16 GEMM instantiations for the weight-gradient layout dW = X^T dY: A(m,k) = X[k,m] (m-contiguous) and
// B(k,n) = dY[k,n] (n-contiguous); k runs over tokens.
#include "gemm_bf16_v2.h"

namespace mlm {

hipError_t launch_gemm_bf16_wgrad(const GemmArgs& a, hipStream_t st) {
  if (a.epi != EPI_STORE) return hipErrorInvalidValue;
  if (gemm_use_v2(a)) return launch_gemm_bf16_v2<false, false, EPI_STORE>(a, a.splitk_ws, st);
  return launch_gemm_bf16_layout<false, false, EPI_STORE>(a, st);
}

}  // namespace mlm
