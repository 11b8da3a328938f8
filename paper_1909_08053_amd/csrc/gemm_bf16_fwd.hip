// bf16 GEMM instantiations for the forward layout: A [M,K] k-contiguous (activations), B [K,N] n-contiguous
// (weights stored [in,out] as in Y = XA).  Epilogues: plain/bias store, bias+GeLU, cross-entropy partials, dlogits.
#include "gemm_bf16_v2.h"

namespace mlm {

hipError_t launch_gemm_bf16_fwd(const GemmArgs& a, hipStream_t st) {
  if (gemm_use_v2(a)) {
    switch (a.epi) {
      case EPI_STORE: return launch_gemm_bf16_v2<true, false, EPI_STORE>(a, a.splitk_ws, st);
      case EPI_BIAS_GELU: return launch_gemm_bf16_v2<true, false, EPI_BIAS_GELU>(a, a.splitk_ws, st);
      case EPI_CE: return launch_gemm_bf16_v2<true, false, EPI_CE>(a, a.splitk_ws, st);
      case EPI_DLOGITS: return launch_gemm_bf16_v2<true, false, EPI_DLOGITS>(a, a.splitk_ws, st);
      default: return hipErrorInvalidValue;
    }
  }
  switch (a.epi) {
    case EPI_STORE: return launch_gemm_bf16_layout<true, false, EPI_STORE>(a, st);
    case EPI_BIAS_GELU: return launch_gemm_bf16_layout<true, false, EPI_BIAS_GELU>(a, st);
    case EPI_CE: return launch_gemm_bf16_layout<true, false, EPI_CE>(a, st);
    case EPI_DLOGITS: return launch_gemm_bf16_layout<true, false, EPI_DLOGITS>(a, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace mlm
