// bf16 GEMM instantiations for the input-gradient layout dX = dY W^T: A [M,K] k-contiguous (dY), B(k,n) = W[n,k]
// with W stored [in,out] = [N,K], i.e. k-contiguous as well.  Epilogues: plain store, GeLU' (fused dG = dY o GeLU'(G)).
#include "gemm_bf16_v2.h"

namespace mlm {

hipError_t launch_gemm_bf16_dgrad(const GemmArgs& a, hipStream_t st) {
  if (gemm_use_v2(a)) {
    switch (a.epi) {
      case EPI_STORE: return launch_gemm_bf16_v2<true, true, EPI_STORE>(a, a.splitk_ws, st);
      case EPI_DGELU: return launch_gemm_bf16_v2<true, true, EPI_DGELU>(a, a.splitk_ws, st);
      default: return hipErrorInvalidValue;
    }
  }
  switch (a.epi) {
    case EPI_STORE: return launch_gemm_bf16_layout<true, true, EPI_STORE>(a, st);
    case EPI_DGELU: return launch_gemm_bf16_layout<true, true, EPI_DGELU>(a, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace mlm
