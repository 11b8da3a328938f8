// bf16 GEMM instantiations for the weight-gradient layout dW = X^T dY: A(m,k) = X[k,m] (m-contiguous) and
// B(k,n) = dY[k,n] (n-contiguous); k runs over tokens.
#include <stdlib.h>
#include "gemm_bf16_v2.h"

namespace mlm {

hipError_t launch_gemm_bf16_wgrad(const GemmArgs& a, hipStream_t st) {
  if (a.epi != EPI_STORE) return hipErrorInvalidValue;
  if (gemm_use_v2(a)) return launch_gemm_bf16_v2<false, false, EPI_STORE>(a, a.splitk_ws, st);
  return launch_gemm_bf16_layout<false, false, EPI_STORE>(a, st);
}

// Estimated time (microseconds, the cost model of v2_plan) of one weight-gradient GEMM launched on its own with the
// tail split, and of a set of them launched as one group without a split.
static double wgrad_cost_alone(const GemmArgs& a) {
  const V2Plan p = v2_plan(a.M, a.N, a.K, true);
  const int V2_CUS = gemm_cu_count();
  const int nk = 2 * ((a.K / V2_BK + 1) / 2);
  const int rounds_full = (p.full_tiles + V2_CUS - 1) / V2_CUS;
  const double fixed = v2_tile_fixed(V2_B), per_slice = v2_slice_cost(V2_B, true);
  double t = rounds_full * (fixed + per_slice * nk);
  if (p.tail_tiles) {
    const double traffic = (double)p.tail_tiles * p.split * (V2_B * V2_B * 4.0) / 5.0e6;
    t += fixed + per_slice * ((nk + p.split - 1) / p.split) + traffic + v2_fixup_cost(traffic);
  }
  return t + 2.0;     // launch + drain of the GEMM kernel itself
}

// The weight gradients of a layer shard (same operand layout, same k = tokens).  One grouped launch when the cost
// model says the shared last round beats the separate launches with their k-splits; separate launches otherwise.
hipError_t launch_gemm_bf16_wgrad_group(const GemmArgs* probs, int n, float* splitk_ws, hipStream_t st) {
  bool groupable = n >= 2 && n <= kMaxGroup;
  double alone = 0.0;
  int tiles = 0;
  for (int q = 0; q < n && groupable; ++q) {
    groupable = probs[q].epi == EPI_STORE && probs[q].bias == nullptr && gemm_use_v2(probs[q]) &&
                probs[q].K == probs[0].K;
    alone += wgrad_cost_alone(probs[q]);
    tiles += v2_tiles(probs[q]);
  }
  if (groupable) {
    const int nk = 2 * ((probs[0].K / V2_BK + 1) / 2);
    const int V2_CUS = gemm_cu_count();
    const double grouped = ((tiles + V2_CUS - 1) / V2_CUS) * (v2_tile_fixed(V2_B) + v2_slice_cost(V2_B, true) * nk) + 2.0;
    static const bool off = [] { const char* e = getenv("MLM_GEMM_GROUP"); return e && atoi(e) == 0; }();
    if (!off && grouped < alone)
      return gemm_v2_waves(false, false) == 4 ? launch_gemm_bf16_v2_group_nw<false, false, 4>(probs, n, st)
                                              : launch_gemm_bf16_v2_group_nw<false, false, 8>(probs, n, st);
  }
  for (int q = 0; q < n; ++q) {
    GemmArgs a = probs[q];
    a.splitk_ws = splitk_ws;
    hipError_t e = launch_gemm_bf16_wgrad(a, st);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace mlm
