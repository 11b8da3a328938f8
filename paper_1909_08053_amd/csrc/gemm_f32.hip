// fp32 GEMM for dtype MLM_F32: LDS-tiled, plain FMA, fp32 throughout.  This path exists for the
// 1e-4 parity configuration (small shapes); the throughput path is gemm_bf16.hip.
// Computes C[m,n] = sum_k A(m,k) B(k,n) with either operand stored k-contiguous or not, and the
// same fused epilogues as the bf16 kernel (bias, bias+GeLU with saved pre-activation, GeLU', dlogits).
#include "common.h"

namespace mlm {

constexpr int FT = 64;   // tile edge
constexpr int FK = 16;   // k step

template <int EPI>
__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmArgs a) {
  __shared__ float sA[FK][FT + 4];
  __shared__ float sB[FK][FT + 4];
  const float* A = (const float*)a.A;
  const float* B = (const float*)a.B;
  const int tid = threadIdx.x;
  const int tx = tid & 15, ty = tid >> 4;
  const int m0 = blockIdx.y * FT, n0 = blockIdx.x * FT;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

  for (int k0 = 0; k0 < a.K; k0 += FK) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = tid + i * 256;
      int m, k;
      if (a.a_kc) { k = e & 15; m = e >> 4; } else { m = e & 63; k = e >> 6; }
      float v = 0.f;
      if (m0 + m < a.M && k0 + k < a.K)
        v = a.a_kc ? A[(size_t)(m0 + m) * a.lda + k0 + k] : A[(size_t)(k0 + k) * a.lda + m0 + m];
      sA[k][m] = v;
      int n;
      if (a.b_kc) { k = e & 15; n = e >> 4; } else { n = e & 63; k = e >> 6; }
      v = 0.f;
      if (n0 + n < a.N && k0 + k < a.K)
        v = a.b_kc ? B[(size_t)(n0 + n) * a.ldb + k0 + k] : B[(size_t)(k0 + k) * a.ldb + n0 + n];
      sB[k][n] = v;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < FK; ++k) {
      float av[4], bv[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { av[i] = sA[k][ty * 4 + i]; bv[i] = sB[k][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
    }
    __syncthreads();
  }

  float* C = (float*)a.C;
  const float* bias = (const float*)a.bias;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m >= a.M) continue;
    float coef = 0.f, Mr = 0.f, invS = 0.f;
    int loc = -1;
    if (EPI == EPI_DLOGITS) {
      coef = (a.loss_w ? a.loss_w[m] : 1.0f) / a.loss_stats[1];
      Mr = a.Mrow[m];
      invS = coef / a.Srow[m];
      loc = a.targets[m] - a.v0;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n >= a.N) continue;
      float v = acc[i][j];
      if (EPI == EPI_STORE) {
        if (bias) v += bias[n];
        C[(size_t)m * a.ldc + n] = v;
      } else if (EPI == EPI_BIAS_GELU) {
        if (bias) v += bias[n];
        ((float*)a.aux)[(size_t)m * a.ldaux + n] = v;
        C[(size_t)m * a.ldc + n] = gelu_fwd(v, a.gelu_tanh != 0);
      } else if (EPI == EPI_DGELU) {
        const float g = ((const float*)a.aux)[(size_t)m * a.ldaux + n];
        C[(size_t)m * a.ldc + n] = v * gelu_bwd(g, a.gelu_tanh != 0);
      } else if (EPI == EPI_DLOGITS) {
        float g = expf(v - Mr) * invS;
        if (n == loc) g -= coef;
        C[(size_t)m * a.ldc + n] = g;
      }
    }
  }
}

hipError_t launch_gemm_f32(const GemmArgs& a, hipStream_t st) {
  dim3 grid((a.N + FT - 1) / FT, (a.M + FT - 1) / FT), block(256);
  switch (a.epi) {
    case EPI_STORE: hipLaunchKernelGGL((gemm_f32_kernel<EPI_STORE>), grid, block, 0, st, a); break;
    case EPI_BIAS_GELU: hipLaunchKernelGGL((gemm_f32_kernel<EPI_BIAS_GELU>), grid, block, 0, st, a); break;
    case EPI_DGELU: hipLaunchKernelGGL((gemm_f32_kernel<EPI_DGELU>), grid, block, 0, st, a); break;
    case EPI_DLOGITS: hipLaunchKernelGGL((gemm_f32_kernel<EPI_DLOGITS>), grid, block, 0, st, a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace mlm
