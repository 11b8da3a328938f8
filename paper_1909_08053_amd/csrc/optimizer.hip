// One model-parallel worker's optimizer step (Section 4.2 of the paper: Adam with decoupled weight decay, global
// gradient-norm clipping, fp32 master weights behind the low-precision weights the GEMMs read; Section 3: every
// worker updates its own parameters, only the squared gradient norm crosses workers).  Bandwidth-bound: 28 bytes
// per bf16 parameter (gradient 2, master / m / v read and written 24, weight 2).
#include "common.h"
#include <string.h>

namespace mlm {

constexpr int kSqnormBlocksMax = 1024;   // partial sums per tensor (one float each in the workspace)
constexpr int kMaxOptTensors = 64;

// out = sum of all partials (fixed order) + *extra (the other workers' squared norm, if given)
__global__ __launch_bounds__(256) void sqnorm_final_kernel(const float* __restrict__ partials, int total,
                                                           const float* extra, float* out) {
  __shared__ float red[4];
  float acc = 0.f;
  for (int i = threadIdx.x; i < total; i += 256) acc += partials[i];
  acc = wave_sum(acc);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) out[0] = (red[0] + red[1]) + (red[2] + red[3]) + (extra ? extra[0] : 0.f);
}

struct AdamArgs {
  float max_norm, lr, beta1, beta2, eps, wd, inv_bc1, inv_bc2;
};

// g <- g * clip;  m, v moments;  w <- w - lr (mh / (sqrt(vh) + eps) + wd w)  on the fp32 master copy;
// weight_out (storage type) = rounded master.
template <typename T>
__device__ __forceinline__ void adamw_vec(size_t i, const T* __restrict__ g, float* __restrict__ master,
                                          float* __restrict__ m, float* __restrict__ v, T* weight_out,
                                          const float* __restrict__ total_sqnorm, const AdamArgs& a) {
  constexpr int VN = Vec16<T>::N;
  float clip = 1.0f;
  if (a.max_norm > 0.f) clip = fminf(1.0f, a.max_norm / (sqrtf(total_sqnorm[0]) + 1e-6f));
  Vec16<T> gv;
  gv.load(g + i * VN);
  Vec16<T> wo;
#pragma unroll
  for (int q = 0; q < VN / 4; ++q) {
    const size_t o = i * VN + q * 4;
    float4 w4 = *reinterpret_cast<const float4*>(master + o);
    float4 m4 = *reinterpret_cast<const float4*>(m + o);
    float4 v4 = *reinterpret_cast<const float4*>(v + o);
    float* pw = reinterpret_cast<float*>(&w4);
    float* pm = reinterpret_cast<float*>(&m4);
    float* pv = reinterpret_cast<float*>(&v4);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const float gg = gv.get(q * 4 + k) * clip;
      pm[k] = a.beta1 * pm[k] + (1.0f - a.beta1) * gg;
      pv[k] = a.beta2 * pv[k] + (1.0f - a.beta2) * gg * gg;
      const float mh = pm[k] * a.inv_bc1, vh = pv[k] * a.inv_bc2;
      pw[k] = pw[k] - a.lr * (mh / (sqrtf(vh) + a.eps) + a.wd * pw[k]);
      wo.set(q * 4 + k, pw[k]);
    }
    *reinterpret_cast<float4*>(master + o) = w4;
    *reinterpret_cast<float4*>(m + o) = m4;
    *reinterpret_cast<float4*>(v + o) = v4;
  }
  if (weight_out) wo.store(weight_out + i * VN);
}

template <typename T>
__global__ __launch_bounds__(256) void adamw_kernel(size_t nvec, const T* __restrict__ g, float* __restrict__ master,
                                                    float* __restrict__ m, float* __restrict__ v, T* weight_out,
                                                    const float* __restrict__ total_sqnorm, AdamArgs a) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= nvec) return;
  adamw_vec<T>(i, g, master, m, v, weight_out, total_sqnorm, a);
}

// Up to kGroup tensors per launch: block b belongs to the tensor t with blk_start[t] <= b < blk_start[t + 1].
constexpr int kGroup = 32;
struct MultiDesc {
  int n;
  int blk_start[kGroup + 1];
  size_t nvec[kGroup];
  const void* g[kGroup];
  float* master[kGroup];
  float* m[kGroup];
  float* v[kGroup];
  void* w[kGroup];
  float wd[kGroup];
};

__device__ __forceinline__ int find_tensor(const MultiDesc& d, int b) {
  int t = 0;
  while (t + 1 < d.n && b >= d.blk_start[t + 1]) ++t;
  return t;
}

template <typename T>
__global__ __launch_bounds__(256) void sqnorm_multi_kernel(MultiDesc d, float* __restrict__ partials) {
  constexpr int VN = Vec16<T>::N;
  __shared__ float red[4];
  const int t = find_tensor(d, blockIdx.x);
  const int lb = blockIdx.x - d.blk_start[t], nb = d.blk_start[t + 1] - d.blk_start[t];
  const T* g = (const T*)d.g[t];
  float acc = 0.f;
  for (size_t i = (size_t)lb * 256 + threadIdx.x; i < d.nvec[t]; i += (size_t)nb * 256) {
    Vec16<T> v;
    v.load(g + i * VN);
#pragma unroll
    for (int e = 0; e < VN; ++e) acc = fmaf(v.get(e), v.get(e), acc);
  }
  acc = wave_sum(acc);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) partials[blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
}

template <typename T>
__global__ __launch_bounds__(256) void adamw_multi_kernel(MultiDesc d, const float* __restrict__ total_sqnorm,
                                                          AdamArgs a) {
  const int t = find_tensor(d, blockIdx.x);
  const size_t i = (size_t)(blockIdx.x - d.blk_start[t]) * 256 + threadIdx.x;
  if (i >= d.nvec[t]) return;
  a.wd = d.wd[t];
  adamw_vec<T>(i, (const T*)d.g[t], d.master[t], d.m[t], d.v[t], (T*)d.w[t], total_sqnorm, a);
}

static inline bool al16(const void* p) { return ((uintptr_t)p & 15) == 0; }

}  // namespace mlm

using namespace mlm;

extern "C" {

MLM_API int mlm_grad_sqnorm(int32_t dtype, const void* const* grads, const int64_t* counts, int32_t n_tensors,
                            const float* other_sqnorm, float* sqnorm_out, void* ws, size_t ws_bytes, void* stream) {
  if (dtype != MLM_F32 && dtype != MLM_BF16) return MLM_E_DTYPE;
  if (!grads || !counts || !sqnorm_out || !ws) return MLM_E_NULL;
  if (n_tensors < 1 || n_tensors > kMaxOptTensors) return MLM_E_SHAPE;
  if (ws_bytes < (size_t)n_tensors * kSqnormBlocksMax * sizeof(float)) return MLM_E_WORKSPACE;
  const int vn = dtype == MLM_BF16 ? 8 : 4;
  for (int t = 0; t < n_tensors; ++t) {
    if (!grads[t]) return MLM_E_NULL;
    if (counts[t] <= 0) return MLM_E_SHAPE;
    if (counts[t] % vn || !al16(grads[t])) return MLM_E_ALIGN;
  }
  if (!al16(ws)) return MLM_E_ALIGN;
  hipStream_t st = (hipStream_t)stream;
  float* partials = (float*)ws;
  int total = 0;
  for (int t0 = 0; t0 < n_tensors; t0 += kGroup) {
    MultiDesc d;
    memset(&d, 0, sizeof(d));
    d.n = n_tensors - t0 < kGroup ? n_tensors - t0 : kGroup;
    int blocks = 0;
    for (int t = 0; t < d.n; ++t) {
      const size_t nvec = (size_t)counts[t0 + t] / vn;
      const size_t want = (nvec + 1023) / 1024;
      d.blk_start[t] = blocks;
      d.nvec[t] = nvec;
      d.g[t] = grads[t0 + t];
      blocks += (int)(want < (size_t)kSqnormBlocksMax ? want : kSqnormBlocksMax);
    }
    d.blk_start[d.n] = blocks;
    if (dtype == MLM_BF16)
      hipLaunchKernelGGL((sqnorm_multi_kernel<bf16>), dim3(blocks), dim3(256), 0, st, d, partials + total);
    else
      hipLaunchKernelGGL((sqnorm_multi_kernel<float>), dim3(blocks), dim3(256), 0, st, d, partials + total);
    if (hipGetLastError() != hipSuccess) return MLM_E_HIP;
    total += blocks;
  }
  hipLaunchKernelGGL(sqnorm_final_kernel, dim3(1), dim3(256), 0, st, partials, total, other_sqnorm, sqnorm_out);
  return hipGetLastError() == hipSuccess ? MLM_OK : MLM_E_HIP;
}

MLM_API int mlm_adamw_step(int32_t dtype, int64_t count, const void* grad, float* master, float* m, float* v,
                           void* weight_out, const float* total_sqnorm, float max_norm, float lr, float beta1,
                           float beta2, float eps, float weight_decay, int32_t step, void* stream) {
  if (dtype != MLM_F32 && dtype != MLM_BF16) return MLM_E_DTYPE;
  if (!grad || !master || !m || !v) return MLM_E_NULL;
  if (max_norm > 0.f && !total_sqnorm) return MLM_E_NULL;
  const int vn = dtype == MLM_BF16 ? 8 : 4;
  if (count <= 0 || step < 1 || !(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f)) return MLM_E_SHAPE;
  if (count % vn || !al16(grad) || !al16(master) || !al16(m) || !al16(v) || (weight_out && !al16(weight_out)))
    return MLM_E_ALIGN;
  AdamArgs a;
  a.max_norm = max_norm; a.lr = lr; a.beta1 = beta1; a.beta2 = beta2; a.eps = eps; a.wd = weight_decay;
  // bias corrections in double on the host: 1 - beta^t loses digits in fp32 for t small and beta close to 1
  a.inv_bc1 = (float)(1.0 / (1.0 - pow((double)beta1, (double)step)));
  a.inv_bc2 = (float)(1.0 / (1.0 - pow((double)beta2, (double)step)));
  const size_t nvec = (size_t)count / vn;
  const unsigned nblk = (unsigned)((nvec + 255) / 256);
  hipStream_t st = (hipStream_t)stream;
  if (dtype == MLM_BF16)
    hipLaunchKernelGGL((adamw_kernel<bf16>), dim3(nblk), dim3(256), 0, st, nvec, (const bf16*)grad, master, m, v,
                       (bf16*)weight_out, total_sqnorm, a);
  else
    hipLaunchKernelGGL((adamw_kernel<float>), dim3(nblk), dim3(256), 0, st, nvec, (const float*)grad, master, m, v,
                       (float*)weight_out, total_sqnorm, a);
  return hipGetLastError() == hipSuccess ? MLM_OK : MLM_E_HIP;
}

MLM_API int mlm_adamw_step_multi(int32_t dtype, int32_t n_tensors, const int64_t* counts, const void* const* grads,
                                 float* const* masters, float* const* ms, float* const* vs, void* const* weights_out,
                                 const float* weight_decays, const float* total_sqnorm, float max_norm, float lr,
                                 float beta1, float beta2, float eps, int32_t step, void* stream) {
  if (dtype != MLM_F32 && dtype != MLM_BF16) return MLM_E_DTYPE;
  if (!counts || !grads || !masters || !ms || !vs || !weights_out || !weight_decays) return MLM_E_NULL;
  if (max_norm > 0.f && !total_sqnorm) return MLM_E_NULL;
  if (n_tensors < 1 || n_tensors > kMaxOptTensors || step < 1 || !(beta1 >= 0.f && beta1 < 1.f) ||
      !(beta2 >= 0.f && beta2 < 1.f))
    return MLM_E_SHAPE;
  const int vn = dtype == MLM_BF16 ? 8 : 4;
  for (int t = 0; t < n_tensors; ++t) {
    if (!grads[t] || !masters[t] || !ms[t] || !vs[t]) return MLM_E_NULL;
    if (counts[t] <= 0) return MLM_E_SHAPE;
    if (counts[t] % vn || !al16(grads[t]) || !al16(masters[t]) || !al16(ms[t]) || !al16(vs[t]) ||
        (weights_out[t] && !al16(weights_out[t])))
      return MLM_E_ALIGN;
  }
  AdamArgs a;
  a.max_norm = max_norm; a.lr = lr; a.beta1 = beta1; a.beta2 = beta2; a.eps = eps; a.wd = 0.f;
  a.inv_bc1 = (float)(1.0 / (1.0 - pow((double)beta1, (double)step)));
  a.inv_bc2 = (float)(1.0 / (1.0 - pow((double)beta2, (double)step)));
  hipStream_t st = (hipStream_t)stream;
  for (int t0 = 0; t0 < n_tensors; t0 += kGroup) {
    MultiDesc d;
    memset(&d, 0, sizeof(d));
    d.n = n_tensors - t0 < kGroup ? n_tensors - t0 : kGroup;
    long blocks = 0;
    for (int t = 0; t < d.n; ++t) {
      const size_t nvec = (size_t)counts[t0 + t] / vn;
      d.blk_start[t] = (int)blocks;
      d.nvec[t] = nvec;
      d.g[t] = grads[t0 + t]; d.master[t] = masters[t0 + t]; d.m[t] = ms[t0 + t]; d.v[t] = vs[t0 + t];
      d.w[t] = weights_out[t0 + t]; d.wd[t] = weight_decays[t0 + t];
      blocks += (long)((nvec + 255) / 256);
    }
    if (blocks > 0x7fffffffL) return MLM_E_SHAPE;
    d.blk_start[d.n] = (int)blocks;
    if (dtype == MLM_BF16)
      hipLaunchKernelGGL((adamw_multi_kernel<bf16>), dim3((unsigned)blocks), dim3(256), 0, st, d, total_sqnorm, a);
    else
      hipLaunchKernelGGL((adamw_multi_kernel<float>), dim3((unsigned)blocks), dim3(256), 0, st, d, total_sqnorm, a);
    if (hipGetLastError() != hipSuccess) return MLM_E_HIP;
  }
  return MLM_OK;
}

}  // extern "C"
