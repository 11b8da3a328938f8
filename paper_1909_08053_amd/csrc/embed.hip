// Vocabulary-parallel input embedding of one shard (Section 3 of the paper: the embedding table is the output
// embedding's matrix E [H, v], split along the vocabulary; each shard contributes the rows of the ids it owns and
// zeros elsewhere, and the reduction g sums the partials).  E_r is stored [H, V_l] -- the layout the logits GEMM
// wants -- so a token's embedding is a COLUMN of E_r: H elements at stride V_l.  Both directions therefore walk the
// tokens in the order of their local id: consecutive waves touch neighbouring columns, which share cache lines, and
// the backward pass gets the tokens of one id as one contiguous, token-ordered segment (a deterministic sum with no
// atomics).  The order is a stable rank-sort computed by brute force (integer work, exact).
#include "common.h"
#include "rng.h"

namespace mlm {

// key[t] = local id if the token's id is in [v0, v0 + Vl), else Vl (sorts last); perm[rank(t)] = t with
// rank(t) = #{t' : key[t'] < key[t]} + #{t' < t : key[t'] == key[t]}.
__global__ __launch_bounds__(256) void embed_rank_kernel(int T, const int32_t* __restrict__ ids, int v0, int Vl,
                                                         int32_t* __restrict__ perm) {
  __shared__ int32_t sk[1024];
  const int t = blockIdx.x * 256 + threadIdx.x;
  auto key_of = [&](int i) {
    const int loc = ids[i] - v0;
    return (loc >= 0 && loc < Vl) ? loc : Vl;
  };
  const int my = t < T ? key_of(t) : 0;
  int rank = 0;
  for (int c0 = 0; c0 < T; c0 += 1024) {
    __syncthreads();
    for (int i = threadIdx.x; i < 1024; i += 256) sk[i] = c0 + i < T ? key_of(c0 + i) : 0x7FFFFFFF;
    __syncthreads();
    const int n = min(1024, T - c0);
    for (int i = 0; i < n; ++i) {
      const int k = sk[i];
      rank += (k < my || (k == my && c0 + i < t)) ? 1 : 0;
    }
  }
  if (t < T) perm[rank] = t;
}

// One wave per sorted position: the token's row of the partial = column (id - v0) of E_r, or zeros.
template <typename T>
__global__ __launch_bounds__(256) void embed_fwd_kernel(int Tn, int H, int Vl, int v0, const int32_t* __restrict__ ids,
                                                        const int32_t* __restrict__ perm, const T* __restrict__ E,
                                                        T* __restrict__ out) {
  constexpr int VN = Vec16<T>::N;
  const int lane = threadIdx.x & 63;
  const int k = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (k >= Tn) return;
  const int t = perm[k];
  const int loc = ids[t] - v0;
  const bool inside = loc >= 0 && loc < Vl;           // wave-uniform
  T* row = out + (size_t)t * H;
  for (int v = lane; v < H / VN; v += 64) {
    Vec16<T> o;
#pragma unroll
    for (int e = 0; e < VN; ++e) o.set(e, inside ? to_f32(E[(size_t)(v * VN + e) * Vl + loc]) : 0.f);
    o.store(row + (size_t)v * VN);
  }
}

// One wave per sorted position; the wave at the head of a run of equal local ids sums the run's rows of dz0 in token
// order (fp32) and adds the sum to column `loc` of dE_r.  Two-byte (or four-byte) accesses: neighbouring columns
// belong to other waves.
template <typename T, int NV>
__global__ __launch_bounds__(256) void embed_bwd_kernel(int Tn, int H, int Vl, int v0, const int32_t* __restrict__ ids,
                                                        const int32_t* __restrict__ perm, const T* __restrict__ dz,
                                                        T* __restrict__ dE) {
  constexpr int VN = Vec16<T>::N;
  const int lane = threadIdx.x & 63;
  const int k = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (k >= Tn) return;
  const int loc = ids[perm[k]] - v0;
  if (loc < 0 || loc >= Vl) return;                   // outside the shard (wave-uniform)
  if (k > 0 && ids[perm[k - 1]] - v0 == loc) return;  // not the head of its run
  float acc[NV][VN];
#pragma unroll
  for (int i = 0; i < NV; ++i)
#pragma unroll
    for (int e = 0; e < VN; ++e) acc[i][e] = 0.f;
  const int nvec = H / VN;
  for (int kk = k; kk < Tn; ++kk) {
    const int t = perm[kk];
    if (ids[t] - v0 != loc) break;                    // end of the run (wave-uniform)
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int v = lane + 64 * i;
      if (v < nvec) {
        Vec16<T> x;
        x.load(dz + (size_t)t * H + (size_t)v * VN);
#pragma unroll
        for (int e = 0; e < VN; ++e) acc[i][e] += x.get(e);
      }
    }
  }
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int v = lane + 64 * i;
    if (v < nvec) {
#pragma unroll
      for (int e = 0; e < VN; ++e) {
        T* p = dE + (size_t)(v * VN + e) * Vl + loc;
        *p = from_f32<T>(to_f32(*p) + acc[i][e]);
      }
    }
  }
}

// dz0 = dropout-mask(dx0) / (1 - p); dpos[i, :] = sum over the batch of dz0[batch s + i, :].  One thread per
// (position, 16-byte vector); the batch is walked in order (deterministic).
template <typename T>
__global__ __launch_bounds__(256) void embed_bwd_replicated_kernel(int b, int s, int H, const T* dx0, T* dz0,
                                                                   T* __restrict__ dpos, DropArgs drop) {
  constexpr int VN = Vec16<T>::N;
  const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;      // vector index inside the [s, H] block
  const size_t per = (size_t)s * H / VN;
  if (idx >= per) return;
  float acc[VN];
#pragma unroll
  for (int e = 0; e < VN; ++e) acc[e] = 0.f;
  for (int bi = 0; bi < b; ++bi) {
    const size_t off = ((size_t)bi * per + idx) * VN;
    Vec16<T> x, o;
    x.load(dx0 + off);
    float v[VN];
#pragma unroll
    for (int e = 0; e < VN; ++e) v[e] = x.get(e);
    if (drop.enabled) drop_apply<VN>(drop, off, v);
#pragma unroll
    for (int e = 0; e < VN; ++e) {
      o.set(e, v[e]);
      acc[e] += o.get(e);
    }
    if (dz0 != nullptr && (drop.enabled || dz0 != dx0)) o.store(dz0 + off);
  }
  if (dpos != nullptr) {
    Vec16<T> o;
#pragma unroll
    for (int e = 0; e < VN; ++e) o.set(e, acc[e]);
    o.store(dpos + idx * VN);
  }
}

hipError_t launch_embed_fwd(int dtype, int T, int H, int Vl, int v0, const int32_t* ids, const void* E, int32_t* perm,
                            void* partial, hipStream_t st) {
  hipLaunchKernelGGL(embed_rank_kernel, dim3((T + 255) / 256), dim3(256), 0, st, T, ids, v0, Vl, perm);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (dtype == MLM_BF16)
    hipLaunchKernelGGL((embed_fwd_kernel<bf16>), dim3((T + 3) / 4), dim3(256), 0, st, T, H, Vl, v0, ids, perm,
                       (const bf16*)E, (bf16*)partial);
  else
    hipLaunchKernelGGL((embed_fwd_kernel<float>), dim3((T + 3) / 4), dim3(256), 0, st, T, H, Vl, v0, ids, perm,
                       (const float*)E, (float*)partial);
  return hipGetLastError();
}

template <typename T>
static hipError_t embed_bwd_dispatch(int Tn, int H, int Vl, int v0, const int32_t* ids, const int32_t* perm,
                                     const void* dz, void* dE, hipStream_t st) {
  constexpr int VN = Vec16<T>::N;
  const int nv = (H / VN + 63) / 64;
  dim3 grid((Tn + 3) / 4), block(256);
#define MLM_EB(NVV)                                                                                         \
  case NVV:                                                                                                 \
    hipLaunchKernelGGL((embed_bwd_kernel<T, NVV>), grid, block, 0, st, Tn, H, Vl, v0, ids, perm, (const T*)dz, \
                       (T*)dE);                                                                             \
    break;
  switch (nv) {
    MLM_EB(1) MLM_EB(2) MLM_EB(3) MLM_EB(4) MLM_EB(5) MLM_EB(6) MLM_EB(7) MLM_EB(8)
    default: return hipErrorInvalidValue;
  }
#undef MLM_EB
  return hipGetLastError();
}

hipError_t launch_embed_bwd(int dtype, int T, int H, int Vl, int v0, const int32_t* ids, const int32_t* perm,
                            const void* dz, void* dE, hipStream_t st) {
  return dtype == MLM_BF16 ? embed_bwd_dispatch<bf16>(T, H, Vl, v0, ids, perm, dz, dE, st)
                           : embed_bwd_dispatch<float>(T, H, Vl, v0, ids, perm, dz, dE, st);
}

hipError_t launch_embed_bwd_replicated(int dtype, int b, int s, int H, const void* dx0, void* dz0, void* dpos,
                                       const mlm_dropout* drop, hipStream_t st) {
  const DropArgs da = make_drop_args(drop);
  if (dtype == MLM_BF16) {
    const size_t per = (size_t)s * H / 8;
    hipLaunchKernelGGL((embed_bwd_replicated_kernel<bf16>), dim3((unsigned)((per + 255) / 256)), dim3(256), 0, st, b, s,
                       H, (const bf16*)dx0, (bf16*)dz0, (bf16*)dpos, da);
  } else {
    const size_t per = (size_t)s * H / 4;
    hipLaunchKernelGGL((embed_bwd_replicated_kernel<float>), dim3((unsigned)((per + 255) / 256)), dim3(256), 0, st, b,
                       s, H, (const float*)dx0, (float*)dz0, (float*)dpos, da);
  }
  return hipGetLastError();
}

}  // namespace mlm
