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
// The T x T comparisons are split over blockIdx.y: block (x, y) counts, for its 256 tokens, the tokens t' of slice y
// that precede them, and writes the partial count; embed_scatter_kernel adds the slices' counts (integers: exact in
// any order) and scatters.  Keys are staged through LDS and compared four per LDS read.
constexpr int kRankChunk = 1024;

__device__ __forceinline__ int embed_key(const int32_t* ids, int i, int v0, int Vl) {
  const int loc = ids[i] - v0;
  return (loc >= 0 && loc < Vl) ? loc : Vl;
}

__global__ __launch_bounds__(256) void embed_rank_kernel(int T, int nslice, const int32_t* __restrict__ ids, int v0,
                                                         int Vl, int32_t* __restrict__ partial) {
  __shared__ __attribute__((aligned(16))) int32_t sk[kRankChunk];
  const int t = blockIdx.x * 256 + threadIdx.x;
  const int my = t < T ? embed_key(ids, t, v0, Vl) : 0;
  // slice y covers chunks y, y + nslice, ... of kRankChunk tokens
  int rank = 0;
  for (int c0 = blockIdx.y * kRankChunk; c0 < T; c0 += nslice * kRankChunk) {
    __syncthreads();
    for (int i = threadIdx.x; i < kRankChunk; i += 256)
      sk[i] = c0 + i < T ? embed_key(ids, c0 + i, v0, Vl) : 0x7FFFFFFF;      // padding sorts after everything
    __syncthreads();
    // tokens before t in index order win ties: in this chunk those are the first (t - c0) entries
    const int before = min(max(t - c0, 0), kRankChunk);
#pragma unroll 4
    for (int i = 0; i < kRankChunk; i += 4) {
      const int4 k = *reinterpret_cast<const int4*>(&sk[i]);
      rank += (k.x < my || (k.x == my && i + 0 < before)) ? 1 : 0;
      rank += (k.y < my || (k.y == my && i + 1 < before)) ? 1 : 0;
      rank += (k.z < my || (k.z == my && i + 2 < before)) ? 1 : 0;
      rank += (k.w < my || (k.w == my && i + 3 < before)) ? 1 : 0;
    }
  }
  if (t < T) partial[(size_t)blockIdx.y * T + t] = rank;
}

__global__ __launch_bounds__(256) void embed_scatter_kernel(int T, int nslice, const int32_t* __restrict__ partial,
                                                            int32_t* __restrict__ perm) {
  const int t = blockIdx.x * 256 + threadIdx.x;
  if (t >= T) return;
  int rank = 0;
  for (int y = 0; y < nslice; ++y) rank += partial[(size_t)y * T + t];
  perm[rank] = t;
}

// One wave per (sorted position, group of 64 rows of E_r): lane h reads E_r[h0 + h, loc] and the wave writes 64
// consecutive elements of the token's row of the partial (zeros for a token outside the shard).  blockIdx.x (the
// sorted positions) varies fastest, so the blocks in flight together share a row group -- 64 rows of E_r, which
// stay in the L2 -- and walk its columns in increasing order.
template <typename T>
__global__ __launch_bounds__(256) void embed_fwd_kernel(int Tn, int H, int Vl, int v0, const int32_t* __restrict__ ids,
                                                        const int32_t* __restrict__ perm, const T* __restrict__ E,
                                                        T* __restrict__ out) {
  const int lane = threadIdx.x & 63;
  const int k = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int h = blockIdx.y * 64 + lane;
  if (k >= Tn || h >= H) return;
  const int t = perm[k];
  const int loc = ids[t] - v0;
  const bool inside = loc >= 0 && loc < Vl;           // wave-uniform
  out[(size_t)t * H + h] = inside ? E[(size_t)h * Vl + loc] : from_f32<T>(0.f);
}

// One wave per (sorted position, group of 64 rows of dE_r); the wave at the head of a run of equal local ids sums the
// run's rows of dz0 in token order (fp32) and adds the sum to column `loc` of dE_r.  Element-sized accesses:
// neighbouring columns belong to other waves.
template <typename T>
__global__ __launch_bounds__(256) void embed_bwd_kernel(int Tn, int H, int Vl, int v0, const int32_t* __restrict__ ids,
                                                        const int32_t* __restrict__ perm, const T* __restrict__ dz,
                                                        T* __restrict__ dE) {
  const int lane = threadIdx.x & 63;
  const int k = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int h = blockIdx.y * 64 + lane;
  if (k >= Tn) return;
  const int loc = ids[perm[k]] - v0;
  if (loc < 0 || loc >= Vl) return;                   // outside the shard (wave-uniform)
  if (k > 0 && ids[perm[k - 1]] - v0 == loc) return;  // not the head of its run
  float acc = 0.f;
  for (int kk = k; kk < Tn; ++kk) {
    const int t = perm[kk];
    if (ids[t] - v0 != loc) break;                    // end of the run (wave-uniform)
    if (h < H) acc += to_f32(dz[(size_t)t * H + h]);
  }
  if (h < H) {
    T* p = dE + (size_t)h * Vl + loc;
    *p = from_f32<T>(to_f32(*p) + acc);
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

// The rank partials ([nslice][T] int32) live in the partial output buffer until the gather overwrites it: a row of
// the partial has H elements, so up to H * sizeof(element) / 4 slices fit.
hipError_t launch_embed_fwd(int dtype, int T, int H, int Vl, int v0, const int32_t* ids, const void* E, int32_t* perm,
                            void* partial, hipStream_t st) {
  const int esz = dtype == MLM_BF16 ? 2 : 4;
  int nslice = (T + kRankChunk - 1) / kRankChunk;
  nslice = nslice < 1 ? 1 : (nslice > 16 ? 16 : nslice);
  if (nslice > H * esz / 4) nslice = H * esz / 4;
  hipLaunchKernelGGL(embed_rank_kernel, dim3((T + 255) / 256, nslice), dim3(256), 0, st, T, nslice, ids, v0, Vl,
                     (int32_t*)partial);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(embed_scatter_kernel, dim3((T + 255) / 256), dim3(256), 0, st, T, nslice, (const int32_t*)partial,
                     perm);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  dim3 grid((T + 3) / 4, (H + 63) / 64);
  if (dtype == MLM_BF16)
    hipLaunchKernelGGL((embed_fwd_kernel<bf16>), grid, dim3(256), 0, st, T, H, Vl, v0, ids, perm, (const bf16*)E,
                       (bf16*)partial);
  else
    hipLaunchKernelGGL((embed_fwd_kernel<float>), grid, dim3(256), 0, st, T, H, Vl, v0, ids, perm, (const float*)E,
                       (float*)partial);
  return hipGetLastError();
}

hipError_t launch_embed_bwd(int dtype, int T, int H, int Vl, int v0, const int32_t* ids, const int32_t* perm,
                            const void* dz, void* dE, hipStream_t st) {
  dim3 grid((T + 3) / 4, (H + 63) / 64);
  if (dtype == MLM_BF16)
    hipLaunchKernelGGL((embed_bwd_kernel<bf16>), grid, dim3(256), 0, st, T, H, Vl, v0, ids, perm, (const bf16*)dz,
                       (bf16*)dE);
  else
    hipLaunchKernelGGL((embed_bwd_kernel<float>), grid, dim3(256), 0, st, T, H, Vl, v0, ids, perm, (const float*)dz,
                       (float*)dE);
  return hipGetLastError();
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
