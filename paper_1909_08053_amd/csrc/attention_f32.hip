// fp32 attention for dtype MLM_F32 (the 1e-4 parity path; small shapes).  Streaming-softmax
// forward and a two-kernel backward (dQ per query row, dK/dV per key row) that recompute the
// probabilities from the saved log-sum-exp, so nothing of size s x s is ever stored and no
// atomics are needed (results are deterministic).  One thread owns one row; K/V (or Q/dO)
// tiles are staged through LDS and read as broadcasts.
// Masking follows the integer predicate allowed(i,j) = (j < key_len[b]) && (!causal || j <= i);
// excluded keys contribute exactly zero.
// Dropout of the probabilities (a.drop.enabled): the forward kernel draws the keep decision of element
// ((batch, head, i), j) from the counter-based generator, saves it as one bit per key and uses p_ij keep / (1 - p) in
// C = P V; the row sum and the log-sum-exp stay those of the undropped scores.  The backward kernels read the bits.
#include "common.h"
#include "rng.h"

namespace mlm {

constexpr int AF_TILE = 32;

template <int D>
__global__ __launch_bounds__(64) void attn_fwd_f32_kernel(AttnArgs a) {
  extern __shared__ float lds[];
  float* sK = lds;                      // [AF_TILE][D]
  float* sV = lds + AF_TILE * D;        // [AF_TILE][D]
  const int lane = threadIdx.x;
  const int i = blockIdx.x * 64 + lane;
  const int hd = blockIdx.y, bi = blockIdx.z;
  const int ld = 3 * a.hl * D;
  const float* qkv = (const float*)a.qkv;
  const size_t tok0 = (size_t)bi * a.s;
  const int klen = attn_key_len(a.key_len, bi, a.s);
  const bool active = i < a.s;
  const float scale = 1.0f / sqrtf((float)D);
  float q[D], o[D];
#pragma unroll
  for (int c = 0; c < D; ++c) {
    q[c] = active ? qkv[(tok0 + i) * ld + hd * D + c] : 0.f;
    o[c] = 0.f;
  }
  float m = -INFINITY, l = 0.f;
  int kend = klen;
  if (a.causal) kend = min(kend, min(a.s, blockIdx.x * 64 + 64));
  const size_t row = ((size_t)bi * a.hl + hd) * a.s + (active ? i : 0);   // row of the [b, hl, s, s] probability tensor
  for (int k0 = 0; k0 < kend; k0 += AF_TILE) {
    for (int e = lane; e < AF_TILE * D; e += 64) {
      const int j = e / D, c = e % D;
      const bool ok = k0 + j < a.s;
      sK[e] = ok ? qkv[(tok0 + k0 + j) * ld + (a.hl + hd) * D + c] : 0.f;
      sV[e] = ok ? qkv[(tok0 + k0 + j) * ld + (2 * a.hl + hd) * D + c] : 0.f;
    }
    __syncthreads();
    if (active) {
      uint32_t bits = 0xFFFFFFFFu;                  // keep bits of keys k0 .. k0 + 31
      if (a.drop.enabled) {
        bits = 0;
#pragma unroll
        for (int g = 0; g < AF_TILE / 4; ++g) bits |= drop_keep4(a.drop, (row * a.s + k0 + 4 * g) >> 2) << (4 * g);
        a.keep_bits[row * a.keep_pitch + k0 / 32] = bits;
      }
      for (int j = 0; j < AF_TILE; ++j) {
        const int key = k0 + j;
        if (key >= klen || (a.causal && key > i)) continue;
        float sc = 0.f;
#pragma unroll
        for (int c = 0; c < D; ++c) sc = fmaf(q[c], sK[j * D + c], sc);
        sc *= scale;
        const float mn = fmaxf(m, sc);
        const float corr = expf(m - mn);
        const float p = expf(sc - mn);
        l = l * corr + p;
        const float pd = ((bits >> j) & 1u) ? p : 0.f;
#pragma unroll
        for (int c = 0; c < D; ++c) o[c] = o[c] * corr + pd * sV[j * D + c];
        m = mn;
      }
    }
    __syncthreads();
  }
  if (active) {
    const float inv = a.drop.scale / l;
    float* ctx = (float*)a.ctx;
#pragma unroll
    for (int c = 0; c < D; ++c) ctx[(tok0 + i) * (a.hl * D) + hd * D + c] = o[c] * inv;
    a.lse[((size_t)bi * a.hl + hd) * a.s + i] = m + logf(l);
  }
}

// dQ_i = scale * sum_j dS_ij K_j,  dS_ij = P_ij (dO_i . V_j - delta_i),  P_ij = exp(scale q_i.k_j - lse_i)
template <int D>
__global__ __launch_bounds__(64) void attn_bwd_dq_f32_kernel(AttnArgs a) {
  extern __shared__ float lds[];
  float* sK = lds;
  float* sV = lds + AF_TILE * D;
  float* sdO = lds + 2 * AF_TILE * D;   // [64][D+1] this block's dO rows
  const int lane = threadIdx.x;
  const int i = blockIdx.x * 64 + lane;
  const int hd = blockIdx.y, bi = blockIdx.z;
  const int ld = 3 * a.hl * D;
  const float* qkv = (const float*)a.qkv;
  const float* dctx = (const float*)a.dctx;
  const size_t tok0 = (size_t)bi * a.s;
  const int klen = attn_key_len(a.key_len, bi, a.s);
  const bool active = i < a.s;
  const float scale = 1.0f / sqrtf((float)D);
  float q[D], dq[D];
#pragma unroll
  for (int c = 0; c < D; ++c) {
    q[c] = active ? qkv[(tok0 + i) * ld + hd * D + c] : 0.f;
    sdO[lane * (D + 1) + c] = active ? dctx[(tok0 + i) * (a.hl * D) + hd * D + c] : 0.f;
    dq[c] = 0.f;
  }
  const float lse = active ? a.lse[((size_t)bi * a.hl + hd) * a.s + i] : 0.f;
  const float dl = active ? a.delta[((size_t)bi * a.hl + hd) * a.s + i] : 0.f;
  const size_t row = ((size_t)bi * a.hl + hd) * a.s + (active ? i : 0);
  int kend = klen;
  if (a.causal) kend = min(kend, min(a.s, blockIdx.x * 64 + 64));
  for (int k0 = 0; k0 < kend; k0 += AF_TILE) {
    for (int e = lane; e < AF_TILE * D; e += 64) {
      const int j = e / D, c = e % D;
      const bool ok = k0 + j < a.s;
      sK[e] = ok ? qkv[(tok0 + k0 + j) * ld + (a.hl + hd) * D + c] : 0.f;
      sV[e] = ok ? qkv[(tok0 + k0 + j) * ld + (2 * a.hl + hd) * D + c] : 0.f;
    }
    __syncthreads();
    if (active) {
      const uint32_t bits = a.drop.enabled ? a.keep_bits[row * a.keep_pitch + k0 / 32] : 0xFFFFFFFFu;
      for (int j = 0; j < AF_TILE; ++j) {
        const int key = k0 + j;
        if (key >= klen || (a.causal && key > i)) continue;
        float sc = 0.f, dp = 0.f;
#pragma unroll
        for (int c = 0; c < D; ++c) {
          sc = fmaf(q[c], sK[j * D + c], sc);
          dp = fmaf(sdO[lane * (D + 1) + c], sV[j * D + c], dp);
        }
        dp = ((bits >> j) & 1u) ? dp * a.drop.scale : 0.f;     // gradient w.r.t. the undropped probability
        const float p = expf(sc * scale - lse);
        const float ds = p * (dp - dl);
#pragma unroll
        for (int c = 0; c < D; ++c) dq[c] = fmaf(ds, sK[j * D + c], dq[c]);
      }
    }
    __syncthreads();
  }
  if (active) {
    float* dqkv = (float*)a.dqkv;
#pragma unroll
    for (int c = 0; c < D; ++c) dqkv[(tok0 + i) * ld + hd * D + c] = dq[c] * scale;
  }
}

// dV_j = sum_i P_ij dO_i,  dK_j = scale * sum_i dS_ij Q_i   (one thread per key row j)
template <int D>
__global__ __launch_bounds__(64) void attn_bwd_dkv_f32_kernel(AttnArgs a) {
  extern __shared__ float lds[];
  float* sQ = lds;                          // [AF_TILE][D]
  float* sdO = lds + AF_TILE * D;           // [AF_TILE][D]
  float* sKj = lds + 2 * AF_TILE * D;       // [64][D+1] this block's K rows
  float* sVj = sKj + 64 * (D + 1);          // [64][D+1]
  float* sLse = sVj + 64 * (D + 1);         // [AF_TILE]
  float* sDl = sLse + AF_TILE;              // [AF_TILE]
  const int lane = threadIdx.x;
  const int j = blockIdx.x * 64 + lane;
  const int hd = blockIdx.y, bi = blockIdx.z;
  const int ld = 3 * a.hl * D;
  const float* qkv = (const float*)a.qkv;
  const float* dctx = (const float*)a.dctx;
  const size_t tok0 = (size_t)bi * a.s;
  const int klen = attn_key_len(a.key_len, bi, a.s);
  const bool active = j < a.s && j < klen;
  const float scale = 1.0f / sqrtf((float)D);
  float dk[D], dv[D];
#pragma unroll
  for (int c = 0; c < D; ++c) {
    const bool ok = j < a.s;
    sKj[lane * (D + 1) + c] = ok ? qkv[(tok0 + j) * ld + (a.hl + hd) * D + c] : 0.f;
    sVj[lane * (D + 1) + c] = ok ? qkv[(tok0 + j) * ld + (2 * a.hl + hd) * D + c] : 0.f;
    dk[c] = 0.f;
    dv[c] = 0.f;
  }
  const int ibeg = a.causal ? (blockIdx.x * 64) / AF_TILE * AF_TILE : 0;
  for (int i0 = ibeg; i0 < a.s; i0 += AF_TILE) {
    for (int e = lane; e < AF_TILE * D; e += 64) {
      const int ii = e / D, c = e % D;
      const bool ok = i0 + ii < a.s;
      sQ[e] = ok ? qkv[(tok0 + i0 + ii) * ld + hd * D + c] : 0.f;
      sdO[e] = ok ? dctx[(tok0 + i0 + ii) * (a.hl * D) + hd * D + c] : 0.f;
    }
    if (lane < AF_TILE) {
      const bool ok = i0 + lane < a.s;
      sLse[lane] = ok ? a.lse[((size_t)bi * a.hl + hd) * a.s + i0 + lane] : 0.f;
      sDl[lane] = ok ? a.delta[((size_t)bi * a.hl + hd) * a.s + i0 + lane] : 0.f;
    }
    __syncthreads();
    if (active) {
      for (int ii = 0; ii < AF_TILE; ++ii) {
        const int i = i0 + ii;
        if (i >= a.s || (a.causal && j > i)) continue;
        float sc = 0.f, dp = 0.f;
#pragma unroll
        for (int c = 0; c < D; ++c) {
          sc = fmaf(sQ[ii * D + c], sKj[lane * (D + 1) + c], sc);
          dp = fmaf(sdO[ii * D + c], sVj[lane * (D + 1) + c], dp);
        }
        const float p = expf(sc * scale - sLse[ii]);
        float keep = 1.0f;
        if (a.drop.enabled) {
          const size_t row = ((size_t)bi * a.hl + hd) * a.s + i;
          keep = ((a.keep_bits[row * a.keep_pitch + (j >> 5)] >> (j & 31)) & 1u) ? a.drop.scale : 0.f;
        }
        dp *= keep;
        const float ds = p * (dp - sDl[ii]);
        const float pd = p * keep;
#pragma unroll
        for (int c = 0; c < D; ++c) {
          dv[c] = fmaf(pd, sdO[ii * D + c], dv[c]);
          dk[c] = fmaf(ds, sQ[ii * D + c], dk[c]);
        }
      }
    }
    __syncthreads();
  }
  if (j < a.s) {
    float* dqkv = (float*)a.dqkv;
#pragma unroll
    for (int c = 0; c < D; ++c) {
      dqkv[(tok0 + j) * ld + (a.hl + hd) * D + c] = dk[c] * scale;
      dqkv[(tok0 + j) * ld + (2 * a.hl + hd) * D + c] = dv[c];
    }
  }
}

bool attn_f32_supported(int d) { return d > 0 && d % 16 == 0 && d <= 128; }

#define MLM_AF_SWITCH(MACRO)                                                                         \
  switch (a.d) {                                                                                     \
    case 16: MACRO(16) break; case 32: MACRO(32) break; case 48: MACRO(48) break;                    \
    case 64: MACRO(64) break; case 80: MACRO(80) break; case 96: MACRO(96) break;                    \
    case 112: MACRO(112) break; case 128: MACRO(128) break;                                          \
    default: return hipErrorInvalidValue;                                                            \
  }

hipError_t launch_attn_fwd_f32(const AttnArgs& a, hipStream_t st) {
  dim3 grid((a.s + 63) / 64, a.hl, a.b), block(64);
#define MLM_AF_FWD(DD)                                                                               \
  {                                                                                                  \
    const size_t lds = (size_t)2 * AF_TILE * DD * sizeof(float);                                     \
    hipLaunchKernelGGL((attn_fwd_f32_kernel<DD>), grid, block, lds, st, a);                          \
  }
  MLM_AF_SWITCH(MLM_AF_FWD)
#undef MLM_AF_FWD
  return hipGetLastError();
}

hipError_t launch_attn_bwd_f32(const AttnArgs& a, hipStream_t st) {
  dim3 grid((a.s + 63) / 64, a.hl, a.b), block(64);
#define MLM_AF_BWD(DD)                                                                               \
  {                                                                                                  \
    const size_t lds1 = ((size_t)2 * AF_TILE * DD + 64 * (DD + 1)) * sizeof(float);                  \
    hipLaunchKernelGGL((attn_bwd_dq_f32_kernel<DD>), grid, block, lds1, st, a);                      \
    const size_t lds2 = ((size_t)2 * AF_TILE * DD + 2 * 64 * (DD + 1) + 2 * AF_TILE) * sizeof(float); \
    if (lds2 > 64 * 1024) {                                                                          \
      hipError_t e = hipFuncSetAttribute((const void*)attn_bwd_dkv_f32_kernel<DD>,                   \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds2);     \
      if (e != hipSuccess) return e;                                                                 \
    }                                                                                                \
    hipLaunchKernelGGL((attn_bwd_dkv_f32_kernel<DD>), grid, block, lds2, st, a);                     \
  }
  MLM_AF_SWITCH(MLM_AF_BWD)
#undef MLM_AF_BWD
  return hipGetLastError();
}

}  // namespace mlm
