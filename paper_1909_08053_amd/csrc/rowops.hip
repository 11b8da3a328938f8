// Bandwidth-bound kernels of the layer shard: layer norm (forward / backward), the single-GPU
// stand-in for the all-reduce (combine), bias-gradient column sums, and the cross-entropy
// partial merges (Section 3 of the paper: replicated LN/residual, g/f reductions, loss fused
// with the vocabulary-parallel logits).  One wavefront (64 lanes) owns one token row; row
// statistics are wave-level shuffles, HBM access is 16-byte vectors, coalesced along H.
#include <mutex>
#include "common.h"
#include "rng.h"

namespace mlm {

struct PartialPtrs { const void* p[kMaxPartials]; };

// One token row (a lane's NV 16-byte vectors) of sum_r partials[r] + bias + residual: partials are added in the fixed
// order r = 0..n-1 (deterministic) in fp32 and the sum is rounded once to the storage type -- the value the separate
// combine kernel would have stored.  All of a partial's vectors are loaded before they are added, so the loads of a
// row overlap; a single partial with nothing to add is passed through untouched.  With dropout the row is
// residual + dropout(sum partials + bias): the mask of element row_off + column comes from the counter-based generator.
// (DROP is a template parameter: the generator's registers must not weigh on the dropout-free instantiation)
template <typename T, int NV, bool DROP>
__device__ __forceinline__ void combine_row(const PartialPtrs& ptrs, int n, const T* bias, const T* residual,
                                            size_t row_off, int lane, int nvec, Vec16<T> (&out)[NV],
                                            const DropArgs& drop) {
  constexpr int VN = Vec16<T>::N;
  if (!DROP && n == 1 && bias == nullptr && residual == nullptr) {
    const T* p = (const T*)ptrs.p[0] + row_off;
#pragma unroll
    for (int i = 0; i < NV; ++i)
      if (lane + 64 * i < nvec) out[i].load(p + (size_t)(lane + 64 * i) * VN);
    return;
  }
  float acc[NV][VN];
  if (!DROP && n == 1) {
    // one partial (the usual case on a GPU that holds one shard): the loads of all three sources are issued before the
    // first use, so a row costs one trip to memory instead of three; the sums are formed in the same order as below
    // (partial, then bias, then residual), hence bit-identical
    Vec16<T> tp[NV], tb[NV], tr[NV];
    const T* pp = (const T*)ptrs.p[0] + row_off;
#pragma unroll
    for (int i = 0; i < NV; ++i)
      if (lane + 64 * i < nvec) {
        tp[i].load(pp + (size_t)(lane + 64 * i) * VN);
        if (bias) tb[i].load(bias + (size_t)(lane + 64 * i) * VN);
        if (residual) tr[i].load(residual + row_off + (size_t)(lane + 64 * i) * VN);
      }
#pragma unroll
    for (int i = 0; i < NV; ++i)
      if (lane + 64 * i < nvec) {
#pragma unroll
        for (int e = 0; e < VN; ++e) {
          float a = 0.f + tp[i].get(e);
          if (bias) a += tb[i].get(e);
          if (residual) a += tr[i].get(e);
          out[i].set(e, a);
        }
      }
    return;
  }
#pragma unroll
  for (int i = 0; i < NV; ++i)
#pragma unroll
    for (int e = 0; e < VN; ++e) acc[i][e] = 0.f;
  for (int k = 0; k < n + 2; ++k) {
    if (DROP && k == n + 1) {                         // everything but the residual is in: drop it out
#pragma unroll
      for (int i = 0; i < NV; ++i)
        if (lane + 64 * i < nvec) drop_apply<VN>(drop, row_off + (size_t)(lane + 64 * i) * VN, acc[i]);
    }
    const T* p = k < n ? (const T*)ptrs.p[k] + row_off : (k == n ? bias : (residual ? residual + row_off : nullptr));
    if (p == nullptr) continue;                       // uniform
    Vec16<T> t[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i)
      if (lane + 64 * i < nvec) t[i].load(p + (size_t)(lane + 64 * i) * VN);
#pragma unroll
    for (int i = 0; i < NV; ++i)
      if (lane + 64 * i < nvec) {
#pragma unroll
        for (int e = 0; e < VN; ++e) acc[i][e] += t[i].get(e);
      }
  }
#pragma unroll
  for (int i = 0; i < NV; ++i)
#pragma unroll
    for (int e = 0; e < VN; ++e) out[i].set(e, acc[i][e]);
}

// ------------------------------------------------------------------------------ layer norm forward
// FUSED: the input row is first formed as sum of partials + bias + residual (the single-GPU stand-in for the
// all-reduce followed by the bias/residual add), stored to x_out, and normalised from registers.
template <typename T, int NV, bool FUSED, bool DROP>
__global__ __launch_bounds__(256) void ln_fwd_kernel(int rows, int H, float eps, const T* __restrict__ x,
                                                     const T* __restrict__ gamma, const T* __restrict__ beta,
                                                     T* __restrict__ y, float* __restrict__ mean,
                                                     float* __restrict__ rstd, PartialPtrs ptrs, int n,
                                                     const T* __restrict__ bias, const T* residual, T* x_out,
                                                     DropArgs drop) {
  constexpr int VN = Vec16<T>::N;
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const int nvec = H / VN;
  const T* xr = x + (size_t)row * H;
  Vec16<T> v[NV];
  float sum = 0.f;
  if (FUSED) combine_row<T, NV, DROP>(ptrs, n, bias, residual, (size_t)row * H, lane, nvec, v, drop);
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int idx = lane + 64 * i;
    if (idx < nvec) {
      if (FUSED) v[i].store(x_out + (size_t)row * H + (size_t)idx * VN);
      else v[i].load(xr + (size_t)idx * VN);
#pragma unroll
      for (int e = 0; e < VN; ++e) sum += v[i].get(e);
    }
  }
  const float mu = wave_sum(sum) / (float)H;
  float sq = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    if (lane + 64 * i < nvec) {
#pragma unroll
      for (int e = 0; e < VN; ++e) { const float d = v[i].get(e) - mu; sq += d * d; }
    }
  }
  const float rs = 1.0f / sqrtf(wave_sum(sq) / (float)H + eps);
  if (lane == 0) { mean[row] = mu; rstd[row] = rs; }
  T* yr = y + (size_t)row * H;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int idx = lane + 64 * i;
    if (idx < nvec) {
      Vec16<T> g, b, o;
      g.load(gamma + (size_t)idx * VN);
      b.load(beta + (size_t)idx * VN);
#pragma unroll
      for (int e = 0; e < VN; ++e) o.set(e, (v[i].get(e) - mu) * rs * g.get(e) + b.get(e));
      o.store(yr + (size_t)idx * VN);
    }
  }
}

template <typename T>
static hipError_t ln_fwd_dispatch(int rows, int H, float eps, const void* x, const void* gamma, const void* beta,
                                  void* y, float* mean, float* rstd, const PartialPtrs* pp, int n, const void* bias,
                                  const void* residual, void* x_out, const DropArgs& drop, hipStream_t st) {
  constexpr int VN = Vec16<T>::N;
  const int nv = (H / VN + 63) / 64;
  dim3 grid((rows + 3) / 4), block(256);
  PartialPtrs none;
  for (int k = 0; k < kMaxPartials; ++k) none.p[k] = nullptr;
#define MLM_LN_FWD(NVV)                                                                                    \
  case NVV:                                                                                                \
    if (pp && drop.enabled)                                                                                \
      hipLaunchKernelGGL((ln_fwd_kernel<T, NVV, true, true>), grid, block, 0, st, rows, H, eps, (const T*)x, \
                         (const T*)gamma, (const T*)beta, (T*)y, mean, rstd, *pp, n, (const T*)bias,       \
                         (const T*)residual, (T*)x_out, drop);                                             \
    else if (pp)                                                                                           \
      hipLaunchKernelGGL((ln_fwd_kernel<T, NVV, true, false>), grid, block, 0, st, rows, H, eps, (const T*)x, \
                         (const T*)gamma, (const T*)beta, (T*)y, mean, rstd, *pp, n, (const T*)bias,       \
                         (const T*)residual, (T*)x_out, drop);                                             \
    else                                                                                                   \
      hipLaunchKernelGGL((ln_fwd_kernel<T, NVV, false, false>), grid, block, 0, st, rows, H, eps, (const T*)x, \
                         (const T*)gamma, (const T*)beta, (T*)y, mean, rstd, none, 0, (const T*)nullptr,   \
                         (const T*)nullptr, (T*)nullptr, drop);                                            \
    break;
  switch (nv) {
    MLM_LN_FWD(1) MLM_LN_FWD(2) MLM_LN_FWD(3) MLM_LN_FWD(4) MLM_LN_FWD(5) MLM_LN_FWD(6) MLM_LN_FWD(7) MLM_LN_FWD(8)
    default: return hipErrorInvalidValue;
  }
#undef MLM_LN_FWD
  return hipGetLastError();
}

hipError_t launch_layernorm_fwd(int dtype, int T, int H, float eps, const void* x, const void* gamma,
                                const void* beta, void* y, float* mean, float* rstd, hipStream_t st) {
  const DropArgs nd = make_drop_args(nullptr);
  return dtype == MLM_BF16
             ? ln_fwd_dispatch<bf16>(T, H, eps, x, gamma, beta, y, mean, rstd, nullptr, 0, nullptr, nullptr, nullptr, nd, st)
             : ln_fwd_dispatch<float>(T, H, eps, x, gamma, beta, y, mean, rstd, nullptr, 0, nullptr, nullptr, nullptr, nd, st);
}

hipError_t launch_combine_layernorm_fwd(int dtype, int T, int H, float eps, const void* const* partials, int n,
                                        const void* bias, const void* residual, void* x_out, const void* gamma,
                                        const void* beta, void* y, float* mean, float* rstd, const mlm_dropout* drop,
                                        hipStream_t st) {
  PartialPtrs pp;
  for (int k = 0; k < kMaxPartials; ++k) pp.p[k] = k < n ? partials[k] : nullptr;
  const DropArgs da = make_drop_args(drop);
  return dtype == MLM_BF16
             ? ln_fwd_dispatch<bf16>(T, H, eps, nullptr, gamma, beta, y, mean, rstd, &pp, n, bias, residual, x_out, da, st)
             : ln_fwd_dispatch<float>(T, H, eps, nullptr, gamma, beta, y, mean, rstd, &pp, n, bias, residual, x_out, da, st);
}

// ------------------------------------------------------------------------------ layer norm backward
// Block = one wave per 64 vectors of a row; the grid has one block per
// kLnBwdRowsPerBlock rows and the rows are dealt to the blocks in batches of kLnBwdBatch, round-robin.  A lane owns
// ONE 16-byte vector of columns in every row, so its dgamma / dbeta (/ dx column-sum) partials are a handful of
// registers and several waves fit on a SIMD (a wave-per-row layout needs the partials of the whole row per lane:
// ~150 registers, one wave per SIMD, and ran at half the HBM rate).  The row statistics s1 = mean(dy gamma),
// s2 = mean(dy gamma xhat) need the whole row: every wave reduces its slab, the per-wave partials meet in LDS and are
// added in a fixed order (deterministic); one barrier per batch (the exchange buffer alternates).  Everything that needs
// no row statistic (dgamma, dbeta) is accumulated in the pass before the barrier; the pass after it is two fused
// multiply-adds per element.  The next batch (and its rows' mean / rstd) is prefetched while the current one is
// worked on.  The block's column partials go to the workspace and reduce_cols_kernel sums them over the blocks.
// VB = bytes per lane and row.  The kernel is bound by vector-ALU issue, not by memory (in-kernel timestamps: with
// 16-byte vectors a 3072-column bf16 row makes 6 waves, i.e. two of the four SIMDs carry two waves, and the barrier of
// every batch waits for those two); with 8-byte vectors the same row is 12 waves of half the work, three per SIMD.
//
// FUSED: dy is formed on the fly as the sum of n partial tensors (stored to dy_out if that is not NULL).
// SUM: the column sums of dx (the bias gradient of the layer that produced this layer norm's input) are accumulated
// as a third per-column partial next to dgamma / dbeta.
constexpr int kLnBwdBatch = 4;

// DZ: also emit dz_out = dropout-mask(dx) / (1 - p) (and sum ITS columns); a template parameter so that the generator
// costs the plain instantiations no registers.
template <typename T, int VB, bool FUSED, bool SUM, bool DZ>
__global__ __launch_bounds__(VB == 8 ? 768 : 512) void ln_bwd_kernel(int rows, int H, const T* __restrict__ dy, const T* __restrict__ x,
                                                     const T* __restrict__ gamma, const float* __restrict__ mean,
                                                     const float* __restrict__ rstd, const T* residual, T* dx,
                                                     float* __restrict__ ws, PartialPtrs ptrs, int n, T* dy_out,
                                                     DropArgs drop, T* dz_out) {
  typedef VecB<T, VB> V;
  constexpr int VN = V::N, RB = kLnBwdBatch, NP = SUM ? 3 : 2;
  static_assert(RB % 2 == 0, "two rows share one 64-lane exchange line");
  // exchange line h of a batch: quantity q = 2 (row & 1) + {0: s1, 1: s2} of rows 2h, 2h + 1 in lanes [16 q, 16 q + 16),
  // one slot per wave
  __shared__ __attribute__((aligned(16))) float red[2][RB / 2][64];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int idx = threadIdx.x;                      // this lane's vector of every row
  const bool active = idx < H / VN;
  const size_t col0 = (size_t)idx * VN;
  const float invH = 1.0f / (float)H;
  // slots of waves that do not exist stay zero, so the exchange can always add all sixteen
  for (int i = threadIdx.x; i < 2 * (RB / 2) * 64; i += blockDim.x) (&red[0][0][0])[i] = 0.f;
  __syncthreads();
  float gam[VN], dg[VN], db[VN], dsum[VN];
  {
    V g;
    if (active) g.load(gamma + col0);
#pragma unroll
    for (int e = 0; e < VN; ++e) {
      gam[e] = active ? g.get(e) : 0.f;
      dg[e] = 0.f; db[e] = 0.f; dsum[e] = 0.f;
    }
  }
  // batches are dealt round-robin over the blocks: at any moment the grid reads ONE contiguous window of each tensor
  // (a block that owned a contiguous chunk of rows would make all blocks walk memory at the same offset of a fixed
  // stride, which concentrates the traffic on a part of the memory channels)
  const int nbatch = (rows + RB - 1) / RB, row_end = rows;
  struct Batch { V dy[RB], x[RB], res[RB]; float mu[RB], rs[RB]; };
  auto load_batch = [&](Batch& nb, int r0) {
#pragma unroll
    for (int j = 0; j < RB; ++j) {
      const int r = r0 + j;
      nb.mu[j] = mean[min(r, row_end - 1)];       // (loads only: arithmetic here would wait for them at once)
      nb.rs[j] = rstd[min(r, row_end - 1)];
      if (r < row_end && active) {
        const size_t off = (size_t)r * H + col0;
        if (FUSED) {
          if (n == 1) {
            nb.dy[j].load((const T*)ptrs.p[0] + off);
          } else {                                   // fixed order k = 0..n-1, fp32, rounded once
            float acc[VN];
#pragma unroll
            for (int e = 0; e < VN; ++e) acc[e] = 0.f;
            for (int k = 0; k < n; ++k) {
              V t;
              t.load((const T*)ptrs.p[k] + off);
#pragma unroll
              for (int e = 0; e < VN; ++e) acc[e] += t.get(e);
            }
#pragma unroll
            for (int e = 0; e < VN; ++e) nb.dy[j].set(e, acc[e]);
          }
          if (dy_out) nb.dy[j].store(dy_out + off);
        } else {
          nb.dy[j].load(dy + off);
        }
        nb.x[j].load(x + off);
        if (residual) nb.res[j].load(residual + off);
      }
    }
  };
  // one batch; par = which half of the exchange buffer (alternates, so one barrier per batch is enough)
  auto work = [&](const Batch& c, int r0, int par) {
    // first pass: everything that needs no row statistic -- the partial sums of s1 and s2 and the column sums
    // dgamma += dy xhat, dbeta += dy; xhat and dy gamma are kept for the second pass
    float xh[RB][VN], gg[RB][VN], ps1[RB], ps2[RB];
#pragma unroll
    for (int j = 0; j < RB; ++j) {
      ps1[j] = 0.f;
      ps2[j] = 0.f;
      const float nmr = -c.mu[j] * c.rs[j];          // xhat = x rstd - mean rstd
      if (r0 + j < row_end && active) {
#pragma unroll
        for (int e = 0; e < VN; ++e) {
          const float d = c.dy[j].get(e);
          xh[j][e] = fmaf(c.x[j].get(e), c.rs[j], nmr);
          gg[j][e] = d * gam[e];
          ps1[j] += gg[j][e];
          ps2[j] = fmaf(gg[j][e], xh[j][e], ps2[j]);
          dg[e] = fmaf(d, xh[j][e], dg[e]);
          db[e] += d;
        }
      }
    }
    // 2 RB independent wave reductions: their dependent chains interleave
#pragma unroll
    for (int j = 0; j < RB; ++j) {
      ps1[j] = wave_sum(ps1[j]);
      ps2[j] = wave_sum(ps2[j]);
    }
    if (lane == 0) {
#pragma unroll
      for (int j = 0; j < RB; ++j) {
        red[par][j >> 1][(2 * (j & 1) + 0) * 16 + wave] = ps1[j];
        red[par][j >> 1][(2 * (j & 1) + 1) * 16 + wave] = ps2[j];
      }
    }
    __syncthreads();
    // the waves' partials are added by the 16-lane row reduction (fixed order): one LDS read and five vector
    // operations per exchange line instead of a chain of adds per quantity in every lane
    float tot[RB / 2];
#pragma unroll
    for (int h = 0; h < RB / 2; ++h) tot[h] = row16_sum(red[par][h][lane]);
    // second pass: dx = rstd (dy gamma - s1 - xhat s2) written as (rstd dy gamma - rstd s1) - xhat (rstd s2)
#pragma unroll
    for (int j = 0; j < RB; ++j) {
      if (r0 + j >= row_end) break;                  // block-uniform
      const float s1 = lane_value(tot[j >> 1], (2 * (j & 1) + 0) * 16 + 15) * invH;
      const float s2 = lane_value(tot[j >> 1], (2 * (j & 1) + 1) * 16 + 15) * invH;
      const float rs1 = c.rs[j] * s1, rs2 = c.rs[j] * s2;
      if (active) {
        V o;
#pragma unroll
        for (int e = 0; e < VN; ++e) {
          float v = fmaf(-xh[j][e], rs2, fmaf(gg[j][e], c.rs[j], -rs1));
          if (residual) v += c.res[j].get(e);
          o.set(e, v);
          if (SUM && !DZ) dsum[e] += o.get(e);   // the stored (rounded) value, as a separate column sum would read it
        }
        o.store(dx + (size_t)(r0 + j) * H + col0);
        if (DZ) {
          // this layer norm's input was residual + dropout(z): emit dz = mask o dx / (1 - p) and sum ITS columns
          float z[VN];
#pragma unroll
          for (int e = 0; e < VN; ++e) z[e] = o.get(e);
          if (drop.enabled) drop_apply<VN>(drop, (size_t)(r0 + j) * H + col0, z);
          V oz;
#pragma unroll
          for (int e = 0; e < VN; ++e) {
            oz.set(e, z[e]);
            if (SUM) dsum[e] += oz.get(e);
          }
          oz.store(dz_out + (size_t)(r0 + j) * H + col0);
        }
      }
    }
  };
  // The next batch is in flight while the current one is worked on.  The batch is COPIED out of the registers the
  // loads target at the top of the loop: that is the one point where the wave waits for memory, and the compiler can
  // place it exactly (with buffers that swap roles, the conditional prefetch makes the count of younger loads depend
  // on the path, and the wait it then inserts before the first use also waits for the prefetch just issued).
  Batch cur, nxt;
  const int G = gridDim.x;
  if ((int)blockIdx.x < nbatch) load_batch(nxt, blockIdx.x * RB);
  int par = 0;
  for (int bt = blockIdx.x; bt < nbatch; bt += G, par ^= 1) {
    cur = nxt;
    if (bt + G < nbatch) load_batch(nxt, (bt + G) * RB);
    work(cur, bt * RB, par);
  }
  if (active) {
    float* out = ws + (size_t)blockIdx.x * NP * H + col0;
#pragma unroll
    for (int e = 0; e < VN; ++e) {
      out[e] = dg[e];
      out[H + e] = db[e];
      if (SUM) out[2 * H + e] = dsum[e];
    }
  }
}

// out[c] = sum_k ws[k][c] over nchunk row-chunks (the columns are up to three output vectors of `seg` entries): 16 float4 column groups x 16 chunk-slices per block; every slice
// sums its chunks in order and the 16 slices are added in a fixed order (deterministic).
template <typename T>
__device__ __forceinline__ void reduce_cols_block(int blk, int nchunk, int ncols, const float* __restrict__ ws,
                                                  T* out0, T* out1, T* out2, int seg) {
  __shared__ float4 red[16][17];
  const int cx = threadIdx.x & 15, sl = threadIdx.x >> 4;
  const int c = (blk * 16 + cx) * 4;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  if (c < ncols) {
#pragma unroll 4
    for (int k = sl; k < nchunk; k += 16) {
      const float4 v = *reinterpret_cast<const float4*>(ws + (size_t)k * ncols + c);
      acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
  }
  red[sl][cx] = acc;
  __syncthreads();
  if (sl == 0 && c < ncols) {
    float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int k = 0; k < 16; ++k) { t.x += red[k][cx].x; t.y += red[k][cx].y; t.z += red[k][cx].z; t.w += red[k][cx].w; }
    const float tv[4] = {t.x, t.y, t.z, t.w};
    T* out = c < seg ? out0 : (c < 2 * seg ? out1 : out2);   // segments are multiples of 4 columns
    const int cc = c % seg;
#pragma unroll
    for (int e = 0; e < 4; ++e) out[cc + e] = from_f32<T>(tv[e]);
  }
}

template <typename T>
__global__ __launch_bounds__(256) void reduce_cols_kernel(int nchunk, int ncols, const float* __restrict__ ws,
                                                          T* out0, T* out1, T* out2, int seg) {
  reduce_cols_block<T>(blockIdx.x, nchunk, ncols, ws, out0, out1, out2, seg);
}

// One finishing reduction: the block partials of a column-sum or layer-norm-backward launch and where their sums go.
struct ColReduce {
  const float* ws;
  void *out0, *out1, *out2;
  int nchunk, ncols, seg, dtype;
};
constexpr int kMaxDeferredSums = 16;
struct ColReduceBatch {
  ColReduce r[kMaxDeferredSums];
  int block_begin[kMaxDeferredSums + 1];
  int n;
};

// Several finishing reductions in one launch: a block looks up the reduction its index falls into and runs the same
// code as reduce_cols_kernel on it, so the sums are bit-identical to separate launches.
__global__ __launch_bounds__(256) void reduce_cols_batch_kernel(ColReduceBatch b) {
  int q = 0;
  while (q + 1 < b.n && (int)blockIdx.x >= b.block_begin[q + 1]) ++q;     // block-uniform
  const ColReduce& r = b.r[q];
  const int blk = blockIdx.x - b.block_begin[q];
  if (r.dtype == MLM_BF16)
    reduce_cols_block<bf16>(blk, r.nchunk, r.ncols, r.ws, (bf16*)r.out0, (bf16*)r.out1, (bf16*)r.out2, r.seg);
  else
    reduce_cols_block<float>(blk, r.nchunk, r.ncols, r.ws, (float*)r.out0, (float*)r.out1, (float*)r.out2, r.seg);
}

static hipError_t launch_reduce_cols(const ColReduce& r, hipStream_t st) {
  const dim3 grid((r.ncols + 63) / 64), block(256);
  if (r.dtype == MLM_BF16)
    hipLaunchKernelGGL((reduce_cols_kernel<bf16>), grid, block, 0, st, r.nchunk, r.ncols, r.ws, (bf16*)r.out0,
                       (bf16*)r.out1, (bf16*)r.out2, r.seg);
  else
    hipLaunchKernelGGL((reduce_cols_kernel<float>), grid, block, 0, st, r.nchunk, r.ncols, r.ws, (float*)r.out0,
                       (float*)r.out1, (float*)r.out2, r.seg);
  return hipGetLastError();
}

// Deferred finishing sums of the calling host thread.  While a list is open, a launch that produces block partials
// takes their storage from the list's own buffer (the call's workspace is reused by the next call) and records its
// reduction instead of launching it; deferred_sums_flush runs all recorded reductions as one kernel.  A launch that
// does not fit (buffer full, list full) finishes on the spot as if no list were open.
struct DeferredSums {
  bool open = false;
  char* buf = nullptr;
  size_t bytes = 0, used = 0;
  ColReduceBatch batch;
};
static thread_local DeferredSums t_defer;

hipError_t deferred_sums_begin(void* buf, size_t bytes) {
  if (t_defer.open || !buf) return hipErrorInvalidValue;
  t_defer.open = true;
  t_defer.buf = (char*)buf;
  t_defer.bytes = bytes;
  t_defer.used = 0;
  t_defer.batch.n = 0;
  t_defer.batch.block_begin[0] = 0;
  return hipSuccess;
}

bool deferred_sums_open() { return t_defer.open; }

// storage for `floats` partial values in the open list, or nullptr (no list, no room)
static float* deferred_reserve(size_t floats) {
  if (!t_defer.open || t_defer.batch.n >= kMaxDeferredSums) return nullptr;
  const size_t need = (floats * sizeof(float) + 255) & ~(size_t)255;
  if (t_defer.used + need > t_defer.bytes) return nullptr;
  float* p = reinterpret_cast<float*>(t_defer.buf + t_defer.used);
  t_defer.used += need;
  return p;
}

static void deferred_record(const ColReduce& r) {
  ColReduceBatch& b = t_defer.batch;
  b.r[b.n] = r;
  b.block_begin[b.n + 1] = b.block_begin[b.n] + (r.ncols + 63) / 64;
  ++b.n;
}

hipError_t deferred_sums_flush(hipStream_t st) {
  if (!t_defer.open) return hipErrorInvalidValue;
  t_defer.open = false;
  const ColReduceBatch& b = t_defer.batch;
  if (b.n == 0) return hipSuccess;
  if (b.n == 1) return launch_reduce_cols(b.r[0], st);
  hipLaunchKernelGGL(reduce_cols_batch_kernel, dim3(b.block_begin[b.n]), dim3(256), 0, st, b);
  return hipGetLastError();
}

template <typename T>
static hipError_t ln_bwd_dispatch(int rows, int H, const void* dy, const void* x, const void* gamma,
                                  const float* mean, const float* rstd, const void* residual, void* dx,
                                  void* dgamma, void* dbeta, float* ws, const PartialPtrs* pp, int n, void* dy_out,
                                  void* dx_colsum, const DropArgs& drop, void* dz_out, hipStream_t st) {
  // bf16 rows of up to 3072 columns (a multiple of 4) take the 8-byte form: twice the waves per row, at most 12
  constexpr bool kNarrow = sizeof(T) == 2;
  const bool narrow = kNarrow && H % 4 == 0 && H / 4 <= 768;
  const int vn = narrow ? 8 / (int)sizeof(T) : Vec16<T>::N;
  const int nwaves = (H / vn + 63) / 64;
  if (nwaves < 1 || nwaves > (narrow ? 12 : 8)) return hipErrorInvalidValue;
  const int nblk = (rows + kLnBwdRowsPerBlock - 1) / kLnBwdRowsPerBlock;
  PartialPtrs none;
  for (int k = 0; k < kMaxPartials; ++k) none.p[k] = nullptr;
  const int np = (pp && dx_colsum) ? 3 : 2;
  float* deferred = deferred_reserve((size_t)nblk * np * H);
  if (deferred) ws = deferred;
  dim3 grid(nblk), block(nwaves * 64);
#define MLM_LN_BWD_VB(VBYTES, F, S, Z)                                                                      \
  hipLaunchKernelGGL((ln_bwd_kernel<T, VBYTES, F, S, Z>), grid, block, 0, st, rows, H, (const T*)dy,        \
                     (const T*)x, (const T*)gamma, mean, rstd, (const T*)residual, (T*)dx, ws,              \
                     pp ? *pp : none, n, (T*)dy_out, drop, (T*)dz_out)
#define MLM_LN_BWD_GO(F, S, Z)                                                                              \
  do {                                                                                                      \
    if constexpr (kNarrow) {                                                                                \
      if (narrow) { MLM_LN_BWD_VB(8, F, S, Z); break; }                                                     \
    }                                                                                                       \
    MLM_LN_BWD_VB(16, F, S, Z);                                                                             \
  } while (0)
  if (pp && dx_colsum && dz_out) MLM_LN_BWD_GO(true, true, true);
  else if (pp && dz_out) MLM_LN_BWD_GO(true, false, true);
  else if (pp && dx_colsum) MLM_LN_BWD_GO(true, true, false);
  else if (pp) MLM_LN_BWD_GO(true, false, false);
  else MLM_LN_BWD_GO(false, false, false);
#undef MLM_LN_BWD_GO
#undef MLM_LN_BWD_VB
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const ColReduce fin = {ws, dgamma, dbeta, dx_colsum, nblk, np * H, H, sizeof(T) == 2 ? MLM_BF16 : MLM_F32};
  if (deferred) {
    deferred_record(fin);
    return hipSuccess;
  }
  return launch_reduce_cols(fin, st);
}

hipError_t launch_layernorm_bwd(int dtype, int T, int H, const void* dy, const void* x, const void* gamma,
                                const float* mean, const float* rstd, const void* residual_grad, void* dx,
                                void* dgamma, void* dbeta, float* ws, hipStream_t st) {
  const DropArgs nd = make_drop_args(nullptr);
  return dtype == MLM_BF16
             ? ln_bwd_dispatch<bf16>(T, H, dy, x, gamma, mean, rstd, residual_grad, dx, dgamma, dbeta, ws, nullptr, 0,
                                     nullptr, nullptr, nd, nullptr, st)
             : ln_bwd_dispatch<float>(T, H, dy, x, gamma, mean, rstd, residual_grad, dx, dgamma, dbeta, ws, nullptr, 0,
                                      nullptr, nullptr, nd, nullptr, st);
}

// ws: [ceil(T/kLnBwdRowsPerBlock)][3][H] float
hipError_t launch_combine_layernorm_bwd(int dtype, int T, int H, const void* const* partials, int n, const void* x,
                                        const void* gamma, const float* mean, const float* rstd,
                                        const void* residual_grad, void* dy_out, void* dx, void* dgamma, void* dbeta,
                                        void* dx_colsum, float* ws, const mlm_dropout* drop, void* dz_out,
                                        hipStream_t st) {
  PartialPtrs pp;
  for (int k = 0; k < kMaxPartials; ++k) pp.p[k] = k < n ? partials[k] : nullptr;
  const DropArgs da = make_drop_args(drop);
  return dtype == MLM_BF16
             ? ln_bwd_dispatch<bf16>(T, H, nullptr, x, gamma, mean, rstd, residual_grad, dx, dgamma, dbeta, ws, &pp, n,
                                     dy_out, dx_colsum, da, dz_out, st)
             : ln_bwd_dispatch<float>(T, H, nullptr, x, gamma, mean, rstd, residual_grad, dx, dgamma, dbeta, ws, &pp, n,
                                      dy_out, dx_colsum, da, dz_out, st);
}

// ------------------------------------------------------------------------------ combine (stand-in for g / f)
template <typename T>
__global__ __launch_bounds__(256) void combine_kernel(size_t nvec, size_t bias_vecs, PartialPtrs ptrs, int n,
                                                      const T* __restrict__ bias, const T* residual, T* out,
                                                      DropArgs drop) {
  constexpr int VN = Vec16<T>::N;
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= nvec) return;
  float acc[VN];
#pragma unroll
  for (int e = 0; e < VN; ++e) acc[e] = 0.f;
  for (int k = 0; k < n; ++k) {          // fixed order r = 0..n-1: deterministic
    Vec16<T> v;
    v.load((const T*)ptrs.p[k] + i * VN);
#pragma unroll
    for (int e = 0; e < VN; ++e) acc[e] += v.get(e);
  }
  if (bias) {
    Vec16<T> v;
    v.load(bias + (i % bias_vecs) * VN);             // bias_vecs = vectors of the [bias_rows, H] bias block
#pragma unroll
    for (int e = 0; e < VN; ++e) acc[e] += v.get(e);
  }
  if (drop.enabled) drop_apply<VN>(drop, i * VN, acc);
  if (residual) {
    Vec16<T> v;
    v.load(residual + i * VN);
#pragma unroll
    for (int e = 0; e < VN; ++e) acc[e] += v.get(e);
  }
  Vec16<T> o;
#pragma unroll
  for (int e = 0; e < VN; ++e) o.set(e, acc[e]);
  o.store(out + i * VN);
}

hipError_t launch_combine(int dtype, int T, int H, const void* const* partials, int n, const void* bias,
                          int bias_rows, const void* residual, void* out, const mlm_dropout* drop, hipStream_t st) {
  PartialPtrs pp;
  for (int k = 0; k < kMaxPartials; ++k) pp.p[k] = k < n ? partials[k] : nullptr;
  const DropArgs da = make_drop_args(drop);
  if (dtype == MLM_BF16) {
    const size_t nvec = (size_t)T * H / 8;
    hipLaunchKernelGGL((combine_kernel<bf16>), dim3((unsigned)((nvec + 255) / 256)), dim3(256), 0, st, nvec,
                       (size_t)bias_rows * H / 8, pp, n, (const bf16*)bias, (const bf16*)residual, (bf16*)out, da);
  } else {
    const size_t nvec = (size_t)T * H / 4;
    hipLaunchKernelGGL((combine_kernel<float>), dim3((unsigned)((nvec + 255) / 256)), dim3(256), 0, st, nvec,
                       (size_t)bias_rows * H / 4, pp, n, (const float*)bias, (const float*)residual, (float*)out, da);
  }
  return hipGetLastError();
}

// ------------------------------------------------------------------------------ column sums (bias gradients)
// Block = 64 vector-columns x 4 row-slices over kColsumRowsPerBlock rows; slices are summed through LDS in a fixed
// order, the chunk partial goes to the workspace and reduce_cols_kernel finishes.
template <typename T>
__global__ __launch_bounds__(256) void colsum_partial_kernel(int rows, int N, const T* __restrict__ dy,
                                                             float* __restrict__ ws) {
  constexpr int VN = Vec16<T>::N;
  __shared__ float red[4][64 * VN + 1];
  const int vx = threadIdx.x & 63, sl = threadIdx.x >> 6;
  const int ncb = (N / VN + 63) / 64;                 // column blocks; grid.x = chunks x column blocks (column block fastest)
  const int chunk = blockIdx.x / ncb;
  const int vcol = (blockIdx.x - chunk * ncb) * 64 + vx;
  const bool ok = vcol * VN < N;
  const int r0 = chunk * kColsumRowsPerBlock;
  const int r1 = min(rows, r0 + kColsumRowsPerBlock);
  float acc[VN];
#pragma unroll
  for (int e = 0; e < VN; ++e) acc[e] = 0.f;
  if (ok) {
#pragma unroll 4
    for (int r = r0 + sl; r < r1; r += 4) {
      Vec16<T> v;
      v.load(dy + (size_t)r * N + (size_t)vcol * VN);
#pragma unroll
      for (int e = 0; e < VN; ++e) acc[e] += v.get(e);
    }
  }
#pragma unroll
  for (int e = 0; e < VN; ++e) red[sl][e * 64 + vx] = acc[e];
  __syncthreads();
  if (sl == 0 && ok) {
#pragma unroll
    for (int e = 0; e < VN; ++e) {
      const float t = (red[0][e * 64 + vx] + red[1][e * 64 + vx]) + (red[2][e * 64 + vx] + red[3][e * 64 + vx]);
      ws[(size_t)chunk * N + (size_t)vcol * VN + e] = t;
    }
  }
}

static hipError_t colsum_impl(int dtype, int T, int N, const void* dy, void* dbias, float* ws, bool may_defer,
                              hipStream_t st) {
  const int nchunk = (T + kColsumRowsPerBlock - 1) / kColsumRowsPerBlock;
  float* deferred = may_defer ? deferred_reserve((size_t)nchunk * N) : nullptr;
  if (deferred) ws = deferred;
  if (dtype == MLM_BF16) {
    dim3 grid(((N / 8 + 63) / 64) * nchunk);
    hipLaunchKernelGGL((colsum_partial_kernel<bf16>), grid, dim3(256), 0, st, T, N, (const bf16*)dy, ws);
  } else {
    dim3 grid(((N / 4 + 63) / 64) * nchunk);
    hipLaunchKernelGGL((colsum_partial_kernel<float>), grid, dim3(256), 0, st, T, N, (const float*)dy, ws);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const ColReduce fin = {ws, dbias, dbias, dbias, nchunk, N, N, dtype};
  if (deferred) {
    deferred_record(fin);
    return hipSuccess;
  }
  return launch_reduce_cols(fin, st);
}

hipError_t launch_colsum(int dtype, int T, int N, const void* dy, void* dbias, float* ws, hipStream_t st) {
  return colsum_impl(dtype, T, N, dy, dbias, ws, true, st);
}

// ------------------------------------------------------------------------------ cross-entropy partials
// (max, sum-exp) pairs merge associatively: M = max(m_a, m_b), S = s_a e^{m_a-M} + s_b e^{m_b-M}.
__global__ __launch_bounds__(256) void ce_tile_merge_kernel(int T, int ntiles, const float* __restrict__ part_m,
                                                            const float* __restrict__ part_s,
                                                            const float* __restrict__ t_ws,
                                                            const int32_t* __restrict__ targets, int v0, int v1,
                                                            float* m_r, float* s_r, float* t_r) {
  // 32 tokens x 8 tile-slices per block; each slice merges its tiles online, slices are merged in a fixed order.
  __shared__ float sm[8][33], ss[8][33];
  const int tx = threadIdx.x & 31, sl = threadIdx.x >> 5;
  const int t = blockIdx.x * 32 + tx;
  float M = -INFINITY, S = 0.f;
  if (t < T) {
    for (int k = sl; k < ntiles; k += 8) {
      const float mk = part_m[(size_t)k * T + t], sk = part_s[(size_t)k * T + t];
      const float Mn = fmaxf(M, mk);
      if (Mn > -INFINITY) S = S * __expf(M - Mn) + sk * __expf(mk - Mn);
      M = Mn;
    }
  }
  sm[sl][tx] = M;
  ss[sl][tx] = S;
  __syncthreads();
  if (sl == 0 && t < T) {
    float Mt = -INFINITY;
#pragma unroll
    for (int k = 0; k < 8; ++k) Mt = fmaxf(Mt, sm[k][tx]);
    float St = 0.f;
#pragma unroll
    for (int k = 0; k < 8; ++k)
      if (sm[k][tx] > -INFINITY) St += ss[k][tx] * __expf(sm[k][tx] - Mt);
    m_r[t] = Mt;
    s_r[t] = St;
    const int tg = targets[t];
    t_r[t] = (tg >= v0 && tg < v1) ? t_ws[t] : 0.f;
  }
}

hipError_t launch_ce_tile_merge(int T, int ntiles, const float* part_m, const float* part_s, const float* t_ws,
                                const int32_t* targets, int v0, int v1, float* m_r, float* s_r, float* t_r,
                                hipStream_t st) {
  hipLaunchKernelGGL(ce_tile_merge_kernel, dim3((T + 31) / 32), dim3(256), 0, st, T, ntiles, part_m, part_s, t_ws,
                     targets, v0, v1, m_r, s_r, t_r);
  return hipGetLastError();
}

// fp32 path: row partials straight from stored logits, one block per token.
__global__ __launch_bounds__(256) void ce_rows_f32_kernel(int Vl, const float* __restrict__ logits,
                                                          const int32_t* __restrict__ targets, int v0,
                                                          float* m_r, float* s_r, float* t_r) {
  __shared__ float red[4];
  const int t = blockIdx.x;
  const float* row = logits + (size_t)t * Vl;
  float mx = -INFINITY;
  for (int j = threadIdx.x; j < Vl; j += 256) mx = fmaxf(mx, row[j]);
  mx = wave_max(mx);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  __syncthreads();
  float se = 0.f;
  for (int j = threadIdx.x; j < Vl; j += 256) se += expf(row[j] - mx);
  se = wave_sum(se);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = se;
  __syncthreads();
  if (threadIdx.x == 0) {
    m_r[t] = mx;
    s_r[t] = (red[0] + red[1]) + (red[2] + red[3]);
    const int loc = targets[t] - v0;
    t_r[t] = (loc >= 0 && loc < Vl) ? row[loc] : 0.f;
  }
}

hipError_t launch_ce_rows_f32(int T, int Vl, const float* logits, const int32_t* targets, int v0, float* m_r,
                              float* s_r, float* t_r, hipStream_t st) {
  hipLaunchKernelGGL(ce_rows_f32_kernel, dim3(T), dim3(256), 0, st, Vl, logits, targets, v0, m_r, s_r, t_r);
  return hipGetLastError();
}

// Merge over shards and the weighted mean: a single block (T is b*s, a few thousand) so that the loss is
// summed in a fixed order.
__global__ __launch_bounds__(1024) void ce_merge_kernel(int T, int n_shards, const float* __restrict__ m,
                                                        const float* __restrict__ s, const float* __restrict__ tl,
                                                        const float* __restrict__ loss_w, float* __restrict__ ce,
                                                        float* __restrict__ Mo, float* __restrict__ So,
                                                        float* __restrict__ loss_out, bool vec) {
  __shared__ float red_l[16], red_w[16];
  float accl = 0.f, accw = 0.f;
  // A thread takes four CONSECUTIVE tokens per step: with 16-byte loads (T a multiple of 4, 16-byte aligned buffers) a step is a handful of
  // independent loads in flight together instead of one round trip to memory per token and shard.
  auto load4 = [&](const float* base, int t0, float (&v)[4]) {
    if (vec) {
      const float4 x = *reinterpret_cast<const float4*>(base + t0);
      v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
    } else {
#pragma unroll
      for (int u = 0; u < 4; ++u) v[u] = base[min(t0 + u, T - 1)];
    }
  };
  // ... and two such groups per pass over the block (8192 tokens per pass), all of their loads issued before the
  // first use when there is one shard (then the merge is the identity and needs no second pass over the maxima)
  constexpr int G = 2;
  for (int base = 0; base < T; base += G * 4096) {
    float M[G][4], S[G][4], tt[G][4], w[G][4];
    int t0[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
      t0[g] = base + g * 4096 + 4 * threadIdx.x;
#pragma unroll
      for (int u = 0; u < 4; ++u) { M[g][u] = -INFINITY; S[g][u] = 0.f; tt[g][u] = 0.f; w[g][u] = 1.f; }
    }
    if (n_shards == 1) {
#pragma unroll
      for (int g = 0; g < G; ++g)
        if (t0[g] < T) {
          if (loss_w) load4(loss_w, t0[g], w[g]);
          load4(m, t0[g], M[g]);
          load4(s, t0[g], S[g]);
          load4(tl, t0[g], tt[g]);
        }
    } else {
#pragma unroll
      for (int g = 0; g < G; ++g) {
        if (t0[g] >= T) continue;
        if (loss_w) load4(loss_w, t0[g], w[g]);
        for (int r = 0; r < n_shards; ++r) {
          float mv[4];
          load4(m + (size_t)r * T, t0[g], mv);
#pragma unroll
          for (int u = 0; u < 4; ++u) M[g][u] = fmaxf(M[g][u], mv[u]);
        }
        for (int r = 0; r < n_shards; ++r) {           // second pass over the (cached) maxima
          float mv[4], sv[4], tv[4];
          load4(m + (size_t)r * T, t0[g], mv);
          load4(s + (size_t)r * T, t0[g], sv);
          load4(tl + (size_t)r * T, t0[g], tv);
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            S[g][u] += sv[u] * expf(mv[u] - M[g][u]);
            tt[g][u] += tv[u];
          }
        }
      }
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float c[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        c[u] = logf(S[g][u]) + M[g][u] - tt[g][u];
        if (t0[g] + u < T) {
          accl += w[g][u] * c[u];
          accw += w[g][u];
        }
      }
      if (vec) {                                       // T % 4 == 0: a group is inside [0, T) or outside
        if (t0[g] < T) {
          *reinterpret_cast<float4*>(ce + t0[g]) = make_float4(c[0], c[1], c[2], c[3]);
          *reinterpret_cast<float4*>(Mo + t0[g]) = make_float4(M[g][0], M[g][1], M[g][2], M[g][3]);
          *reinterpret_cast<float4*>(So + t0[g]) = make_float4(S[g][0], S[g][1], S[g][2], S[g][3]);
        }
      } else {
#pragma unroll
        for (int u = 0; u < 4; ++u)
          if (t0[g] + u < T) { ce[t0[g] + u] = c[u]; Mo[t0[g] + u] = M[g][u]; So[t0[g] + u] = S[g][u]; }
      }
    }
  }
  accl = wave_sum(accl);
  accw = wave_sum(accw);
  if ((threadIdx.x & 63) == 0) { red_l[threadIdx.x >> 6] = accl; red_w[threadIdx.x >> 6] = accw; }
  __syncthreads();
  if (threadIdx.x == 0) {
    float l = 0.f, w = 0.f;
    for (int k = 0; k < 16; ++k) { l += red_l[k]; w += red_w[k]; }
    loss_out[0] = l / w;
    loss_out[1] = w;
  }
}

hipError_t launch_ce_merge(int T, int n_shards, const float* m, const float* s, const float* t, const float* loss_w,
                           float* ce, float* M, float* S, float* loss_out, hipStream_t st) {
  auto a16 = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; };
  const bool vec = (T & 3) == 0 && a16(m) && a16(s) && a16(t) && a16(loss_w) && a16(ce) && a16(M) && a16(S);
  hipLaunchKernelGGL(ce_merge_kernel, dim3(1), dim3(1024), 0, st, T, n_shards, m, s, t, loss_w, ce, M, S, loss_out, vec);
  return hipGetLastError();
}

// dL = w_t / sum(w) * (exp(L - M_t) / S_t - onehot), written over the stored logits.
template <typename T>
__global__ __launch_bounds__(256) void dlogits_inplace_kernel(int Vl, T* logits, const int32_t* __restrict__ targets,
                                                              int v0, const float* __restrict__ M,
                                                              const float* __restrict__ S,
                                                              const float* __restrict__ loss_w,
                                                              const float* __restrict__ loss_stats) {
  constexpr int VN = Vec16<T>::N;
  const int ncb = (Vl / VN + 255) / 256;              // grid.x = tokens x column blocks (column block fastest)
  const int t = blockIdx.x / ncb;
  const int vcol = (blockIdx.x - t * ncb) * 256 + threadIdx.x;
  if (vcol * VN >= Vl) return;
  const float coef = (loss_w ? loss_w[t] : 1.0f) / loss_stats[1];
  const float Mt = M[t];
  const float inv = coef / S[t];
  const int loc = targets[t] - v0;
  T* p = logits + (size_t)t * Vl + (size_t)vcol * VN;
  Vec16<T> v, o;
  v.load(p);
#pragma unroll
  for (int e = 0; e < VN; ++e) {
    float g = __expf(v.get(e) - Mt) * inv;
    if (vcol * VN + e == loc) g -= coef;
    o.set(e, g);
  }
  o.store(p);
}

hipError_t launch_dlogits_inplace(int dtype, int T, int Vl, void* logits, const int32_t* targets, int v0,
                                  const float* M, const float* S, const float* loss_w, const float* loss_stats,
                                  hipStream_t st) {
  if (dtype == MLM_BF16) {
    dim3 grid(((Vl / 8 + 255) / 256) * T);
    hipLaunchKernelGGL((dlogits_inplace_kernel<bf16>), grid, dim3(256), 0, st, Vl, (bf16*)logits, targets, v0, M, S,
                       loss_w, loss_stats);
  } else {
    dim3 grid(((Vl / 4 + 255) / 256) * T);
    hipLaunchKernelGGL((dlogits_inplace_kernel<float>), grid, dim3(256), 0, st, Vl, (float*)logits, targets, v0, M, S,
                       loss_w, loss_stats);
  }
  return hipGetLastError();
}

// ------------------------------------------------------------------------------ row gather / scatter
// out[k, :] = x[idx[k], :] for k < n, zeros for n <= k < n_out (gather); out[idx[k], :] = y[k, :] and zeros in every
// other row (scatter; idx strictly increasing, so each output row has at most one source: found by binary search).
template <typename T>
__global__ __launch_bounds__(256) void rows_gather_kernel(int n, int n_out, int H, const int32_t* __restrict__ idx,
                                                          const T* __restrict__ x, T* __restrict__ out) {
  constexpr int VN = Vec16<T>::N;
  const int k = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (k >= n_out) return;
  const int lane = threadIdx.x & 63;
  const T* src = k < n ? x + (size_t)idx[k] * H : nullptr;
  for (int v = lane; v < H / VN; v += 64) {
    Vec16<T> t;
    if (src) t.load(src + (size_t)v * VN);
    else {
#pragma unroll
      for (int e = 0; e < VN; ++e) t.set(e, 0.f);
    }
    t.store(out + (size_t)k * H + (size_t)v * VN);
  }
}

template <typename T>
__global__ __launch_bounds__(256) void rows_scatter_kernel(int n, int rows, int H, const int32_t* __restrict__ idx,
                                                           const T* __restrict__ y, T* __restrict__ out) {
  constexpr int VN = Vec16<T>::N;
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= rows) return;
  const int lane = threadIdx.x & 63;
  int lo = 0, hi = n;                                  // first k with idx[k] >= r (wave-uniform search)
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (idx[mid] < r) lo = mid + 1; else hi = mid;
  }
  const T* src = (lo < n && idx[lo] == r) ? y + (size_t)lo * H : nullptr;
  for (int v = lane; v < H / VN; v += 64) {
    Vec16<T> t;
    if (src) t.load(src + (size_t)v * VN);
    else {
#pragma unroll
      for (int e = 0; e < VN; ++e) t.set(e, 0.f);
    }
    t.store(out + (size_t)r * H + (size_t)v * VN);
  }
}

hipError_t launch_rows_gather(int dtype, int n, int n_out, int H, const int32_t* idx, const void* x, void* out,
                              hipStream_t st) {
  dim3 grid((n_out + 3) / 4), block(256);
  if (dtype == MLM_BF16)
    hipLaunchKernelGGL((rows_gather_kernel<bf16>), grid, block, 0, st, n, n_out, H, idx, (const bf16*)x, (bf16*)out);
  else
    hipLaunchKernelGGL((rows_gather_kernel<float>), grid, block, 0, st, n, n_out, H, idx, (const float*)x, (float*)out);
  return hipGetLastError();
}

hipError_t launch_rows_scatter(int dtype, int n, int rows, int H, const int32_t* idx, const void* y, void* out,
                               hipStream_t st) {
  dim3 grid((rows + 3) / 4), block(256);
  if (dtype == MLM_BF16)
    hipLaunchKernelGGL((rows_scatter_kernel<bf16>), grid, block, 0, st, n, rows, H, idx, (const bf16*)y, (bf16*)out);
  else
    hipLaunchKernelGGL((rows_scatter_kernel<float>), grid, block, 0, st, n, rows, H, idx, (const float*)y, (float*)out);
  return hipGetLastError();
}

// delta[b, head, i] = sum_c dctx[t, head*d + c] * ctx[t, head*d + c]  (row sum of dP o P in the softmax gradient)
template <typename T>
__global__ __launch_bounds__(256) void attn_delta_kernel(int Tn, int hl, int d, int s, const T* __restrict__ ctx,
                                                         const T* __restrict__ dctx, float* __restrict__ delta) {
  constexpr int VN = Vec16<T>::N;
  const int idx = blockIdx.x * 256 + threadIdx.x;   // (t, head)
  if (idx >= Tn * hl) return;
  const int t = idx / hl, hd = idx % hl;
  const size_t off = (size_t)t * hl * d + (size_t)hd * d;
  float acc = 0.f;
  for (int c = 0; c < d; c += VN) {
    Vec16<T> a, g;
    a.load(ctx + off + c);
    g.load(dctx + off + c);
#pragma unroll
    for (int e = 0; e < VN; ++e) acc += a.get(e) * g.get(e);
  }
  const int bi = t / s, i = t % s;
  delta[((size_t)bi * hl + hd) * s + i] = acc;
}

hipError_t launch_attn_delta(int dtype, int T, int hl, int d, int b, int s, const void* ctx, const void* dctx,
                             float* delta, hipStream_t st) {
  (void)b;
  dim3 grid((T * hl + 255) / 256);
  if (dtype == MLM_BF16)
    hipLaunchKernelGGL((attn_delta_kernel<bf16>), grid, dim3(256), 0, st, T, hl, d, s, (const bf16*)ctx,
                       (const bf16*)dctx, delta);
  else
    hipLaunchKernelGGL((attn_delta_kernel<float>), grid, dim3(256), 0, st, T, hl, d, s, (const float*)ctx,
                       (const float*)dctx, delta);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------ column sums without a workspace
// For callers that cannot allocate (code under graph capture, serving loops): the chunk partials of the column sum
// live in a file-scope device array instead of a caller workspace.  Every GPU holds its own copy of the array at its
// own address until the process ends; the address is looked up once per device, with that device current, and host
// code uses only that looked-up pointer (the array's name is a host-side stand-in, not a device address).
static __device__ __align__(256) float scratch[kStaticScratchFloats];

static hipError_t static_scratch_ptr(float** out) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static float* per_device[kMaxDevices] = {};
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(mu);
  if (per_device[dev] == nullptr) {
    float* ptr = nullptr;
    e = hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (ptr == nullptr) return hipErrorInvalidSymbol;
    per_device[dev] = ptr;
  }
  *out = per_device[dev];
  return hipSuccess;
}

// Same kernels as launch_colsum, partials in the static array.  Every [chunk][column] slot that the reduction reads
// is written by the partial kernel of the same call first, so nothing has to start at zero and stale contents of an
// earlier (larger) call are never read.  The caller has checked ceil(T / kColsumRowsPerBlock) * N <= kStaticScratchFloats.
hipError_t launch_colsum_static(int dtype, int T, int N, const void* dy, void* dbias, hipStream_t st) {
  float* ws = nullptr;
  hipError_t e = static_scratch_ptr(&ws);
  if (e != hipSuccess) return e;
  return colsum_impl(dtype, T, N, dy, dbias, ws, false, st);     // always finishes inside the call
}

}  // namespace mlm
