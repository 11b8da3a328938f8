// Counter-based random numbers for dropout (gfx950).  The paper (Appendix B.2) asks for two streams -- one seeded
// identically on every model-parallel worker for the dropouts outside the model-parallel regions, one seeded uniquely
// per worker for the dropout inside the attention block -- and fixes neither generator nor seed rule.  This library
// uses Philox4x32-10 (Salmon et al., SC'11): stateless, so a kernel regenerates any element's random word from its
// index alone, in any order, on any lane.
//
// Element e (row-major index in the tensor the worker holds) of the site named by the 64-bit `offset` reads word
// e mod 4 of the block with counter (lo32(e / 4), hi32(e / 4), lo32(offset), hi32(offset)) under key
// (lo32(seed), hi32(seed)); it is KEPT iff that word >= thr = floor(p 2^32).  Kept values are scaled by 1 / (1 - p).
#pragma once
#include "common.h"

namespace mlm {


inline DropArgs make_drop_args(const mlm_dropout* d) {
  DropArgs a;
  a.k0 = a.k1 = a.off_lo = a.off_hi = a.thr = 0;
  a.scale = 1.0f;
  a.enabled = 0;
  if (d && d->p > 0.0f) {
    a.k0 = (uint32_t)(d->seed & 0xFFFFFFFFull);
    a.k1 = (uint32_t)(d->seed >> 32);
    a.off_lo = (uint32_t)(d->offset & 0xFFFFFFFFull);
    a.off_hi = (uint32_t)(d->offset >> 32);
    a.thr = (uint32_t)((double)d->p * 4294967296.0);   // floor: p < 1 and the product is exact in double
    a.scale = 1.0f / (1.0f - d->p);
    a.enabled = 1;
  }
  return a;
}

struct U32x4 { uint32_t w[4]; };

__device__ __forceinline__ U32x4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                               uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    if (r) { k0 += 0x9E3779B9u; k1 += 0xBB67AE85u; }
    const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
    c0 = hi1 ^ c1 ^ k0;
    c1 = lo1;
    c2 = hi0 ^ c3 ^ k1;
    c3 = lo0;
  }
  U32x4 o;
  o.w[0] = c0; o.w[1] = c1; o.w[2] = c2; o.w[3] = c3;
  return o;
}

// The four random words of the block holding elements 4 blk .. 4 blk + 3 of the site.
__device__ __forceinline__ U32x4 drop_block(const DropArgs& d, uint64_t blk) {
  return philox4x32_10((uint32_t)blk, (uint32_t)(blk >> 32), d.off_lo, d.off_hi, d.k0, d.k1);
}

// 4-bit keep mask (bit i = element 4 blk + i is kept).
__device__ __forceinline__ uint32_t drop_keep4(const DropArgs& d, uint64_t blk) {
  const U32x4 w = drop_block(d, blk);
  return (w.w[0] >= d.thr ? 1u : 0u) | (w.w[1] >= d.thr ? 2u : 0u) | (w.w[2] >= d.thr ? 4u : 0u) |
         (w.w[3] >= d.thr ? 8u : 0u);
}

// Inverted dropout of the N consecutive elements starting at element index e0 (a multiple of 4; N = 4 or 8).
template <int N>
__device__ __forceinline__ void drop_apply(const DropArgs& d, uint64_t e0, float (&v)[N]) {
  static_assert(N % 4 == 0, "whole blocks");
#pragma unroll
  for (int b = 0; b < N / 4; ++b) {
    const uint32_t k = drop_keep4(d, (e0 >> 2) + b);
#pragma unroll
    for (int i = 0; i < 4; ++i) v[4 * b + i] = ((k >> i) & 1u) ? v[4 * b + i] * d.scale : 0.f;
  }
}

}  // namespace mlm
