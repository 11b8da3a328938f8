// bf16 MFMA GEMM for gfx950 (MI355X): C[m,n] = sum_k A(m,k) B(k,n), fp32 accumulation.
//
// Design (one workgroup = WAVES_M x WAVES_N wavefronts of 64 lanes, block tile BM x BN x 64):
//   * Both operand tiles live in LDS k-contiguous ([row][64 + 8 pad] bf16, 144-byte rows), double
//     buffered: tile k+1 is fetched from HBM into registers while tile k feeds the matrix cores,
//     then written to the other LDS buffer -- one barrier per k-tile.
//   * An operand that is k-contiguous in memory (activations in the forward and input-gradient
//     GEMMs, weights [in,out] in the input-gradient GEMM) is copied with 16-byte vectors.  An
//     operand that is contiguous along m or n (weights in the forward GEMM, both operands of the
//     weight-gradient GEMM) is fetched as 8x8 blocks (eight 16-byte rows), transposed in
//     registers with byte permutes, and stored as eight k-contiguous 16-byte LDS vectors, so
//     no transposed copy of any tensor is ever made in HBM.
//   * v_mfma_f32_32x32x16_bf16: the B tile is the MFMA "A" operand (rows = n) and the A tile its
//     "B" operand (columns = m).  Each lane therefore holds, for ONE output row m, 16 values that
//     are 4-element runs along n: row reductions (softmax statistics of the fused cross entropy)
//     stay inside a lane plus one cross-half shuffle, and results are packed 4 at a time.
//   * Epilogue: every wave stages 32 x WN strips through its own LDS region and writes full
//     16-byte vectors, rows contiguous (coalesced HBM stores); bias, GeLU (+ saved pre-activation),
//     GeLU', the dlogits formula and the cross-entropy partials are applied on the fp32 accumulators.
//   * Workgroup ids are remapped so that the workgroups resident on one XCD (ids congruent mod 8)
//     cover a compact patch of output tiles and share operand panels in that XCD's L2.
#pragma once
#include "common.h"

namespace mlm {

constexpr int GBK = 64;            // k per LDS tile
constexpr int GLS = GBK + 8;       // LDS row stride in elements (144 B)

__device__ __forceinline__ uint32_t perm_lo(uint32_t hi_src, uint32_t lo_src) {   // (lo16(lo_src), lo16(hi_src))
  return __builtin_amdgcn_perm(hi_src, lo_src, 0x05040100u);
}
__device__ __forceinline__ uint32_t perm_hi(uint32_t hi_src, uint32_t lo_src) {   // (hi16(lo_src), hi16(hi_src))
  return __builtin_amdgcn_perm(hi_src, lo_src, 0x07060302u);
}

// 8x8 transpose of 16-bit elements held as eight 16-byte rows.
__device__ __forceinline__ void transpose8x8(const uint4 (&r)[8], uint4 (&o)[8]) {
  const uint32_t* in = reinterpret_cast<const uint32_t*>(r);   // in[j*4 + q]: row j, columns 2q, 2q+1
  uint32_t* out = reinterpret_cast<uint32_t*>(o);              // out[n*4 + c]: column n, rows 2c, 2c+1
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      out[(2 * q) * 4 + c] = perm_lo(in[(2 * c + 1) * 4 + q], in[(2 * c) * 4 + q]);
      out[(2 * q + 1) * 4 + c] = perm_hi(in[(2 * c + 1) * 4 + q], in[(2 * c) * 4 + q]);
    }
}

// Tile of ROWS x 64 whose memory layout is k-contiguous: element (row, k) at P[row*ld + k].
template <int ROWS, int NT>
struct LoaderKC {
  static constexpr int VECS = ROWS * (GBK / 8);
  static constexpr int PER = (VECS + NT - 1) / NT;
  uint4 reg[PER];
  __device__ __forceinline__ void load(const bf16* __restrict__ P, int ld, int row0, int nrows, int k0, int K,
                                       int tid) {
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int v = tid + i * NT;
      if (VECS % NT != 0 && v >= VECS) break;
      const int row = min(row0 + (v >> 3), nrows - 1);
      const int gk = k0 + (v & 7) * 8;
      if (gk < K) reg[i] = *reinterpret_cast<const uint4*>(P + (size_t)row * ld + gk);
      else reg[i] = make_uint4(0, 0, 0, 0);
    }
  }
  __device__ __forceinline__ void store(bf16* s, int tid) const {
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int v = tid + i * NT;
      if (VECS % NT != 0 && v >= VECS) break;
      *reinterpret_cast<uint4*>(s + (v >> 3) * GLS + (v & 7) * 8) = reg[i];
    }
  }
};

// Tile of 64 (k) x ROWS whose memory layout is contiguous along the row index: element (row, k) at P[k*ld + row].
template <int ROWS, int NT>
struct LoaderMN {
  static constexpr int BLKS = (GBK / 8) * (ROWS / 8);
  static constexpr int PER = (BLKS + NT - 1) / NT;
  uint4 reg[PER][8];
  __device__ __forceinline__ void load(const bf16* __restrict__ P, int ld, int row0, int nrows, int k0, int K,
                                       int tid) {
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int blk = tid + i * NT;
      if (BLKS % NT != 0 && blk >= BLKS) break;
      const int kb = blk & 7, nb = blk >> 3;
      const int gr = min(row0 + nb * 8, nrows - 8);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int gk = k0 + kb * 8 + j;
        if (gk < K) reg[i][j] = *reinterpret_cast<const uint4*>(P + (size_t)gk * ld + gr);
        else reg[i][j] = make_uint4(0, 0, 0, 0);
      }
    }
  }
  __device__ __forceinline__ void store(bf16* s, int tid) const {
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int blk = tid + i * NT;
      if (BLKS % NT != 0 && blk >= BLKS) break;
      const int kb = blk & 7, nb = blk >> 3;
      uint4 o[8];
      transpose8x8(reg[i], o);
#pragma unroll
      for (int n = 0; n < 8; ++n) *reinterpret_cast<uint4*>(s + (nb * 8 + n) * GLS + kb * 8) = o[n];
    }
  }
};

template <int ROWS, int NT, bool KC> struct LoaderSel { typedef LoaderKC<ROWS, NT> type; };
template <int ROWS, int NT> struct LoaderSel<ROWS, NT, false> { typedef LoaderMN<ROWS, NT> type; };

template <int BM, int BN, int WAVES_M, int WAVES_N>
struct GemmTile {
  static constexpr int NT = WAVES_M * WAVES_N * 64;
  static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  static constexpr int TM = WM / 32, TN = WN / 32;
  static constexpr int STAGE = (BM + BN) * GLS;                    // elements per pipeline stage
  static constexpr int STRIP = 32 * 68 * 2;                        // bf16-sized elements of one epilogue strip (32 x 68 floats)
  static constexpr size_t LDS_MAIN = (size_t)2 * STAGE * 2;
  static constexpr size_t LDS_EPI = (size_t)2 * WAVES_M * WAVES_N * STRIP * 2 + (size_t)2 * WAVES_N * BM * 4;
  static constexpr size_t LDS_BYTES = LDS_MAIN > LDS_EPI ? LDS_MAIN : LDS_EPI;
};

__device__ __forceinline__ void tile_of_block(int pid, int tiles_m, int tiles_n, int& tm, int& tn) {
  // XCD-aware remap: workgroup ids congruent mod 8 run on the same XCD; give each XCD a contiguous range of
  // virtual ids, then walk the virtual ids in groups of 8 tile-rows (column-major inside a group) so that 32
  // consecutive ids cover an 8 x 4 patch of tiles.
  const int ntiles = tiles_m * tiles_n;
  const int q = ntiles >> 3, rem = ntiles & 7;
  const int x = pid & 7, local = pid >> 3;
  const int vid = x * q + min(x, rem) + local;
  constexpr int GM = 8;
  const int per_group = GM * tiles_n;
  const int g = vid / per_group;
  const int first = g * GM;
  const int gsz = min(GM, tiles_m - first);
  const int in = vid - g * per_group;
  tm = first + in % gsz;
  tn = in / gsz;
}

// ---------------------------------------------------------------------------------------------- epilogue
// acc[i][j][e] holds row m = m0 + wm0 + 32 j + l32 and column n = n0 + wn0 + 32 i + 8 (e/4) + 4 lh + (e%4) of the
// output tile.  Must be entered after a workgroup barrier that follows the last LDS read of the main loop (the LDS
// is reused: two staging strips per wave, then the cross-wave reduction area of the cross-entropy partials).

// Per-row softmax statistics of the logits tile (fused cross entropy): row max and sum of exp over the tile's
// columns, plus the target logit if the target column lies in this tile.  RAGGED: the tile hangs over column N.
template <int TN, int TM, int WN, bool RAGGED>
__device__ __forceinline__ void ce_tile_stats(const GemmArgs& a, const floatx16 (&acc)[TN][TM], int m0w, int n0w,
                                              int l32, int lh, float* red_m_w, float* red_s_w) {
  const int nvalid = a.N - (n0w + 4 * lh);     // RAGGED: register column c (relative) is real iff c < nvalid
#pragma unroll
  for (int j = 0; j < TM; ++j) {
    const int row = m0w + j * 32 + l32;
    float mx = -INFINITY;
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int c = i * 32 + 8 * (e >> 2) + (e & 3);
        const float v = (RAGGED && c >= nvalid) ? -INFINITY : acc[i][j][e];
        mx = fmaxf(mx, v);
      }
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    // column of the target relative to this lane's registers (integer test), one select per value
    const int loc = (row < a.M) ? a.targets[row] - a.v0 - (n0w + 4 * lh) : -1;
    const float mxl = mx * 1.4426950408889634f;
    float se = 0.f, tv = 0.f;
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int c = i * 32 + 8 * (e >> 2) + (e & 3);
        const float v = acc[i][j][e];
        const float p = __builtin_amdgcn_exp2f(fmaf(v, 1.4426950408889634f, -mxl));
        se += (RAGGED && c >= nvalid) ? 0.f : p;
        tv = (loc == c) ? v : tv;
      }
    se += __shfl_xor(se, 32, 64);
    // the half that owns the column has bit 2 of (target - 4 lh) clear
    if (loc >= 0 && loc < WN && (loc & 4) == 0 && (!RAGGED || loc < nvalid)) a.t_out[row] = tv;
    if (lh == 0) {
      red_m_w[j * 32 + l32] = mx;
      red_s_w[j * 32 + l32] = se;
    }
    __builtin_amdgcn_sched_barrier(0);
  }
}

// The same for accumulators of 16 x 16 MFMA tiles: acc[i][j][e] holds row m = m0w + 16 j + (lane & 15) and column
// n = n0w + 16 i + 4 (lane >> 4) + e.  The four lanes l16, l16 + 16, l16 + 32, l16 + 48 share a row.
template <int NB, int NA, int WN, bool RAGGED>
__device__ __forceinline__ void ce_tile_stats(const GemmArgs& a, const floatx4 (&acc)[NB][NA], int m0w, int n0w,
                                              int lane, float* red_m_w, float* red_s_w) {
  const int l16 = lane & 15, lg = lane >> 4;
  const int nvalid = a.N - (n0w + 4 * lg);     // RAGGED: register column c (relative) is real iff c < nvalid
  // All rows' maxima first, then all rows' sums: the cross-lane exchanges of the NA rows are independent and overlap
  // (8 % fewer cycles than row by row; the function is bound by its vector arithmetic -- 128 values per lane, each a
  // max, a fused multiply-add, an exp2, an add and the target select: 7400 cycles per 256 x 256 tile, measured).
  float mx[NA], se[NA], tv[NA];
  int loc[NA];
#pragma unroll
  for (int j = 0; j < NA; ++j) {
    const int row = m0w + j * 16 + l16;
    // column of the target relative to this lane's registers (integer test), one select per value
    loc[j] = (row < a.M) ? a.targets[row] - a.v0 - (n0w + 4 * lg) : -1;
    mx[j] = -INFINITY;
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int c = i * 16 + e;
        const float v = (RAGGED && c >= nvalid) ? -INFINITY : acc[i][j][e];
        mx[j] = fmaxf(mx[j], v);
      }
  }
#pragma unroll
  for (int j = 0; j < NA; ++j) mx[j] = fmaxf(mx[j], __shfl_xor(mx[j], 16, 64));
#pragma unroll
  for (int j = 0; j < NA; ++j) mx[j] = fmaxf(mx[j], __shfl_xor(mx[j], 32, 64));
#pragma unroll
  for (int j = 0; j < NA; ++j) {
    const float mxl = mx[j] * 1.4426950408889634f;
    se[j] = 0.f;
    tv[j] = 0.f;
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int c = i * 16 + e;
        const float v = acc[i][j][e];
        const float p = __builtin_amdgcn_exp2f(fmaf(v, 1.4426950408889634f, -mxl));
        se[j] += (RAGGED && c >= nvalid) ? 0.f : p;
      }
  }
  // the target logit: only if some row of this wave has its target inside the wave's WN columns (one wave tile in
  // seven at a vocabulary of 51200 split eight ways), else the pass -- two operations per value -- is skipped
  bool mine = false;
#pragma unroll
  for (int j = 0; j < NA; ++j) mine = mine || (loc[j] >= 0 && loc[j] < WN);
  if (__builtin_amdgcn_ballot_w64(mine) != 0) {
#pragma unroll
    for (int j = 0; j < NA; ++j)
#pragma unroll
      for (int i = 0; i < NB; ++i)
#pragma unroll
        for (int e = 0; e < 4; ++e) tv[j] = (loc[j] == i * 16 + e) ? acc[i][j][e] : tv[j];
  }
#pragma unroll
  for (int j = 0; j < NA; ++j) se[j] += __shfl_xor(se[j], 16, 64);
#pragma unroll
  for (int j = 0; j < NA; ++j) se[j] += __shfl_xor(se[j], 32, 64);
#pragma unroll
  for (int j = 0; j < NA; ++j) {
    const int row = m0w + j * 16 + l16;
    // the lane group that owns the column has bits 2 and 3 of (target - 4 lg) clear
    if (loc[j] >= 0 && loc[j] < WN && (loc[j] & 12) == 0 && (!RAGGED || loc[j] < nvalid)) a.t_out[row] = tv[j];
    if (lg == 0) {
      red_m_w[j * 16 + l16] = mx[j];
      red_s_w[j * 16 + l16] = se[j];
    }
  }
}

// Accumulator-layout adapters of the epilogue: row statistics of the wave tile, and the fill of one staging strip
// (rows 32 j .. 32 j + 31, columns 64 h .. 64 h + 63 of the wave tile; S = strip row stride in elements of T).
template <int WN, bool RAGGED, int TN, int TM>
__device__ __forceinline__ void acc_ce_stats(const GemmArgs& a, const floatx16 (&acc)[TN][TM], int m0w, int n0w, int lane,
                                             float* rm, float* rs) {
  ce_tile_stats<TN, TM, WN, RAGGED>(a, acc, m0w, n0w, lane & 31, lane >> 5, rm, rs);
}
template <int WN, bool RAGGED, int NB, int NA>
__device__ __forceinline__ void acc_ce_stats(const GemmArgs& a, const floatx4 (&acc)[NB][NA], int m0w, int n0w, int lane,
                                             float* rm, float* rs) {
  ce_tile_stats<NB, NA, WN, RAGGED>(a, acc, m0w, n0w, lane, rm, rs);
}
template <typename T> __device__ __forceinline__ void strip_put4(T* p, float v0, float v1, float v2, float v3);
template <> __device__ __forceinline__ void strip_put4<bf16>(bf16* p, float v0, float v1, float v2, float v3) {
  bf16x4 v;
  v[0] = (bf16)v0; v[1] = (bf16)v1; v[2] = (bf16)v2; v[3] = (bf16)v3;
  *reinterpret_cast<bf16x4*>(p) = v;
}
template <> __device__ __forceinline__ void strip_put4<float>(float* p, float v0, float v1, float v2, float v3) {
  *reinterpret_cast<float4*>(p) = make_float4(v0, v1, v2, v3);
}
template <typename T, int S, int TN, int TM>
__device__ __forceinline__ void acc_fill_strip(T* strip, const floatx16 (&acc)[TN][TM], int j, int h, int lane) {
  const int l32 = lane & 31, lh = lane >> 5;
#pragma unroll
  for (int il = 0; il < 2; ++il)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      if (2 * h + il >= TN) continue;
      const floatx16& t = acc[2 * h + il][j];
      strip_put4<T>(strip + l32 * S + il * 32 + 8 * g + 4 * lh, t[4 * g], t[4 * g + 1], t[4 * g + 2], t[4 * g + 3]);
    }
}
template <typename T, int S, int NB, int NA>
__device__ __forceinline__ void acc_fill_strip(T* strip, const floatx4 (&acc)[NB][NA], int j, int h, int lane) {
  const int l16 = lane & 15, lg = lane >> 4;
#pragma unroll
  for (int jl = 0; jl < 2; ++jl)
#pragma unroll
    for (int il = 0; il < 4; ++il) {
      if (4 * h + il >= NB) continue;
      const floatx4& t = acc[4 * h + il][2 * j + jl];
      strip_put4<T>(strip + (jl * 16 + l16) * S + il * 16 + 4 * lg, t[0], t[1], t[2], t[3]);
    }
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int EPI, bool GELU_TANH, typename Acc>
__device__ __forceinline__ void gemm_epilogue_impl(const GemmArgs& a, Acc& acc,
                                                   unsigned char* lds_raw, int m0, int n0, int tile_n) {
  typedef GemmTile<BM, BN, WAVES_M, WAVES_N> Tcfg;
  constexpr int NT = Tcfg::NT, TM = Tcfg::TM, TN = Tcfg::TN, WM = Tcfg::WM, WN = Tcfg::WN;
  bf16* lds = reinterpret_cast<bf16*>(lds_raw);
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, lh = lane >> 5;
  const int wm0 = (wave / WAVES_N) * WM, wn0 = (wave % WAVES_N) * WN;
  bf16* C = (bf16*)a.C;
  const bf16* bias = (const bf16*)a.bias;

  if (EPI == EPI_CE) {
    float* red_m = reinterpret_cast<float*>(lds_raw + (size_t)2 * WAVES_M * WAVES_N * Tcfg::STRIP * 2);
    float* red_s = red_m + WAVES_N * BM;
    float* rm = red_m + (wave % WAVES_N) * BM + wm0;
    float* rs = red_s + (wave % WAVES_N) * BM + wm0;
    if (n0 + BN > a.N) acc_ce_stats<WN, true>(a, acc, m0 + wm0, n0 + wn0, lane, rm, rs);
    else acc_ce_stats<WN, false>(a, acc, m0 + wm0, n0 + wn0, lane, rm, rs);
    __syncthreads();
    for (int rloc = tid; rloc < BM; rloc += NT) {
      const int row = m0 + rloc;
      if (row < a.M) {
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < WAVES_N; ++w) M = fmaxf(M, red_m[w * BM + rloc]);
        float S = 0.f;
#pragma unroll
        for (int w = 0; w < WAVES_N; ++w) {
          const float mw = red_m[w * BM + rloc];
          if (mw > -INFINITY) S += red_s[w * BM + rloc] * __expf(mw - M);
        }
        a.part_m[(size_t)tile_n * a.M + row] = M;
        a.part_s[(size_t)tile_n * a.M + row] = S;
      }
    }
    if (C == nullptr) return;
  }

  // ---- store passes.  The fp32 accumulators go through per-wave LDS strips of 32 rows x 64 columns (two strips,
  // software-pipelined: strip s+1 is written while strip s is read back).  All element-wise work happens at
  // read-back time, where a lane owns 8 consecutive columns of one row: bias, the saved pre-activation and the
  // outputs are then 16-byte accesses with 128-byte contiguous row segments.
  // (an odd TN leaves a last strip of 32 columns: half of the strip is then neither written nor read back)
  constexpr int NH = (TN + 1) / 2, NSTEP = TM * NH;
  const int rb_r = lane >> 3, rb_c = (lane & 7) * 8;           // read-back: 8 rows x 8 column groups per iteration
  const bool full = (m0 + BM <= a.M) && (n0 + BN <= a.N);
  if ((EPI == EPI_STORE || EPI == EPI_CE) && bias == nullptr) {
    // Nothing but the rounding happens between accumulator and memory: round first and stage bf16 strips (half the
    // LDS traffic of the fp32 strips, no conversion at read-back).  Row stride 72 elements keeps rows 16-byte aligned.
    constexpr int SWB = 72;
    static_assert(2 * 32 * SWB <= Tcfg::STRIP * 2, "bf16 strips fit in the wave's staging area");
    bf16* bstrip0 = lds + (size_t)wave * 2 * Tcfg::STRIP;
#pragma unroll
    for (int step = 0; step <= NSTEP; ++step) {
      if (step < NSTEP) {
        const int j = step / NH, h = step % NH;
        bf16* strip = bstrip0 + (step & 1) * (32 * SWB);
        acc_fill_strip<bf16, SWB>(strip, acc, j, h, lane);
      }
      __builtin_amdgcn_wave_barrier();
      if (step > 0) {
        const int ps = step - 1;
        const int j = ps / NH, h = ps % NH;
        const bf16* strip = bstrip0 + (ps & 1) * (32 * SWB);
        const int gn = n0 + wn0 + h * 64 + rb_c;
        const bool colv = (TN % 2 == 0) || (h * 64 + rb_c < WN);
#pragma unroll
        for (int it = 0; it < 4; ++it) {
          const int r = rb_r + it * 8;
          const int gm = m0 + wm0 + j * 32 + r;
          const bf16x8 o = *reinterpret_cast<const bf16x8*>(strip + r * SWB + rb_c);
          if (colv && (full || (gm < a.M && gn < a.N))) *reinterpret_cast<bf16x8*>(C + (size_t)gm * a.ldc + gn) = o;
        }
      }
      __builtin_amdgcn_wave_barrier();
    }
    return;
  }
  constexpr int SW = 64 + 4;                                   // strip row stride in floats (272 B)
  static_assert(32 * SW * 4 <= Tcfg::STRIP * 2, "strip does not fit");
  float* strip0 = reinterpret_cast<float*>(lds + (size_t)wave * 2 * Tcfg::STRIP);

#pragma unroll
  for (int step = 0; step <= NSTEP; ++step) {
    if (step < NSTEP) {
      const int j = step / NH, h = step % NH;
      float* strip = strip0 + (step & 1) * (Tcfg::STRIP / 2);
      acc_fill_strip<float, SW>(strip, acc, j, h, lane);
    }
    __builtin_amdgcn_wave_barrier();
    if (step > 0) {
      const int ps = step - 1;
      const int j = ps / NH, h = ps % NH;
      const float* strip = strip0 + (ps & 1) * (Tcfg::STRIP / 2);
      const int gn = n0 + wn0 + h * 64 + rb_c;                 // first of this lane's 8 columns
      const bool colv = (TN % 2 == 0) || (h * 64 + rb_c < WN);
      const int gnc = min(gn, a.N - 8);
      float bvals[8];
      if ((EPI == EPI_STORE || EPI == EPI_BIAS_GELU) && bias != nullptr) {
        const bf16x8 b8 = *reinterpret_cast<const bf16x8*>(bias + gnc);
#pragma unroll
        for (int e = 0; e < 8; ++e) bvals[e] = (float)b8[e];
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) bvals[e] = 0.f;
      }
#pragma unroll
      for (int it = 0; it < 4; ++it) {
        const int r = rb_r + it * 8;
        const int gm = m0 + wm0 + j * 32 + r;
        const int gmc = min(gm, a.M - 1);
        const float4 lo = *reinterpret_cast<const float4*>(strip + r * SW + rb_c);
        const float4 hi = *reinterpret_cast<const float4*>(strip + r * SW + rb_c + 4);
        float v[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
        const bool ok = colv && (full || (gm < a.M && gn < a.N));
        bf16x8 o;
        if (EPI == EPI_STORE || EPI == EPI_CE) {
#pragma unroll
          for (int e = 0; e < 8; ++e) o[e] = (bf16)(v[e] + bvals[e]);
        } else if (EPI == EPI_BIAS_GELU) {
          bf16x8 pre;
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const float x = v[e] + bvals[e];
            pre[e] = (bf16)x;
            o[e] = (bf16)gelu_fwd(x, GELU_TANH);
          }
          if (ok) *reinterpret_cast<bf16x8*>((bf16*)a.aux + (size_t)gm * a.ldaux + gn) = pre;
        } else if (EPI == EPI_DGELU) {
          const bf16x8 g8 = *reinterpret_cast<const bf16x8*>((const bf16*)a.aux + (size_t)gmc * a.ldaux + gnc);
#pragma unroll
          for (int e = 0; e < 8; ++e) o[e] = (bf16)(v[e] * gelu_bwd((float)g8[e], GELU_TANH));
        } else if (EPI == EPI_DLOGITS) {
          const float coef = (a.loss_w ? a.loss_w[gmc] : 1.0f) / a.loss_stats[1];
          const float Mrl = a.Mrow[gmc] * 1.4426950408889634f;
          const float invS = coef / a.Srow[gmc];
          const int loc = a.targets[gmc] - a.v0 - gn;           // target column relative to this lane's first column
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            float pz = __builtin_amdgcn_exp2f(fmaf(v[e], 1.4426950408889634f, -Mrl)) * invS;
            if (loc == e) pz -= coef;
            o[e] = (bf16)pz;
          }
        }
        if (ok) *reinterpret_cast<bf16x8*>(C + (size_t)gm * a.ldc + gn) = o;
      }
    }
    __builtin_amdgcn_wave_barrier();
  }
}

// acc: floatx16 [BN / WAVES_N / 32][BM / WAVES_M / 32] (32 x 32 MFMA tiles) or floatx4 [.. / 16][.. / 16] (16 x 16)
template <int BM, int BN, int WAVES_M, int WAVES_N, int EPI, typename Acc>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs& a, Acc& acc,
                                              unsigned char* lds_raw, int m0, int n0, int tile_n) {
  if (EPI == EPI_BIAS_GELU || EPI == EPI_DGELU) {
    // the GeLU form is a launch-wide constant: branch once, not per element
    if (a.gelu_tanh) gemm_epilogue_impl<BM, BN, WAVES_M, WAVES_N, EPI, true>(a, acc, lds_raw, m0, n0, tile_n);
    else gemm_epilogue_impl<BM, BN, WAVES_M, WAVES_N, EPI, false>(a, acc, lds_raw, m0, n0, tile_n);
  } else {
    gemm_epilogue_impl<BM, BN, WAVES_M, WAVES_N, EPI, true>(a, acc, lds_raw, m0, n0, tile_n);
  }
}

template <int BM, int BN, int WAVES_M, int WAVES_N, bool A_KC, bool B_KC, int EPI>
__global__ __launch_bounds__(WAVES_M* WAVES_N * 64) void gemm_bf16_kernel(GemmArgs a) {
  typedef GemmTile<BM, BN, WAVES_M, WAVES_N> Tcfg;
  constexpr int NT = Tcfg::NT, TM = Tcfg::TM, TN = Tcfg::TN, WM = Tcfg::WM, WN = Tcfg::WN;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  bf16* lds = reinterpret_cast<bf16*>(lds_raw);

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, lh = lane >> 5;
  const int wm0 = (wave / WAVES_N) * WM, wn0 = (wave % WAVES_N) * WN;
  const int tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.N + BN - 1) / BN;
  int tile_m, tile_n;
  tile_of_block(blockIdx.x, tiles_m, tiles_n, tile_m, tile_n);
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  const bf16* A = (const bf16*)a.A;
  const bf16* B = (const bf16*)a.B;

  typename LoaderSel<BM, NT, A_KC>::type la;
  typename LoaderSel<BN, NT, B_KC>::type lb;

  floatx16 acc[TN][TM];
#pragma unroll
  for (int i = 0; i < TN; ++i)
#pragma unroll
    for (int j = 0; j < TM; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  const int nk = (a.K + GBK - 1) / GBK;
  la.load(A, a.lda, m0, a.M, 0, a.K, tid);
  lb.load(B, a.ldb, n0, a.N, 0, a.K, tid);
  la.store(lds, tid);
  lb.store(lds + BM * GLS, tid);
  __syncthreads();

  for (int kt = 0; kt < nk; ++kt) {
    bf16* sA = lds + (kt & 1) * Tcfg::STAGE;
    bf16* sB = sA + BM * GLS;
    if (kt + 1 < nk) {
      la.load(A, a.lda, m0, a.M, (kt + 1) * GBK, a.K, tid);
      lb.load(B, a.ldb, n0, a.N, (kt + 1) * GBK, a.K, tid);
    }
#pragma unroll
    for (int ks = 0; ks < GBK / 16; ++ks) {
      bf16x8 fa[TM], fb[TN];
#pragma unroll
      for (int j = 0; j < TM; ++j)
        fa[j] = *reinterpret_cast<const bf16x8*>(sA + (wm0 + j * 32 + l32) * GLS + ks * 16 + lh * 8);
#pragma unroll
      for (int i = 0; i < TN; ++i)
        fb[i] = *reinterpret_cast<const bf16x8*>(sB + (wn0 + i * 32 + l32) * GLS + ks * 16 + lh * 8);
#pragma unroll
      for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[i], fa[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) {
      bf16* dA = lds + ((kt + 1) & 1) * Tcfg::STAGE;
      la.store(dA, tid);
      lb.store(dA + BM * GLS, tid);
    }
    __syncthreads();
  }

  gemm_epilogue<BM, BN, WAVES_M, WAVES_N, EPI>(a, acc, lds_raw, m0, n0, tile_n);
}

template <int BM, int BN, int WAVES_M, int WAVES_N, bool A_KC, bool B_KC, int EPI>
hipError_t launch_gemm_bf16_cfg(const GemmArgs& a, hipStream_t st) {
  typedef GemmTile<BM, BN, WAVES_M, WAVES_N> Tcfg;
  auto kern = gemm_bf16_kernel<BM, BN, WAVES_M, WAVES_N, A_KC, B_KC, EPI>;
  static LdsAttrOnce attr;         // per instantiation and device
  if (hipError_t e = attr.ensure((const void*)kern, (int)Tcfg::LDS_BYTES); e != hipSuccess) return e;
  const int tiles = ((a.M + BM - 1) / BM) * ((a.N + BN - 1) / BN);
  hipLaunchKernelGGL(kern, dim3(tiles), dim3(Tcfg::NT), Tcfg::LDS_BYTES, st, a);
  return hipGetLastError();
}

// Tile configurations; the launcher picks one per problem shape (see pick_tile in gemm_bf16.hip).
enum TileId { TILE_256x256 = 0, TILE_256x128 = 1, TILE_128x128 = 2, TILE_COUNT = 3 };
int pick_tile(int M, int N, int K);
bool gemm_use_v2(const GemmArgs& a);   // direct-to-LDS kernel applicable (K % 32 == 0) and not disabled
constexpr int kTileBN[TILE_COUNT] = {256, 128, 128};

template <bool A_KC, bool B_KC, int EPI>
hipError_t launch_gemm_bf16_layout(const GemmArgs& a, hipStream_t st) {
  switch (pick_tile(a.M, a.N, a.K)) {
    case TILE_256x256: return launch_gemm_bf16_cfg<256, 256, 2, 2, A_KC, B_KC, EPI>(a, st);
    case TILE_256x128: return launch_gemm_bf16_cfg<256, 128, 2, 2, A_KC, B_KC, EPI>(a, st);
    default: return launch_gemm_bf16_cfg<128, 128, 2, 2, A_KC, B_KC, EPI>(a, st);
  }
}

// One translation unit per operand layout (keeps compile times parallel).
hipError_t launch_gemm_bf16_fwd(const GemmArgs& a, hipStream_t st);     // A k-contiguous, B n-contiguous
hipError_t launch_gemm_bf16_dgrad(const GemmArgs& a, hipStream_t st);   // both k-contiguous
hipError_t launch_gemm_bf16_wgrad(const GemmArgs& a, hipStream_t st);   // A m-contiguous, B n-contiguous

}  // namespace mlm
