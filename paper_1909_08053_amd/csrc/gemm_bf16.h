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
  static constexpr int STRIP = 32 * (WN + 8);                      // elements of one wave's epilogue strip
  static constexpr size_t LDS_MAIN = (size_t)2 * STAGE * 2;
  static constexpr size_t LDS_EPI = (size_t)WAVES_M * WAVES_N * STRIP * 2 + (size_t)2 * WAVES_N * BM * 4;
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

// Epilogue shared by the GEMM kernels.  acc[i][j][e] holds row m = m0 + wm0 + 32 j + l32 and column
// n = n0 + wn0 + 32 i + 8 (e/4) + 4 lh + (e%4) of the output tile.  Must be entered after a workgroup barrier that
// follows the last LDS read of the main loop (the LDS is reused for the staging strips).
template <int BM, int BN, int WAVES_M, int WAVES_N, int EPI>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs& a, floatx16 (&acc)[BN / WAVES_N / 32][BM / WAVES_M / 32],
                                              unsigned char* lds_raw, int m0, int n0, int tile_n) {
  typedef GemmTile<BM, BN, WAVES_M, WAVES_N> Tcfg;
  constexpr int NT = Tcfg::NT, TM = Tcfg::TM, TN = Tcfg::TN, WM = Tcfg::WM, WN = Tcfg::WN;
  bf16* lds = reinterpret_cast<bf16*>(lds_raw);
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, lh = lane >> 5;
  const int wm0 = (wave / WAVES_N) * WM, wn0 = (wave % WAVES_N) * WN;
  bf16* strip = lds + wave * Tcfg::STRIP;
  bf16* C = (bf16*)a.C;
  const bf16* bias = (const bf16*)a.bias;

  if (EPI == EPI_CE) {
    float* red_m = reinterpret_cast<float*>(lds_raw + (size_t)WAVES_M * WAVES_N * Tcfg::STRIP * 2);
    float* red_s = red_m + WAVES_N * BM;
    if (n0 + BN > a.N) {
      // ragged last column tile: columns past N take no part in the statistics (exp(-inf) = 0)
#pragma unroll
      for (int j = 0; j < TM; ++j)
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
          for (int e = 0; e < 16; ++e)
            if (n0 + wn0 + i * 32 + 8 * (e >> 2) + 4 * lh + (e & 3) >= a.N) acc[i][j][e] = -INFINITY;
    }
#pragma unroll
    for (int j = 0; j < TM; ++j) {
      const int row = m0 + wm0 + j * 32 + l32;
      float mx = -INFINITY;
#pragma unroll
      for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) mx = fmaxf(mx, acc[i][j][e]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      // column of the target inside this lane's registers, or -1: integer test, then one select per value
      const int loc = (row < a.M) ? a.targets[row] - a.v0 - (n0 + wn0 + 4 * lh) : -1;
      const float mxl = mx * 1.4426950408889634f;
      float se = 0.f, tv = 0.f;
#pragma unroll
      for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const float v = acc[i][j][e];
          se += __builtin_amdgcn_exp2f(fmaf(v, 1.4426950408889634f, -mxl));
          tv = (loc == i * 32 + 8 * (e >> 2) + (e & 3)) ? v : tv;
        }
      se += __shfl_xor(se, 32, 64);
      if (loc >= 0 && loc < WN && ((loc >> 2) & 1) == 0) a.t_out[row] = tv;   // (loc & 4) == 0: column owned by this half
      if (lh == 0) {
        red_m[(wave % WAVES_N) * BM + wm0 + j * 32 + l32] = mx;
        red_s[(wave % WAVES_N) * BM + wm0 + j * 32 + l32] = se;
      }
      __builtin_amdgcn_sched_barrier(0);
    }
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

  constexpr int NPASS = (EPI == EPI_BIAS_GELU) ? 2 : 1;
#pragma unroll
  for (int j = 0; j < TM; ++j) {
    const int row = m0 + wm0 + j * 32 + l32;
    const int rowc = min(row, a.M - 1);
    float coef = 0.f, Mr = 0.f, invS = 0.f;
    int loc = -1;
    if (EPI == EPI_DLOGITS) {
      coef = (a.loss_w ? a.loss_w[rowc] : 1.0f) / a.loss_stats[1];
      Mr = a.Mrow[rowc];
      invS = coef / a.Srow[rowc];
      loc = a.targets[rowc] - a.v0;
    }
#pragma unroll
    for (int pass = 0; pass < NPASS; ++pass) {
#pragma unroll
      for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int nl = i * 32 + 8 * g + 4 * lh;            // column inside the wave tile
          const int n = n0 + wn0 + nl;
          const int nc = min(n, a.N - 4);
          float v[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = acc[i][j][4 * g + e];
          if (EPI == EPI_STORE || EPI == EPI_BIAS_GELU) {
            if (bias) {
              const bf16x4 bv = *reinterpret_cast<const bf16x4*>(bias + nc);
#pragma unroll
              for (int e = 0; e < 4; ++e) v[e] += (float)bv[e];
            }
            if (EPI == EPI_BIAS_GELU && pass == 1) {
#pragma unroll
              for (int e = 0; e < 4; ++e) v[e] = gelu_fwd(v[e], a.gelu_tanh != 0);
            }
          } else if (EPI == EPI_DGELU) {
            const bf16x4 gv = *reinterpret_cast<const bf16x4*>((const bf16*)a.aux + (size_t)rowc * a.ldaux + nc);
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] *= gelu_bwd((float)gv[e], a.gelu_tanh != 0);
          } else if (EPI == EPI_DLOGITS) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              v[e] = __expf(v[e] - Mr) * invS;
              if (n + e == loc) v[e] -= coef;
            }
          }
          bf16x4 o;
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = (bf16)v[e];
          *reinterpret_cast<bf16x4*>(strip + l32 * (WN + 8) + nl) = o;
        }
      __builtin_amdgcn_sched_barrier(0);
      __builtin_amdgcn_wave_barrier();
      bf16* dst = (EPI == EPI_BIAS_GELU && pass == 0) ? (bf16*)a.aux : C;
      const int ldd = (EPI == EPI_BIAS_GELU && pass == 0) ? a.ldaux : a.ldc;
      constexpr int VPR = WN / 8;                              // 16-byte vectors per strip row
#pragma unroll
      for (int it = 0; it < (32 * VPR) / 64; ++it) {
        const int v = lane + it * 64;
        const int r = v / VPR, cv = v % VPR;
        const int gm = m0 + wm0 + j * 32 + r;
        const int gn = n0 + wn0 + cv * 8;
        if (gm < a.M && gn < a.N)
          *reinterpret_cast<uint4*>(dst + (size_t)gm * ldd + gn) =
              *reinterpret_cast<const uint4*>(strip + r * (WN + 8) + cv * 8);
      }
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_sched_barrier(0);
    }
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
  static bool attr_set = false;   // per instantiation; idempotent, so a race only repeats the call
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)Tcfg::LDS_BYTES);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
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
