// Second-generation bf16 MFMA GEMM main loop for gfx950, built on three CDNA4 features:
//   * global_load_lds_dwordx4: tiles go from HBM/L2 straight into LDS (no VGPR staging, no LDS-write
//     instructions, no VALU permutes), asynchronously, tracked by vmcnt.  Each wave instruction moves
//     64 lanes x 16 B = 1 KB into one contiguous LDS kilobyte, so the bank-conflict swizzle is applied on
//     the GLOBAL side: lane t fetches the 16-byte unit that belongs at LDS position t.
//   * ds_read_b64_tr_b16: an operand that is contiguous along m or n in memory (weights [in,out] in the
//     forward GEMM, both operands of the weight-gradient GEMM) stays in LDS in its natural [k][n] layout and
//     is transposed by the LDS read itself: 16 lanes read a 4(k) x 16(n) patch and each lane receives four
//     consecutive k of one column.  Two such reads give the same 8-consecutive-k operand registers that a
//     16-byte read of a k-contiguous tile gives, so both kinds of tiles feed the same MFMA loop.
//   * 160 KB LDS: a 256 x 256 block tile with a FOUR-stage ring of 32-deep k-slices (128 KB).  The operands of a
//     slice are pulled into registers while the slice before it is multiplied, so its stage is re-armed while it is
//     still being multiplied: three slices are in flight and one is landed, about 3500 MFMA clocks of prefetch
//     distance, one barrier per slice.
//   * v_mfma_f32_16x16x32_bf16 in the 8-wave variants: the same peak rate as the 32 x 32 x 16 shape, but a higher
//     sustained rate on real (normally distributed) operands, where the chip's power limit sets the clock.
// Requirements: K % 32 == 0 and K >= 64 (the dispatcher falls back to the register-staged kernel otherwise).  k is
// walked in pairs of 32-deep slices; when K is an odd multiple of 32 the LAST pair starts at K - 64, i.e. it overlaps
// the pair before it by one slice, and the MFMAs of its first (already counted) slice are skipped: every copy stays
// inside the operand and the instruction stream of the steady state is unchanged.
//
// Tail split: when the tile count does not fill a whole number of rounds of the 256 CUs, the tiles of the last
// partial round are split along k into f pieces (f = floor(256 / remainder)); each piece writes an fp32 partial
// tile to a workspace and gemm_v2_fixup_kernel sums the pieces in a fixed order (deterministic) and applies
// the bias.  Only the plain-store epilogue takes part.
#pragma once
#include "gemm_bf16.h"
#include "lds_dma.h"
#include <string.h>
#include <type_traits>

namespace mlm {

// MFMA shape of the main loop: 16 (v_mfma_f32_16x16x32_bf16) unless the library is built with
// -DMLM_GEMM_MFMA_SHAPE=32 (v_mfma_f32_32x32x16_bf16, the earlier loop, kept for comparison builds).
#ifndef MLM_GEMM_MFMA_SHAPE
#define MLM_GEMM_MFMA_SHAPE 16
#endif
constexpr int V2_MF = MLM_GEMM_MFMA_SHAPE;
// The 4-wave variant (128 x 128 per wave, 256 accumulator registers) keeps the 32 x 32 x 16 shape: with 64 separate
// 16 x 16 accumulators the compiler spills over a thousand registers, and the measured gain of the shape is half as
// large there (fewer fragment reads per MFMA to begin with).
template <int NW> constexpr int v2_mf() { return NW == 4 ? 32 : V2_MF; }
constexpr int V2_B = 256;                   // block tile edge (M and N)
constexpr int V2_BK = 32;                   // k per stage
constexpr int V2_STAGES = 4;
constexpr int V2_OP_BYTES = V2_B * V2_BK * 2;          // 16 KB per operand per stage
constexpr int V2_REGION_BYTES = V2_STAGES * V2_OP_BYTES;   // 64 KB ring per operand: A's ring, then B's ring
constexpr size_t V2_LDS_BYTES = (size_t)2 * V2_REGION_BYTES;          // 128 KB
constexpr int V2_MAX_CUS = 256;              // bound of the tail-split workspace: at most this many fp32 partial tiles
// Compute units of the current device (tiles that run concurrently: one 128-KB workgroup per unit), capped at
// V2_MAX_CUS; asked from the runtime once per device.
int gemm_cu_count();

// Bank swizzle of the [k][row] tile layout (XOR on the 16-byte unit index of a 512-byte k-row).  A transposing read
// is served in two passes of 32 lanes; a pass reads 64 contiguous bytes (four units) of each of four consecutive
// k-rows, and every k-row starts at bank 0.  XORing the unit index with 4 (k & 3) sends the four rows to four different
// 64-byte slots of the 256-byte bank row, so a pass touches every bank once (checked by simulation and with the
// LDS bank-conflict counter: an earlier swizzle that only spread the rows over 128 bytes showed 50 % conflict cycles).
// The 16 x 16 x 32 MFMA's operand puts k = 8 g .. 8 g + 7 into lane group g = lane / 16, so a pass of its transposing
// read covers k-rows 0 .. 3 (or 4 .. 7) AND 8 .. 11 (12 .. 15), 32 bytes of each: bit 3 of k moves a row by another 32
// bytes.  With this term both MFMA shapes read conflict-free (simulated for both).
__device__ __forceinline__ int v2_mn_swizzle(int k) { return ((k & 3) << 2) | (((k >> 3) & 1) << 1); }

// LDS position (16-byte unit inside the k-row) of logical row-chunk u of k-row k, and its inverse, for a [k][ROWS]
// tile.  256 rows: the XOR above.  192 rows: a k-row is 384 bytes = 24 units and starts at bank 0 or 32 alternately
// (384 = 256 + 128), so the four k-rows of a pass would pair up on the same 64-byte slots; rotating the rows with
// bit 1 of k set by four units sends the four 64-byte windows to the four different slots of the 256-byte bank row
// (slot = (6 k + position / 4) mod 4 -> 0, 2, 1, 3), wrap-around included.
// (192 rows, 16 x 16 x 32 reads: two more units for bit 3 of k, as above)
__device__ __forceinline__ int v2_mn_rot192(int k) { return (((k >> 1) & 1) << 2) + (((k >> 3) & 1) << 1); }
template <int ROWS> __device__ __forceinline__ int v2_mn_pos(int u, int k) {
  if (ROWS == V2_B) return u ^ v2_mn_swizzle(k);
  const int t = u + v2_mn_rot192(k);
  return t >= ROWS / 8 ? t - ROWS / 8 : t;
}
template <int ROWS> __device__ __forceinline__ int v2_mn_chunk(int pos, int k) {
  if (ROWS == V2_B) return pos ^ v2_mn_swizzle(k);
  const int t = pos - v2_mn_rot192(k);
  return t < 0 ? t + ROWS / 8 : t;
}

// Bank swizzle of a k-contiguous operand's ring: rows of 128 bytes (two consecutive k-slices side by side, eight
// 16-byte units), unit index XORed with this value; 16 consecutive rows reading the same logical unit then hit 16
// different bank groups.
__device__ __forceinline__ int v2_kc_swizzle(int row) { return (((row >> 1) & 1) << 2) | ((row >> 2) & 3); }

// Per-lane source pointers of one operand's DMA copies (NP 1-KB copies per wave).
//  * k-contiguous operand (KC): the ring holds two PAIRS of slices; a pair is [256 rows][64 k] = 128 bytes per row,
//    so one copy instruction fetches 8 rows x one full 128-byte line (fetching the two 64-byte halves separately,
//    slice by slice, costs twice the cache-line requests and was measured 40 % slower on the copy side).  A pair
//    takes 2 QPW copies per wave and is fetched once every two slices.
//  * operand contiguous along m / n (MN): a slice is [32 k][256 rows] = 512 bytes per k, QPW copies per slice.
template <bool KC, int NP_, int ROWS = V2_B>
struct V2Src {
  static constexpr int NP = NP_;       // KC: 1-KB copies per wave and PAIR (rows / (8 waves)); MN: per wave and slice
  // MN: a slice is ROWS / 16 one-KB copies; where that is no multiple of the wave count (192 rows: 12 copies, 8
  // waves x 2) the surplus copies repeat the last one (same source, same destination: harmless, keeps the per-wave
  // copy count -- and with it the vmcnt bookkeeping -- uniform)
  static constexpr int LAST = KC ? (1 << 20) : ROWS / 16 - 1;
  const bf16* p[NP];
  size_t step;     // elements to advance per 32-deep k-slice
  __device__ __forceinline__ void init(const bf16* P, int ld, int row0, int nrows, int k_begin, int wave, int lane) {
    if (KC) {
#pragma unroll
      for (int q = 0; q < NP; ++q) {
        const int row = (wave * NP + q) * 8 + (lane >> 3);
        const int u = (lane & 7) ^ v2_kc_swizzle(row);
        p[q] = P + (size_t)min(row0 + row, nrows - 1) * ld + k_begin + u * 8;
      }
      step = V2_BK;
    } else {
      // unit u of k-row holds row-chunk u ^ v2_mn_swizzle(k)
#pragma unroll
      for (int q = 0; q < NP; ++q) {
        const int g = 64 * min(wave * NP + q, LAST) + lane;      // linear 16-byte unit of the slice buffer
        const int k = g / (ROWS / 8);
        const int u = v2_mn_chunk<ROWS>(g % (ROWS / 8), k);
        p[q] = P + (size_t)(k_begin + k) * ld + min(row0 + u * 8, nrows - 8);
      }
      step = (size_t)V2_BK * ld;
    }
  }
  // dst: LDS byte address of the pair's (KC) / slice's (MN) buffer; ks: first 32-deep k-slice of the pair / the slice,
  // relative to k_begin; wave_u: wave index as a uniform (SGPR) value
  __device__ __forceinline__ void issue_one(uint32_t dst, int wave_u, int ks, int q) const {
    dma16(p[q] + (ptrdiff_t)ks * (ptrdiff_t)step, dst + min(wave_u * NP + q, LAST) * 1024);
  }
  __device__ __forceinline__ void issue(uint32_t dst, int wave_u, int ks) const {
#pragma unroll
    for (int q = 0; q < NP; ++q) issue_one(dst, wave_u, ks, q);
  }
};

// Operand registers (8 consecutive k of one row/column per lane) for the 32-row MFMA tile starting at row `r0`,
// k-step ks (0 / 1) of the slice in ring stage `stage` of the operand ring at `ring`.
template <bool KC, int ROWS = V2_B>           // ROWS: rows of the operand's tile
__device__ __forceinline__ bf16x8 v2_frag(const unsigned char* ring, int stage, int r0, int ks, int lane) {
  constexpr int OPB = ROWS * V2_BK * 2;       // bytes of one k-slice of the operand
  const int l32 = lane & 31, lh = lane >> 5;
  if (KC) {
    const int row = r0 + l32;
    const int u = (stage & 1) * 4 + ks * 2 + lh;
    return *reinterpret_cast<const bf16x8*>(ring + (stage >> 1) * (2 * OPB) + row * 128 +
                                            ((u ^ v2_kc_swizzle(row)) << 4));
  } else {
    const unsigned char* op_base = ring + stage * OPB;
    const int g = lane >> 4, i16 = lane & 15;
    const int u = (r0 >> 3) + 2 * (g & 1) + ((i16 & 3) >> 1);
    v4s_t h[2];
#pragma unroll
    for (int r = 0; r < 2; ++r) {
      const int k = ks * 16 + 8 * (g >> 1) + 4 * r + (i16 >> 2);
      h[r] = lds_read_tr16(op_base + k * (ROWS * 2) + (v2_mn_pos<ROWS>(u, k) * 16) + (i16 & 1) * 8);
    }
    const v8s_t v = __builtin_shufflevector(h[0], h[1], 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
  }
}

// Operand registers of the 16 x 16 x 32 MFMA for the 16-row tile starting at row `r0`: lane l holds k = 8 (l / 16) ..
// + 7 (the whole 32-deep slice is one MFMA deep) of row r0 + l % 16.
template <bool KC, int ROWS = V2_B>
__device__ __forceinline__ bf16x8 v2_frag16(const unsigned char* ring, int stage, int r0, int lane) {
  constexpr int OPB = ROWS * V2_BK * 2;       // bytes of one k-slice of the operand
  const int l16 = lane & 15, lg = lane >> 4;
  if (KC) {
    const int row = r0 + l16;
    const int u = (stage & 1) * 4 + lg;
    return *reinterpret_cast<const bf16x8*>(ring + (stage >> 1) * (2 * OPB) + row * 128 +
                                            ((u ^ v2_kc_swizzle(row)) << 4));
  } else {
    // two transposing reads: lane j of a group addresses 4 rows (r0 + 4 (j % 4) ..) of k-row 8 g + 4 r + j / 4 and
    // lane i receives k = 8 g + 4 r .. + 3 of row r0 + i
    const unsigned char* op_base = ring + stage * OPB;
    const int u = (r0 >> 3) + ((l16 & 3) >> 1);
    v4s_t h[2];
#pragma unroll
    for (int r = 0; r < 2; ++r) {
      const int k = 8 * lg + 4 * r + (l16 >> 2);
      h[r] = lds_read_tr16(op_base + k * (ROWS * 2) + (v2_mn_pos<ROWS>(u, k) * 16) + (l16 & 1) * 8);
    }
    const v8s_t v = __builtin_shufflevector(h[0], h[1], 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
  }
}

struct V2Plan {
  int tiles_m, tiles_n, full_tiles, tail_tiles, split;   // grid = full_tiles + tail_tiles * split
  int bn;                                                 // tile width (256, or 192 for the narrow-tile variant)
  double cost;                                            // estimated kernel time in microseconds (host side only)
};

// Cost-model constants (microseconds, fitted to rocprofv3 kernel durations of unsplit two-round launches at two
// k-lengths each on MI355X): fixed cost of a tile (fill + epilogue) and cost of one 32-deep k-slice, for the
// 256 x 256 tile and for the 256 x 192 tile (either B layout).  The narrow tile does 3/4 of the MFMA work per slice
// in 0.88 of the time, so it wins where it saves a round or fills one and loses on long-k shapes whose last round
// can be split instead.  The fix-up kernel reads the pieces mostly out of the last-level cache.
inline double v2_tile_fixed(int bn) { return bn == V2_B ? 9.2 : 8.0; }
inline double v2_slice_cost(int bn, bool /*b_mn*/) { return bn == V2_B ? 0.67 : 0.59; }
inline double v2_fixup_cost(double traffic_us) { return 3.0 + 0.6 * traffic_us; }

// Decide whether, and how far, to split the last partial round along k.  Cost model in microseconds: a tile costs
// its fixed part + the per-slice cost of its k-slices; the pieces write fp32 partial tiles at ~5 TB/s and the fix-up
// kernel reads them back.
inline V2Plan v2_plan(int M, int N, int K, bool allow_split, int bn = V2_B, bool b_mn = false) {
  const int V2_CUS = gemm_cu_count();
  V2Plan p;
  p.bn = bn;
  p.tiles_m = (M + V2_B - 1) / V2_B;
  p.tiles_n = (N + bn - 1) / bn;
  const int tiles = p.tiles_m * p.tiles_n;
  const int rem = tiles % V2_CUS;
  const int nk = 2 * ((K / V2_BK + 1) / 2);           // slices walked: pairs of 32 (an odd count repeats one slice)
  const double fixed = v2_tile_fixed(bn), per_slice = v2_slice_cost(bn, b_mn);
  int split = 1;
  double tail = rem ? fixed + per_slice * nk : 0.0;   // unsplit tail round
  if (allow_split && rem != 0 && rem * 2 <= V2_CUS) {
    int smax = V2_CUS / rem;
    if (smax > 16) smax = 16;
    for (int sp = 2; sp <= smax; ++sp) {
      if (nk / sp < 8) break;                         // keep at least 8 k-slices per piece
      const double traffic = (double)rem * sp * (V2_B * (double)bn * 4.0) / 5.0e6;
      const double t = fixed + per_slice * ((nk + sp - 1) / sp) + traffic + v2_fixup_cost(traffic);
      if (t < tail) { tail = t; split = sp; }
    }
  }
  p.split = split;
  p.tail_tiles = split > 1 ? rem : 0;
  p.full_tiles = tiles - p.tail_tiles;
  p.cost = (tiles / V2_CUS) * (fixed + per_slice * nk) + tail;
  return p;
}

// NW = waves per workgroup: 4 (2 x 2 waves of 128 x 128) or 8 (2 x 4 waves of 128 x 64, two waves per SIMD).
// One work item (pid) of one GEMM: the body of the kernels below.
// BN = 256: 2 x (NW / 2) waves of 128 x (512 / NW).  BN = 192 (8 waves, k-contiguous B only): 4 x 2 waves of 64 x 96 --
// a tile count of 32 x (N / 192) fills the 256 CUs where N / 256 column tiles leave a quarter of them idle
// (N = 1536: 256 tiles instead of 192) or a half-empty second round (N = 3072: 512 instead of 384).
// MF = MFMA shape: 16 (v_mfma_f32_16x16x32_bf16, the default) or 32 (v_mfma_f32_32x32x16_bf16, kept for comparison).
// Same wave tiles, same LDS traffic and the same peak rate, but on normally distributed operands the 16 x 16 x 32
// shape sustains 2.04 PFLOP/s against 1.77 with the matrix pipe alone, 1.60 against 1.45 with this loop's fragment
// reads and copies around it (256 x 256 tile, 8 waves; measured with a stand-alone loop of the same structure).
template <bool A_KC, bool B_KC, int EPI, int NW, int BN = V2_B, int MF = 16>
__device__ __forceinline__ void gemm_v2_work_item(const GemmArgs& a, const V2Plan& plan, float* splitk_ws, int pid,
                                                  unsigned char* lds_raw) {
  static_assert(BN == V2_B || (BN == 192 && NW == 8), "narrow tile: 8 waves");
  static_assert(MF == 16 || MF == 32, "MFMA shape");
  constexpr int WAVES_M = BN == V2_B ? 2 : 4, WAVES_N = NW / WAVES_M;
  constexpr int WM = V2_B / WAVES_M, WN = BN / WAVES_N, TM = WM / 32, TN = WN / 32;
  constexpr int OPB_B = BN * V2_BK * 2;                        // bytes of one k-slice of the B operand
  // 1-KB copies per wave: per pair of slices for a k-contiguous operand, per slice otherwise
  constexpr int NPA = A_KC ? V2_B / (8 * NW) : 16 / NW, NPB = B_KC ? BN / (8 * NW) : (BN / 16 + NW - 1) / NW;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave / WAVES_N) * WM, wn0 = (wave % WAVES_N) * WN;

  // work item: a full tile, or one k-piece of a tail tile
  int vt, piece = 0, npieces = 1;
  if (pid < plan.full_tiles) {
    vt = pid;
  } else {
    const int t = pid - plan.full_tiles;
    vt = plan.full_tiles + t / plan.split;
    piece = t % plan.split;
    npieces = plan.split;
  }
  // Plain order, tile row fastest: the 256 concurrent tiles form 8 tile-columns of 32 tile-rows, and the ids that
  // share an XCD (congruent mod 8) share tile rows, so each XCD's L2 sees few distinct operand panels.
  const int tile_m = vt % plan.tiles_m, tile_n = vt / plan.tiles_m;
  const int m0 = tile_m * V2_B, n0 = tile_n * BN;
  const int ns_total = a.K / V2_BK;                  // 32-deep k-slices of the problem
  const int np_total = (ns_total + 1) / 2;           // k is walked in pairs of slices
  const int kt_begin = 2 * (int)((long)np_total * piece / npieces);
  const int kt_end = 2 * (int)((long)np_total * (piece + 1) / npieces);
  const int nk = kt_end - kt_begin;                  // even, >= 2
  // Odd slice count: the last pair of the problem starts one slice early (at K - 64) and its first slice, which the
  // pair before it has already multiplied, is skipped.  shift = 1 for the piece that holds that pair.
  const int shift = (kt_end > ns_total) ? 1 : 0;
  // first k-slice (relative to kt_begin) of walked slice kt / of walked pair pr
  auto slice_of = [&](int kt) { return kt - (kt >= nk - 2 ? shift : 0); };
  auto pair_of = [&](int pr) { return 2 * pr - (pr == nk / 2 - 1 ? shift : 0); };

  V2Src<A_KC, NPA> sa;
  V2Src<B_KC, NPB, BN> sb;
  sa.init((const bf16*)a.A, a.lda, m0, a.M, kt_begin * V2_BK, wave, lane);
  sb.init((const bf16*)a.B, a.ldb, n0, a.N, kt_begin * V2_BK, wave, lane);

  const uint32_t ldsA = lds_offset_of(lds_raw), ldsB = ldsA + V2_REGION_BYTES;
  const unsigned char* ringA = lds_raw;
  const unsigned char* ringB = lds_raw + V2_REGION_BYTES;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  constexpr int NKC = (A_KC ? 1 : 0) + (B_KC ? 1 : 0), NMN = 2 - NKC;
  // Four slices are always in flight or landed; past the end of k the last pair / slice is fetched again into a
  // stage nobody reads (keeps the vmcnt bookkeeping and the instruction stream free of tail cases).  Issue order of
  // the initial fill = the order the steady state would have produced: pair 0, slices 0 1, pair 1, slices 2 3.
  const int last_pair = nk / 2 - 1, last_slice = nk - 1;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    if (A_KC) sa.issue(ldsA + h * 2 * V2_OP_BYTES, wave_u, pair_of(min(h, last_pair)));
    if (B_KC) sb.issue(ldsB + h * 2 * OPB_B, wave_u, pair_of(min(h, last_pair)));
#pragma unroll
    for (int s = 2 * h; s < 2 * h + 2; ++s) {
      if (!A_KC) sa.issue(ldsA + s * V2_OP_BYTES, wave_u, slice_of(min(s, last_slice)));
      if (!B_KC) sb.issue(ldsB + s * OPB_B, wave_u, slice_of(min(s, last_slice)));
    }
  }
  // The operand registers of what is multiplied next are read from LDS while the matrix cores work (32 x 32 x 16
  // shape: by half-slices of 16 k; 16 x 16 x 32 shape: by whole slices, see there).  The slice hand-over sits inside
  // slice kt: wait for the copies of slice kt+1, barrier, then re-arm what slice kt leaves behind (its operands are all
  // in registers by then): an MN operand's stage gets slice kt+4; a KC operand's pair-stage is free after the ODD
  // slice of the pair and then gets the pair two ahead.  Copies are ISSUED ONE AT A TIME BETWEEN MFMAs: back-to-back 1-KB copies fill
  // the vector-memory queue and would stall the wave, and with it the matrix pipe, for hundreds of clocks.
  //
  // Copies per wave issued at the hand-over of an even slice: EV = NMN QPW; of an odd slice: OD = NKC 2 QPW + NMN QPW
  // (pairs first).  Copies return in order, so "slice kt+1 has landed" is a bound on the copies still outstanding:
  //   even kt: everything up to the hand-over of kt-3 must be done           -> at most EV + OD = 4 QPW outstanding
  //   odd kt:  the pair issued first at the hand-over of kt-2 must be done   -> at most 2 EV outstanding (if NKC > 0)
  constexpr int C_SLICE = (A_KC ? 0 : NPA) + (B_KC ? 0 : NPB);     // copies per wave that re-arm a slice stage
  constexpr int C_PAIR = (A_KC ? NPA : 0) + (B_KC ? NPB : 0);      // copies per wave that re-arm a pair stage
  constexpr int EV = C_SLICE, OD = C_PAIR + C_SLICE;
  constexpr int W_INIT = 3 * C_SLICE + C_PAIR, W_EVEN = EV + OD, W_ODD = NKC > 0 ? 2 * EV : EV + OD;
  (void)NMN;
  if constexpr (MF == 32) {
    floatx16 acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
      for (int j = 0; j < TM; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    constexpr int NMF = TN * TM;           // MFMAs per half-slice per wave
    static_assert(NMF > TM + TN, "one fragment read after each MFMA but the first must cover all fragments");
    bf16x8 fa0[TM], fb0[TN], fa1[TM], fb1[TN];
    wait_vmcnt<W_INIT>();                  // slice 0 landed
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int j = 0; j < TM; ++j) fa0[j] = v2_frag<A_KC>(ringA, 0, wm0 + j * 32, 0, lane);
#pragma unroll
    for (int i = 0; i < TN; ++i) fb0[i] = v2_frag<B_KC, BN>(ringB, 0, wn0 + i * 32, 0, lane);

    // one 32-deep slice; PAR = parity of kt (compile time: it fixes the ring stage bits and the copy schedule);
    // live: false for the slice that repeats one multiplied already (odd slice count): everything but its MFMAs runs.
    // It is a compile-time true in the steady-state loop and a wave-uniform flag (scalar branches) in the peeled last pair.
    auto slice = [&](auto par_c, auto live, int kt) {
      constexpr int PAR = decltype(par_c)::value;
      const int stage = kt & (V2_STAGES - 1);
      // First half.  Order pinned with scheduling barriers: one MFMA first (its operands were read half a slice ago,
      // so the loop-top wait is free), then ONE fragment read of the second half's operands after each MFMA.  Spread
      // like this the reads never queue up in the LDS pipe (all eight waves reach this point together after the
      // barrier), and the MFMAs in between cover their latency.  (Left alone, the scheduler bunches the reads and
      // either hoists them above the loop-top wait or sinks them to the barrier; both expose their full latency.)
#pragma unroll
      for (int idx = 0; idx < NMF; ++idx) {
        if (live) acc[idx / TM][idx % TM] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb0[idx / TM], fa0[idx % TM], acc[idx / TM][idx % TM], 0, 0, 0);
        if (idx >= 1 && idx - 1 < TM + TN) {
          const int q = idx - 1;
          __builtin_amdgcn_sched_barrier(0);
          if (q < TM) fa1[q] = v2_frag<A_KC>(ringA, stage, wm0 + q * 32, 1, lane);
          else fb1[q - TM] = v2_frag<B_KC, BN>(ringB, stage, wn0 + (q - TM) * 32, 1, lane);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      __builtin_amdgcn_sched_barrier(0);     // ... and the MFMAs ahead of the hand-over
      wait_vmcnt<PAR == 0 ? W_EVEN : W_ODD>();   // this wave's copies of slice kt+1 have landed
      // this wave's LDS reads of slice kt (second-half operands, issued above) have returned ...
      __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0) only
      // ... so after this bare s_barrier (no memory fence: a fence would also wait for the copies in flight)
      // everyone's part of slice kt+1 is in LDS and nobody reads slice kt's stage any more.
      __builtin_amdgcn_s_barrier();
      // Second half: after each MFMA one fragment read of slice kt+1's first-half operands, and the copies that
      // re-arm the freed stage(s) spread evenly between the MFMAs.
      const int nstage = (kt + 1) & (V2_STAGES - 1);
      constexpr int NC = PAR == 0 ? EV : OD;                 // copies to issue in this half
      const int pair_idx = pair_of(min((kt + 3) >> 1, last_pair));   // PAR == 1: the pair two ahead of this slice's pair
      const uint32_t pair_sel = (uint32_t)(((kt + 3) >> 1) & 1);
      const uint32_t pair_off_a = pair_sel * (2 * V2_OP_BYTES), pair_off_b = pair_sel * (2 * OPB_B);
      const int slice_idx = slice_of(min(kt + V2_STAGES, last_slice));
      const uint32_t slice_off_a = (uint32_t)stage * V2_OP_BYTES, slice_off_b = (uint32_t)stage * OPB_B;
#pragma unroll
      for (int idx = 0; idx < NMF; ++idx) {
        if (live) acc[idx / TM][idx % TM] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb1[idx / TM], fa1[idx % TM], acc[idx / TM][idx % TM], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (idx < TM + TN) {
          const int q = idx;
          if (q < TM) fa0[q] = v2_frag<A_KC>(ringA, nstage, wm0 + q * 32, 0, lane);
          else fb0[q - TM] = v2_frag<B_KC, BN>(ringB, nstage, wn0 + (q - TM) * 32, 0, lane);
        }
#pragma unroll
        for (int c = 0; c < NC; ++c) {
          if ((c * NMF) / (NC > 0 ? NC : 1) != idx) continue;   // copy c goes after MFMA (c NMF) / NC
          // order: A's pair, B's pair (odd slices only), then A's slice, B's slice
          int r = c;
          constexpr int KA = (PAR == 1 && A_KC) ? NPA : 0, KB = (PAR == 1 && B_KC) ? NPB : 0;
          constexpr int MA = A_KC ? 0 : NPA;
          if (r < KA) { sa.issue_one(ldsA + pair_off_a, wave_u, pair_idx, r); continue; }
          r -= KA;
          if (r < KB) { sb.issue_one(ldsB + pair_off_b, wave_u, pair_idx, r); continue; }
          r -= KB;
          if (r < MA) { sa.issue_one(ldsA + slice_off_a, wave_u, slice_idx, r); continue; }
          r -= MA;
          sb.issue_one(ldsB + slice_off_b, wave_u, slice_idx, r);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    typedef std::integral_constant<int, 0> c0_t;
    typedef std::integral_constant<int, 1> c1_t;
    for (int kt = 0; kt < nk - 2; kt += 2) {
      slice(c0_t{}, std::true_type{}, kt);
      slice(c1_t{}, std::true_type{}, kt + 1);
    }
    slice(c0_t{}, shift == 0, nk - 2);                  // odd slice count: this one repeats slice nk - 3, copies only
    slice(c1_t{}, std::true_type{}, nk - 1);
    // The ring is kept full to the end, so copies of the (clamped) last slice are still in flight here.  They were
    // issued from inline assembly, which the compiler's wait-count tracking does not see: wait for them explicitly
    // before the epilogue reuses the ring's memory for its staging strips.
    wait_vmcnt<0>();
    __syncthreads();

    if (npieces > 1) {
      // fp32 partial tile: piece-major [tail tile][piece][256][BN]
      const int l32 = lane & 31, lh = lane >> 5;
      float* dst = splitk_ws + ((size_t)(vt - plan.full_tiles) * plan.split + piece) * (V2_B * BN);
#pragma unroll
      for (int j = 0; j < TM; ++j)
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            float4 v = make_float4(acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]);
            *reinterpret_cast<float4*>(dst + (wm0 + j * 32 + l32) * BN + wn0 + i * 32 + 8 * g + 4 * lh) = v;
          }
      return;
    }
    gemm_epilogue<V2_B, BN, WAVES_M, WAVES_N, EPI>(a, acc, lds_raw, m0, n0, tile_n);
  } else {
    // ---- 16 x 16 x 32 MFMAs: one MFMA spans the slice's 32 k, so a wave holds the fragments of ONE slice: NA of A, NB
    // of B.  MFMA order: A fragment outer, B fragment inner.  A fragment j is replaced by the next slice's behind
    // its last MFMA (j, NB - 1) and is next used about NMF - NB MFMAs later; the B fragments are double-buffered (the slice's
    // parity picks the set) and the next slice's are read right after the hand-over.  The hand-over (wait for the
    // copies of slice kt + 1, barrier) sits after MFMA HO, ahead of the first read of slice kt + 1; the copies that
    // re-arm slice kt's stage (all of its fragments were in registers before the slice began) follow it, one at a
    // time between the MFMAs.  Measured on the benchmark step: HO = 0 .. 2 within noise of each other, later
    // hand-overs slower (HO = 15: +0.5 %); B fragment outer with in-place replacement of both operands (A fragments
    // then have NA MFMAs between read and use) the same step time, 1 % slower on the logits GEMM.
    constexpr int NA = WM / 16, NB = WN / 16, NMF = NA * NB;
    constexpr int HO = 1;
    static_assert(HO + 1 + NB <= NMF, "the next slice's B fragments are read in this slice");
    floatx4 acc[NB][NA];
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
      for (int j = 0; j < NA; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.f;
    bf16x8 fa[NA], fb[2][NB];
    wait_vmcnt<W_INIT>();                  // slice 0 landed
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int j = 0; j < NA; ++j) fa[j] = v2_frag16<A_KC>(ringA, 0, wm0 + j * 16, lane);
#pragma unroll
    for (int i = 0; i < NB; ++i) fb[0][i] = v2_frag16<B_KC, BN>(ringB, 0, wn0 + i * 16, lane);

    // one 32-deep slice; PAR = parity of kt (compile time: it fixes the ring stage bits and the copy schedule);
    // live: false for the slice that repeats one multiplied already (odd slice count): everything but its MFMAs runs.
    auto slice = [&](auto par_c, auto live, int kt) {
      constexpr int PAR = decltype(par_c)::value;
      const int stage = kt & (V2_STAGES - 1), nstage = (kt + 1) & (V2_STAGES - 1);
      constexpr int NC = PAR == 0 ? EV : OD;                 // copies to issue in this slice
      constexpr int NAFTER = NMF - HO - 1;                   // MFMAs after the hand-over
      const int pair_idx = pair_of(min((kt + 3) >> 1, last_pair));   // PAR == 1: the pair two ahead of this slice's pair
      const uint32_t pair_sel = (uint32_t)(((kt + 3) >> 1) & 1);
      const uint32_t pair_off_a = pair_sel * (2 * V2_OP_BYTES), pair_off_b = pair_sel * (2 * OPB_B);
      const int slice_idx = slice_of(min(kt + V2_STAGES, last_slice));
      const uint32_t slice_off_a = (uint32_t)stage * V2_OP_BYTES, slice_off_b = (uint32_t)stage * OPB_B;
#pragma unroll
      for (int idx = 0; idx < NMF; ++idx) {
        const int i = idx % NB, j = idx / NB;
        constexpr int CUR = PAR, NXT = 1 - PAR;
        if (live) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[CUR][i], fa[j], acc[i][j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (idx == HO) {
          wait_vmcnt<PAR == 0 ? W_EVEN : W_ODD>();   // this wave's copies of slice kt+1 have landed
          // this wave's LDS reads of slice kt's stage (the last fragments, read at the end of slice kt - 1) have returned ...
          __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0) only
          // ... so after this bare s_barrier (no memory fence: a fence would also wait for the copies in flight)
          // everyone's part of slice kt+1 is in LDS and nobody reads slice kt's stage any more.
          __builtin_amdgcn_s_barrier();
        }
        if (idx > HO) {
          // fragments of slice kt + 1 into the registers that slice kt has finished with
#pragma unroll
          for (int q = 0; q < NB; ++q)
            if (idx == HO + 1 + q) fb[NXT][q] = v2_frag16<B_KC, BN>(ringB, nstage, wn0 + q * 16, lane);
#pragma unroll
          for (int q = 0; q < NA; ++q) {
            // one MFMA after the fragment's last one (q, NB - 1) -- directly behind it the read needs wait states, the
            // MFMA still reads the registers -- but inside the slice and not before the hand-over
            const int last = q * NB + NB < NMF - 1 ? q * NB + NB : NMF - 1;
            const int at = last > HO ? last : HO + 1;
            if (idx == at) fa[q] = v2_frag16<A_KC>(ringA, nstage, wm0 + q * 16, lane);
          }
#pragma unroll
          for (int c = 0; c < NC; ++c) {
            if (HO + 1 + (c * NAFTER) / (NC > 0 ? NC : 1) != idx) continue;   // copy c goes after MFMA HO + 1 + (c NAFTER) / NC
            // order: A's pair, B's pair (odd slices only), then A's slice, B's slice
            int r = c;
            constexpr int KA = (PAR == 1 && A_KC) ? NPA : 0, KB = (PAR == 1 && B_KC) ? NPB : 0;
            constexpr int MA = A_KC ? 0 : NPA;
            if (r < KA) { sa.issue_one(ldsA + pair_off_a, wave_u, pair_idx, r); continue; }
            r -= KA;
            if (r < KB) { sb.issue_one(ldsB + pair_off_b, wave_u, pair_idx, r); continue; }
            r -= KB;
            if (r < MA) { sa.issue_one(ldsA + slice_off_a, wave_u, slice_idx, r); continue; }
            r -= MA;
            sb.issue_one(ldsB + slice_off_b, wave_u, slice_idx, r);
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    typedef std::integral_constant<int, 0> c0_t;
    typedef std::integral_constant<int, 1> c1_t;
    for (int kt = 0; kt < nk - 2; kt += 2) {
      slice(c0_t{}, std::true_type{}, kt);
      slice(c1_t{}, std::true_type{}, kt + 1);
    }
    slice(c0_t{}, shift == 0, nk - 2);                  // odd slice count: this one repeats slice nk - 3, copies only
    slice(c1_t{}, std::true_type{}, nk - 1);
    // copies of the (clamped) last slices are still in flight and target the ring the epilogue reuses
    wait_vmcnt<0>();
    __syncthreads();

    if (npieces > 1) {
      // fp32 partial tile: piece-major [tail tile][piece][256][BN]
      const int l16 = lane & 15, lg = lane >> 4;
      float* dst = splitk_ws + ((size_t)(vt - plan.full_tiles) * plan.split + piece) * (V2_B * BN);
#pragma unroll
      for (int j = 0; j < NA; ++j)
#pragma unroll
        for (int i = 0; i < NB; ++i) {
          const float4 v = make_float4(acc[i][j][0], acc[i][j][1], acc[i][j][2], acc[i][j][3]);
          *reinterpret_cast<float4*>(dst + (wm0 + j * 16 + l16) * BN + wn0 + i * 16 + 4 * lg) = v;
        }
      return;
    }
    gemm_epilogue<V2_B, BN, WAVES_M, WAVES_N, EPI>(a, acc, lds_raw, m0, n0, tile_n);
  }
}

template <bool A_KC, bool B_KC, int EPI, int NW, int BN = V2_B>
__global__ __launch_bounds__(NW * 64) void gemm_bf16_v2_kernel(GemmArgs a, V2Plan plan, float* splitk_ws) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  gemm_v2_work_item<A_KC, B_KC, EPI, NW, BN, v2_mf<NW>()>(a, plan, splitk_ws, blockIdx.x, lds_raw);
}

// Several independent GEMMs of one operand layout in ONE launch (plain-store epilogue, no k-split): the tiles of
// problem q follow those of problem q - 1 in the grid, so the launch pays the partially filled last round of the
// 256 CUs once instead of once per GEMM.  Used for the weight gradients of a layer shard, which nothing but the
// optimizer waits for: four GEMMs with 72 + 72 + 24 + 60 tiles at the 8.3B-shape 1/8 shard become one round.
constexpr int kMaxGroup = 4;
struct GemmGroup {
  int n;
  int tile_begin[kMaxGroup + 1];       // first work item of each problem; tile_begin[n] = grid size
  GemmArgs args[kMaxGroup];
  V2Plan plan[kMaxGroup];
};

template <bool A_KC, bool B_KC, int NW>
__global__ __launch_bounds__(NW * 64) void gemm_bf16_v2_group_kernel(GemmGroup g) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  const int pid = blockIdx.x;
  // the problem index is uniform over the workgroup: select its arguments with scalar compares
  int q = 0;
#pragma unroll
  for (int i = 1; i < kMaxGroup; ++i) q += (i < g.n && pid >= g.tile_begin[i]) ? 1 : 0;
  GemmArgs a = g.args[0];
  V2Plan plan = g.plan[0];
  int first = g.tile_begin[0];
#pragma unroll
  for (int i = 1; i < kMaxGroup; ++i)
    if (q == i) { a = g.args[i]; plan = g.plan[i]; first = g.tile_begin[i]; }
  gemm_v2_work_item<A_KC, B_KC, EPI_STORE, NW, V2_B, v2_mf<NW>()>(a, plan, nullptr, pid - first, lds_raw);
}

// Tail tiles: sum the k-pieces in piece order (deterministic) and apply the epilogue to the fp32 sums.  A wave owns
// whole 256-column tile rows (a lane: 4 consecutive columns), so the row statistics of the cross-entropy epilogue are
// one wave reduction.  Grid: (256 / kFixRows row groups, tail tiles), 4 waves, kFixRows / 4 rows per wave.
constexpr int kFixRows = 8;
template <int EPI>
__global__ __launch_bounds__(256) void gemm_v2_fixup_kernel(GemmArgs a, V2Plan plan, const float* __restrict__ ws) {
  const int t = blockIdx.y;                          // tail tile
  const int vt = plan.full_tiles + t;
  const int tile_n = vt / plan.tiles_m;
  const int bn = plan.bn;                             // tile width: a partial tile is [256][bn] floats
  const int m0 = (vt % plan.tiles_m) * V2_B, n0 = tile_n * bn;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = n0 + lane * 4;
  const bool col_ok = n < a.N && lane * 4 < bn;       // N is a multiple of 8: a 4-column group is all in or all out
  const int nc = col_ok ? n : 0;
  const int lcol = lane * 4 < bn ? lane * 4 : 0;
  const float* base = ws + (size_t)t * plan.split * (V2_B * bn) + lcol;
  float bv[4] = {0.f, 0.f, 0.f, 0.f};
  if ((EPI == EPI_STORE || EPI == EPI_BIAS_GELU) && a.bias != nullptr) {
    const bf16x4 b = *reinterpret_cast<const bf16x4*>((const bf16*)a.bias + nc);
#pragma unroll
    for (int e = 0; e < 4; ++e) bv[e] = (float)b[e];
  }
  constexpr int RPW = kFixRows / 4;
  float v[RPW][4];
#pragma unroll
  for (int i = 0; i < RPW; ++i) {
    const int r = blockIdx.x * kFixRows + wave * RPW + i;
#pragma unroll
    for (int e = 0; e < 4; ++e) v[i][e] = bv[e];
    for (int p = 0; p < plan.split; ++p) {
      const float4 x = *reinterpret_cast<const float4*>(base + (size_t)p * (V2_B * bn) + r * bn);
      v[i][0] += x.x; v[i][1] += x.y; v[i][2] += x.z; v[i][3] += x.w;
    }
  }
#pragma unroll
  for (int i = 0; i < RPW; ++i) {
    const int r = blockIdx.x * kFixRows + wave * RPW + i;
    const int m = m0 + r;
    if (m >= a.M) break;                              // wave-uniform
    const bool ok = col_ok;
    bf16x4 o;
    if (EPI == EPI_STORE) {
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] = (bf16)v[i][e];
    } else if (EPI == EPI_BIAS_GELU) {
      bf16x4 pre;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        pre[e] = (bf16)v[i][e];
        o[e] = (bf16)gelu_fwd(v[i][e], a.gelu_tanh != 0);
      }
      if (ok) *reinterpret_cast<bf16x4*>((bf16*)a.aux + (size_t)m * a.ldaux + n) = pre;
    } else if (EPI == EPI_DGELU) {
      const bf16x4 g4 = *reinterpret_cast<const bf16x4*>((const bf16*)a.aux + (size_t)m * a.ldaux + nc);
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] = (bf16)(v[i][e] * gelu_bwd((float)g4[e], a.gelu_tanh != 0));
    } else if (EPI == EPI_CE) {
      float mx = -INFINITY;
      if (ok) mx = fmaxf(fmaxf(v[i][0], v[i][1]), fmaxf(v[i][2], v[i][3]));
      mx = wave_max(mx);
      const float mxl = mx * 1.4426950408889634f;
      float se = 0.f;
      if (ok) {
#pragma unroll
        for (int e = 0; e < 4; ++e) se += __builtin_amdgcn_exp2f(fmaf(v[i][e], 1.4426950408889634f, -mxl));
      }
      se = wave_sum(se);
      const int loc = a.targets[m] - a.v0 - n0;       // target column inside this tile, if 0 <= loc < 256
      if (ok && loc >= 0 && (loc >> 2) == lane) {
        float tv = v[i][0];
#pragma unroll
        for (int e = 1; e < 4; ++e) tv = ((loc & 3) == e) ? v[i][e] : tv;
        a.t_out[m] = tv;
      }
      if (lane == 0) {
        a.part_m[(size_t)tile_n * a.M + m] = mx;
        a.part_s[(size_t)tile_n * a.M + m] = se;
      }
      if (a.C == nullptr) continue;
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] = (bf16)v[i][e];
    } else if (EPI == EPI_DLOGITS) {
      const float coef = (a.loss_w ? a.loss_w[m] : 1.0f) / a.loss_stats[1];
      const float Mrl = a.Mrow[m] * 1.4426950408889634f;
      const float invS = coef / a.Srow[m];
      const int loc = a.targets[m] - a.v0 - n;        // target column relative to this lane's first column
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float pz = __builtin_amdgcn_exp2f(fmaf(v[i][e], 1.4426950408889634f, -Mrl)) * invS;
        if (loc == e) pz -= coef;
        o[e] = (bf16)pz;
      }
    }
    if (ok) *reinterpret_cast<bf16x4*>((bf16*)a.C + (size_t)m * a.ldc + n) = o;
  }
}

inline size_t v2_splitk_ws_bytes() { return (size_t)V2_MAX_CUS * V2_B * V2_B * sizeof(float); }   // 64 MB upper bound

int gemm_v2_waves(bool a_kc, bool b_kc);   // 4 or 8 waves per workgroup for this operand layout

template <bool A_KC, bool B_KC, int EPI, int NW, int BN = V2_B>
hipError_t launch_gemm_bf16_v2_nw(const GemmArgs& a, float* splitk_ws, hipStream_t st) {
  auto kern = gemm_bf16_v2_kernel<A_KC, B_KC, EPI, NW, BN>;
  // the ring (128 KB) or, with 8 waves, the epilogue's staging strips (2 per wave) + reduction area, whichever is larger
  constexpr int WAVES_M = BN == V2_B ? 2 : 4;
  constexpr size_t kEpi = GemmTile<V2_B, BN, WAVES_M, NW / WAVES_M>::LDS_EPI;
  constexpr size_t kLds = V2_LDS_BYTES > kEpi ? V2_LDS_BYTES : kEpi;
  static_assert(kLds <= 160 * 1024, "LDS budget");
  static LdsAttrOnce attr;         // per instantiation and device
  if (hipError_t e = attr.ensure((const void*)kern, (int)kLds); e != hipSuccess) return e;
  const V2Plan plan = v2_plan(a.M, a.N, a.K, splitk_ws != nullptr, BN, !B_KC);
  const int grid = plan.full_tiles + plan.tail_tiles * plan.split;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(NW * 64), kLds, st, a, plan, splitk_ws);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (plan.tail_tiles) {
    hipLaunchKernelGGL((gemm_v2_fixup_kernel<EPI>), dim3(V2_B / kFixRows, plan.tail_tiles), dim3(256), 0, st, a, plan,
                       splitk_ws);
    e = hipGetLastError();
  }
  return e;
}

// Tiles (work items without a k-split) of one problem.
inline int v2_tiles(const GemmArgs& a) { return ((a.M + V2_B - 1) / V2_B) * ((a.N + V2_B - 1) / V2_B); }

template <bool A_KC, bool B_KC, int NW>
hipError_t launch_gemm_bf16_v2_group_nw(const GemmArgs* probs, int n, hipStream_t st) {
  auto kern = gemm_bf16_v2_group_kernel<A_KC, B_KC, NW>;
  constexpr size_t kEpi = GemmTile<V2_B, V2_B, 2, NW / 2>::LDS_EPI;
  constexpr size_t kLds = V2_LDS_BYTES > kEpi ? V2_LDS_BYTES : kEpi;
  static LdsAttrOnce attr;
  if (hipError_t e = attr.ensure((const void*)kern, (int)kLds); e != hipSuccess) return e;
  GemmGroup g;
  memset(&g, 0, sizeof(g));
  g.n = n;
  int total = 0;
  for (int q = 0; q < n; ++q) {
    g.args[q] = probs[q];
    g.plan[q] = v2_plan(probs[q].M, probs[q].N, probs[q].K, false);
    g.tile_begin[q] = total;
    total += g.plan[q].full_tiles;
  }
  for (int q = n; q <= kMaxGroup; ++q) g.tile_begin[q] = total;
  hipLaunchKernelGGL(kern, dim3(total), dim3(NW * 64), kLds, st, g);
  return hipGetLastError();
}

int gemm_v2_forced_bn();                    // MLM_GEMM_BN=192|256 forces a tile width where both exist, else 0

template <bool A_KC, bool B_KC, int EPI>
hipError_t launch_gemm_bf16_v2(const GemmArgs& a, float* splitk_ws, hipStream_t st) {
  if (gemm_v2_waves(A_KC, B_KC) == 8) {
    // both tile widths exist for the input-gradient layout and for the plain / bias + GeLU forward GEMMs: take the
    // one the cost model prices lower for this shape
    constexpr bool kHasNarrow = A_KC && (B_KC || EPI == EPI_STORE || EPI == EPI_BIAS_GELU);
    if (kHasNarrow) {
      const int forced = gemm_v2_forced_bn();
      const bool narrow = forced ? forced == 192
                                 : v2_plan(a.M, a.N, a.K, splitk_ws != nullptr, 192, !B_KC).cost <
                                       v2_plan(a.M, a.N, a.K, splitk_ws != nullptr, V2_B, !B_KC).cost;
      if (narrow) return launch_gemm_bf16_v2_nw<A_KC, B_KC, EPI, 8, kHasNarrow ? 192 : V2_B>(a, splitk_ws, st);
    }
    return launch_gemm_bf16_v2_nw<A_KC, B_KC, EPI, 8>(a, splitk_ws, st);
  }
  return launch_gemm_bf16_v2_nw<A_KC, B_KC, EPI, 4>(a, splitk_ws, st);
}

}  // namespace mlm
