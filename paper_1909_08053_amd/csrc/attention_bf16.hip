// bf16 MFMA attention over a shard's local heads (gfx950): forward with a streaming softmax, and a
// two-kernel backward (dQ per query block; dK/dV per key block) that recomputes the probabilities from
// the saved log-sum-exp.  Nothing of size s x s touches HBM and no atomics are used, so results are
// deterministic.
//
// Layout trick shared by the three kernels: score tiles are computed TRANSPOSED relative to the row that a
// wave owns, so that v_mfma_f32_32x32x16_bf16 leaves, in every lane, 16 score values that all belong to ONE
// owned row (a query in forward / dQ, a key in dK/dV).  Row statistics (max, sum, lse, delta) are then
// per-lane scalars (plus one cross-half shuffle), and the probability registers are already in the operand
// layout of the second MFMA (k index = the other sequence axis) -- P never goes through LDS.  The streamed
// tiles (K, V, Q, dO) are copied HBM -> LDS asynchronously, several tiles ahead, and an operand that must be read
// with k along the sequence axis is fetched from the same LDS tile with the transposing read instruction.
//
// Mask: allowed(i, j) = (j < key_len[b]) && (!causal || j <= i); excluded entries get probability exactly 0.
//
// Dropout of the probabilities (DROP instantiations): the forward kernel draws the keep decision of element
// ((batch, head, i), j) from the counter-based generator -- a lane's 16 scores of a 32-key half tile are four runs of
// four consecutive keys, i.e. four generator blocks -- zeroes the dropped probabilities before the second MFMA, folds
// 1 / (1 - p) into the final normalisation and saves the decisions as one bit per key.  The row sum and the
// log-sum-exp stay those of the undropped scores.  The backward kernels read the saved bits instead of running the
// generator again: dQ loads its query row's two words per tile, dK/dV gets the tile's 64 x 128-bit block through the
// DMA ring.  delta = rowsum(dO o O) needs no change: O already contains the dropout.
#include "lds_dma.h"
#include "rng.h"

namespace mlm {

constexpr int ATILE = 64;           // rows of the streamed tile (keys in fwd/dQ, queries in dK/dV)
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

constexpr int ANW = 4;              // waves per workgroup: 32 owned rows each
constexpr int ANT = ANW * 64;

// Workgroup id -> (block along the sequence, local head, batch).  Workgroups are handed to the eight XCDs round-robin
// by id and every XCD has its own L2, so the (batch, head) index takes the low three bits of the id: all sequence
// blocks of one (batch, head) pair -- they stream the same K / V (or Q / dO) rows -- run on ONE XCD and re-read those
// rows from its L2 (x-fastest ids put the eight blocks of a pair on eight XCDs and every XCD fetched every pair).
// Within an XCD the ids keep the sequence block as the faster index, so the longest causal blocks still start first.
// Grid: attn_grid(nx, hl, b) workgroups in x; ids whose pair does not exist (hl b not a multiple of 8) exit at once.
struct AttnBlock { int xb, hd, bi; bool valid; };
__device__ __forceinline__ AttnBlock attn_block(int nx, int hl, int b) {
  const int id = blockIdx.x, r = id >> 3;
  const int bh = (r / nx) * 8 + (id & 7);
  AttnBlock o;
  o.xb = r % nx;
  o.valid = bh < hl * b;
  o.hd = bh % hl;
  o.bi = bh / hl;
  return o;
}
static inline dim3 attn_grid(int nx, int hl, int b) { return dim3(8 * nx * ((hl * b + 7) / 8)); }

__device__ __forceinline__ bf16x8 pack8(const floatx16& v, int off) {
  bf16x8 r;
#pragma unroll
  for (int e = 0; e < 8; ++e) r[e] = (bf16)v[off + e];
  return r;
}

// ---- streamed [64][D] bf16 tiles copied HBM -> LDS by the DMA path -------------------------------------------
// A tile is 64 rows of U = D/8 16-byte units, stored densely (the copy writes 1 KB per wave instruction in lane
// order) with the unit index XOR-swizzled per row, so that both kinds of operand read are bank-conflict free:
//   * "kc" fragments (contraction along D: 16 lanes read one 16-byte unit of 16 consecutive rows), and
//   * transposing reads (contraction along the tile's rows: 32 lanes read 64 bytes of 4 consecutive rows).
template <int D>
struct ATile {
  static constexpr int U = D / 8;
  static constexpr int BYTES = ATILE * D * 2;
  static constexpr int QPW = U / ANW;              // 1-KB copies per wave and tile
  static_assert(U % ANW == 0 && (U == 8 || U == 12 || U == 16 || U == 24), "head size");
  __device__ static __forceinline__ int sw(int row) {
    if (U == 16) return ((row & 3) << 2) | ((row >> 2) & 3);
    if (U == 12) return (row >> 2) & 3;
    return (((row >> 1) & 1) << 2) | ((row >> 2) & 3);   // U = 8 and U = 24: the row stride is 8 units mod 16
  }
  // operand with k along D: 8 consecutive elements [16 ks + 8 lh, +8) of row r0 + l32
  __device__ static __forceinline__ bf16x8 frag_kc(const unsigned char* tile, int r0, int ks, int lane) {
    const int row = r0 + (lane & 31), c = 2 * ks + (lane >> 5);
    return *reinterpret_cast<const bf16x8*>(tile + row * (U * 16) + ((c ^ sw(row)) << 4));
  }
  // operand with k along the tile's rows, for column d0 + l32: k-slot (lh, e) <-> row 16 c4 + 8 (e/4) + 4 lh + e%4,
  // which is how a transposed score accumulator lays out its rows
  __device__ static __forceinline__ bf16x8 frag_tr(const unsigned char* tile, int c4, int d0, int lane) {
    const int g = lane >> 4, j = lane & 15;
    const int col = d0 + 16 * (g & 1) + 4 * (j & 3);
    const int cu = col >> 3, half = (col >> 2) & 1;
    v4s_t h[2];
#pragma unroll
    for (int r = 0; r < 2; ++r) {
      const int row = 16 * c4 + 4 * (g >> 1) + 8 * r + (j >> 2);
      h[r] = lds_read_tr16(tile + row * (U * 16) + ((cu ^ sw(row)) << 4) + half * 8);
    }
    const v8s_t v = __builtin_shufflevector(h[0], h[1], 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
  }
};

// Which 16 bytes of a tile each lane copies (fixed per lane), and the copy of one tile.
template <int D>
struct ATileSrc {
  typedef ATile<D> TL;
  int row[TL::QPW], col[TL::QPW];
  __device__ __forceinline__ void init(int wave, int lane) {
#pragma unroll
    for (int i = 0; i < TL::QPW; ++i) {
      const int u = 64 * (wave * TL::QPW + i) + lane;
      row[i] = u / TL::U;
      col[i] = ((u % TL::U) ^ TL::sw(row[i])) * 8;
    }
  }
  // P: element (0, 0) of the streamed matrix (row stride ld); rows beyond nrows - 1 re-read the last row (callers mask)
  __device__ __forceinline__ void issue_one(const bf16* P, int ld, int row0, int nrows, uint32_t lds_tile, int wave_u, int i) const {
    dma16(P + (size_t)min(row0 + row[i], nrows - 1) * ld + col[i], lds_tile + (wave_u * TL::QPW + i) * 1024);
  }
  __device__ __forceinline__ void issue(const bf16* P, int ld, int row0, int nrows, uint32_t lds_tile, int wave_u) const {
#pragma unroll
    for (int i = 0; i < TL::QPW; ++i)
      dma16(P + (size_t)min(row0 + row[i], nrows - 1) * ld + col[i], lds_tile + (wave_u * TL::QPW + i) * 1024);
  }
};

// ------------------------------------------------------------------------------------------ forward
// Workgroup = 128 queries of one (batch, head), 4 waves of 32 queries.  K and V tiles of 64 keys stream through a
// three-stage LDS ring filled by DMA two tiles ahead; per tile: S^T = K Q^T (12 MFMAs at d = 96), online softmax in
// registers, O^T += V^T P^T with V read through the transposing LDS loads (12 MFMAs).  One barrier per tile.
// Forward and dQ run TWO wave groups (8 waves) per 128 owned rows: group g takes the streamed tiles 2j + g, each
// group has its own DMA ring, and the groups' partial results are merged through LDS at the end.  That halves the
// serial chain of the longest (causal) blocks and puts two waves on every SIMD, so one wave's exp2 / VALU work
// overlaps the other's MFMAs.  Ring stages per group: 3, or 2 at d = 128 (LDS budget).  d = 192 keeps ONE group: its
// 24-KB tiles leave no LDS for a second ring, and its accumulators need more than the 256 registers per lane that
// two waves per SIMD allow.
template <int D> constexpr int attn_groups() { return D > 128 ? 1 : 2; }
template <int D> constexpr int group_stages() { return D == 128 ? 2 : 3; }
template <int D> constexpr int dkv_dsplit() { return D >= 128 ? 2 : 1; }
// dK/dV: two wave groups (alternate query tiles, merged through LDS at the end) for the head sizes whose registers
// allow two waves per SIMD once the wave's own K / V rows are kept in LDS instead of registers; ring stages per group
// by the LDS budget (rings + the 128 owned K and V rows).
template <int D> constexpr int dkv_groups() { return D <= 128 ? 2 : 1; }
template <int D> constexpr int dkv_stages() { return (D == 96 || D == 128) ? 2 : 3; }
template <int D> constexpr bool dkv_own_lds() { return D <= 96; }    // d = 128: half the D columns per workgroup, rows stay in registers

// (two waves per SIMD requested: with at most 256 registers per lane the MFMA accumulators live in ordinary VGPRs, so
// the softmax arithmetic needs no accumulator-register moves)
template <int D, bool DROP>
__global__ __launch_bounds__(attn_groups<D>() * ANT) void attn_fwd_bf16_kernel(AttnArgs a) {
  typedef ATile<D> TL;
  constexpr int BQ = 32 * ANW, STAGE = 2 * TL::BYTES, LPT = 2 * TL::QPW;   // LPT: copies per tile and wave (K + V)
  constexpr int NST = group_stages<D>(), NG = attn_groups<D>();
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, lh = lane >> 5;
  // wave-uniform values must be known as such: the mask test below is a scalar branch
  const int grp = NG == 1 ? 0 : __builtin_amdgcn_readfirstlane(tid >> 8);    // wave group: 0 takes the even tiles, 1 the odd tiles
  const int wave = __builtin_amdgcn_readfirstlane((tid >> 6) & 3);   // wave inside its group: 32 queries
  const int wave_u = wave;
  const int nqb = (a.s + BQ - 1) / BQ;
  const AttnBlock blk = attn_block(nqb, a.hl, a.b);
  if (!blk.valid) return;
  const int qb = nqb - 1 - blk.xb;                // longest (causal) blocks first
  const int hd = blk.hd, bi = blk.bi;
  const int ld = 3 * a.hl * D;
  const bf16* base = (const bf16*)a.qkv + (size_t)bi * a.s * ld;
  const int klen = attn_key_len(a.key_len, bi, a.s);
  const int q0 = qb * BQ, qw0 = q0 + wave * 32, qi = qw0 + l32;

  bf16x8 qf[D / 16];
  {
    const bf16* qrow = base + (size_t)min(qi, a.s - 1) * ld + hd * D;
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) qf[ks] = *reinterpret_cast<const bf16x8*>(qrow + ks * 16 + lh * 8);
  }
  floatx16 o[D / 32];
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int e = 0; e < 16; ++e) o[dt][e] = 0.f;
  float m = -INFINITY, lsum = 0.f;
  const size_t prow = ((size_t)bi * a.hl + hd) * a.s + min(qi, a.s - 1);   // row of the [b, hl, s, s] probabilities
  int kv_end = klen;
  if (a.causal) kv_end = min(kv_end, q0 + BQ);
  const int nt = (kv_end + ATILE - 1) / ATILE;
  const float sc = kLog2e / sqrtf((float)D);
  const bf16* Kb = base + (a.hl + hd) * D;
  const bf16* Vb = base + (2 * a.hl + hd) * D;
  ATileSrc<D> src;
  src.init(wave, lane);
  unsigned char* ring = lds_raw + grp * (NST * STAGE);   // this group's ring
  const uint32_t lds0 = lds_offset_of(ring);
  const int njt = (nt + NG - 1) / NG;              // steps: group g handles tile NG j + g in step j (if it exists)
  // The ring is always kept full: past the last tile the copies re-read tile nt - 1 into a stage nobody reads, so
  // the outstanding-copy count is the same in every iteration.
#pragma unroll
  for (int t = 0; t < NST - 1; ++t) {
    const int tc = min(NG * t + grp, nt - 1) * ATILE;
    src.issue(Kb, ld, tc, a.s, lds0 + t * STAGE, wave_u);
    src.issue(Vb, ld, tc, a.s, lds0 + t * STAGE + TL::BYTES, wave_u);
  }
  int stage = 0;
  for (int j = 0; j < njt; ++j) {
    const int t = NG * j + grp;
    const int k0 = t * ATILE;
    wait_vmcnt<LPT*(NST - 2)>();                   // this wave's copies of step j have landed; step j + 1 may be in flight
    __builtin_amdgcn_s_barrier();                 // everyone's have; and everyone is done with step j - 1
    // The copies that re-arm the stage of step j - 1 (= stage of step j + NST - 1) are NOT issued here in one burst:
    // all eight waves leave the barrier together, 48 one-KB copies queue in the CU's address unit and every wave sits
    // in front of its first fragment read for 0.6 us of a 2-us step (in-kernel timestamps).  They are issued one at
    // a time between the exponentials below, where the wave has no LDS read in flight that the copy's compiler-level
    // memory barrier would pin (placed behind the MFMAs of the two products instead, it measured no gain: 24.9 against
    // 23.5 us).  Head sizes above 96 keep the burst: the longer live ranges cost them registers they do not have.
    const int pst = stage == 0 ? NST - 1 : stage - 1;
    const int tc_next = min(t + NG * (NST - 1), nt - 1) * ATILE;
    const uint32_t dstK = lds0 + pst * STAGE, dstV = dstK + TL::BYTES;
    const unsigned char* sK = ring + stage * STAGE;
    const unsigned char* sV = sK + TL::BYTES;
    stage = stage == NST - 1 ? 0 : stage + 1;
    constexpr bool SPREAD = D <= 96;
    const bool live = t < nt && !(a.causal && k0 > qw0 + 31);   // else: no such tile / entirely above this wave's diagonal (wave-uniform)
    if (!SPREAD || !live) {
      src.issue(Kb, ld, tc_next, a.s, dstK, wave_u);
      src.issue(Vb, ld, tc_next, a.s, dstV, wave_u);
    }
    if (!live) continue;
    floatx16 sacc[2];
    float lsum_t = 0.f;
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int e = 0; e < 16; ++e) sacc[kt][e] = 0.f;
    // the two 32-key halves are independent accumulation chains: alternate them so that a dependent MFMA never
    // follows its predecessor directly
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks)
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
        sacc[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(TL::frag_kc(sK, kt * 32, ks, lane), qf[ks], sacc[kt], 0, 0, 0);
    // raw scores s; probabilities p = exp2(s * sc - max) with the scale folded into one fma per element
    const bool need_mask = (a.causal && k0 + ATILE - 1 > qw0) || (k0 + ATILE > klen);   // wave-uniform
    float mt = -INFINITY;
    if (need_mask) {
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int key = k0 + kt * 32 + 8 * (e >> 2) + 4 * lh + (e & 3);
          const bool off = key >= klen || (a.causal && key > qi);
          sacc[kt][e] = off ? -INFINITY : sacc[kt][e];
          mt = fmaxf(mt, sacc[kt][e]);
        }
    } else {
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int e = 0; e < 16; ++e) mt = fmaxf(mt, sacc[kt][e]);
    }
    mt = fmaxf(mt, __shfl_xor(mt, 32, 64)) * sc;
    const float mn = fmaxf(m, mt);               // finite from the first tile on: key 0 is allowed for every query
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const float p = __builtin_amdgcn_exp2f(fmaf(sacc[kt][e], sc, -mn));
        sacc[kt][e] = p;
        lsum_t += p;
        if (SPREAD) {
#pragma unroll
          for (int c = 0; c < LPT; ++c)                    // copy c after element (32 c + 16) / LPT of the 32
            if (kt * 16 + e == (32 * c + 16) / LPT) {
              if (c < TL::QPW) src.issue_one(Kb, ld, tc_next, a.s, dstK, wave_u, c);
              else src.issue_one(Vb, ld, tc_next, a.s, dstV, wave_u, c - TL::QPW);
            }
        }
      }
    // rescale the running sums only when some row's maximum moved (wave-uniform test)
    if (__builtin_amdgcn_ballot_w64(mn > m) != 0) {
      const float corr = __builtin_amdgcn_exp2f(m - mn);
      lsum *= corr;
#pragma unroll
      for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[dt][e] *= corr;
      m = mn;
    }
    lsum += lsum_t;
    if (DROP) {
#pragma unroll
      for (int kt = 0; kt < 2; ++kt) {
        uint32_t word = 0;                       // this lane's 16 of the 32 keep bits of keys k0 + 32 kt ..
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const uint32_t k4 = drop_keep4(a.drop, (prow * a.s + k0 + kt * 32 + 8 * g + 4 * lh) >> 2);
#pragma unroll
          for (int e = 0; e < 4; ++e) sacc[kt][4 * g + e] = ((k4 >> e) & 1u) ? sacc[kt][4 * g + e] : 0.f;
          word |= k4 << (8 * g + 4 * lh);
        }
        word |= __shfl_xor(word, 32, 64);        // the other half-wave holds the other 16 bits
        if (lh == kt && qi < a.s) a.keep_bits[prow * a.keep_pitch + (k0 >> 5) + kt] = word;
      }
    }
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const bf16x8 pf = pack8(sacc[c >> 1], 8 * (c & 1));
#pragma unroll
      for (int dt = 0; dt < D / 32; ++dt)
        o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(TL::frag_tr(sV, c, dt * 32, lane), pf, o[dt], 0, 0, 0);
    }
  }
  wait_vmcnt<0>();                                // copies still in flight target this workgroup's LDS
  // merge the two groups' (m, l, O): group 1 parks its values in LDS ([wave][value][lane]: conflict-free)
  if (NG == 2) {
    __syncthreads();
    constexpr int NR = D / 2 + 2;
    float* park = reinterpret_cast<float*>(lds_raw) + (size_t)wave * NR * 64 + lane;
    if (grp == 1) {
#pragma unroll
      for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
        for (int e = 0; e < 16; ++e) park[(dt * 16 + e) * 64] = o[dt][e];
      park[(D / 2) * 64] = m;
      park[(D / 2 + 1) * 64] = lsum;
    }
    __syncthreads();
    if (grp == 1) return;
    const float m1 = park[(D / 2) * 64], l1 = park[(D / 2 + 1) * 64];
    const float mn = fmaxf(m, m1);                // group 0 always has tile 0: finite
    const float c0 = __builtin_amdgcn_exp2f(m - mn), c1 = __builtin_amdgcn_exp2f(m1 - mn);
    lsum = lsum * c0 + l1 * c1;
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
      for (int e = 0; e < 16; ++e) o[dt][e] = o[dt][e] * c0 + park[(dt * 16 + e) * 64] * c1;
    m = mn;
  }
  lsum += __shfl_xor(lsum, 32, 64);
  if (qi < a.s) {
    const float inv = (DROP ? a.drop.scale : 1.0f) / lsum;
    bf16* crow = (bf16*)a.ctx + ((size_t)bi * a.s + qi) * (a.hl * D) + hd * D;
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        bf16x4 ov;
#pragma unroll
        for (int e = 0; e < 4; ++e) ov[e] = (bf16)(o[dt][4 * g + e] * inv);
        *reinterpret_cast<bf16x4*>(crow + dt * 32 + 8 * g + 4 * lh) = ov;
      }
    if (lh == 0) a.lse[((size_t)bi * a.hl + hd) * a.s + qi] = (m + log2f(lsum)) * kLn2;
  }
}

// ------------------------------------------------------------------------------------------ backward: dQ
// Same streaming structure as the forward kernel.  Per tile: S^T = K Q^T and dP^T = V dO^T (contraction along D),
// P = exp2(S sc - lse), dS = P o (dP - delta), dQ^T += K^T dS^T with K read a second time through the transposing
// loads.  delta_i = sum_d dO_id O_id is computed here from the rows the lanes already hold and stored for the
// dK/dV kernel, which runs after this one.
template <int D, bool DROP>
__global__ __launch_bounds__(attn_groups<D>() * ANT) void attn_bwd_dq_bf16_kernel(AttnArgs a) {
  typedef ATile<D> TL;
  constexpr int BQ = 32 * ANW, STAGE = 2 * TL::BYTES, LPT = 2 * TL::QPW, NST = group_stages<D>(), NG = attn_groups<D>();
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, lh = lane >> 5;
  const int grp = NG == 1 ? 0 : __builtin_amdgcn_readfirstlane(tid >> 8);   // wave group: even / odd tiles
  const int wave = __builtin_amdgcn_readfirstlane((tid >> 6) & 3);   // wave inside its group (uniform: scalar mask branches)
  const int nqb = (a.s + BQ - 1) / BQ;
  const AttnBlock blk = attn_block(nqb, a.hl, a.b);
  if (!blk.valid) return;
  const int qb = nqb - 1 - blk.xb;
  const int hd = blk.hd, bi = blk.bi;
  const int ld = 3 * a.hl * D;
  const bf16* base = (const bf16*)a.qkv + (size_t)bi * a.s * ld;
  const int klen = attn_key_len(a.key_len, bi, a.s);
  const int q0 = qb * BQ, qw0 = q0 + wave * 32, qi = qw0 + l32;
  const int qc = min(qi, a.s - 1);

  bf16x8 qf[D / 16], dof[D / 16];
  float dl = 0.f;
  {
    const bf16* qrow = base + (size_t)qc * ld + hd * D;
    const bf16* drow = (const bf16*)a.dctx + ((size_t)bi * a.s + qc) * (a.hl * D) + hd * D;
    const bf16* orow = (const bf16*)a.ctx + ((size_t)bi * a.s + qc) * (a.hl * D) + hd * D;
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) {
      qf[ks] = *reinterpret_cast<const bf16x8*>(qrow + ks * 16 + lh * 8);
      dof[ks] = *reinterpret_cast<const bf16x8*>(drow + ks * 16 + lh * 8);
      const bf16x8 of = *reinterpret_cast<const bf16x8*>(orow + ks * 16 + lh * 8);
#pragma unroll
      for (int e = 0; e < 8; ++e) dl = fmaf((float)dof[ks][e], (float)of[e], dl);
    }
    dl += __shfl_xor(dl, 32, 64);
  }
  const float lse2 = a.lse[((size_t)bi * a.hl + hd) * a.s + qc] * kLog2e;
  const uint32_t* kbrow = DROP ? a.keep_bits + (((size_t)bi * a.hl + hd) * a.s + qc) * a.keep_pitch : nullptr;
  if (grp == 0 && lh == 0 && qi < a.s) {          // for the dK/dV kernel: [0] delta, [1] log-sum-exp in log2 units
    a.delta[((size_t)bi * a.hl + hd) * a.s + qi] = dl;
    a.delta[(size_t)a.b * a.hl * a.s + ((size_t)bi * a.hl + hd) * a.s + qi] = lse2;
  }
  floatx16 dq[D / 32];
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int e = 0; e < 16; ++e) dq[dt][e] = 0.f;
  int kv_end = klen;
  if (a.causal) kv_end = min(kv_end, q0 + BQ);
  const int nt = (kv_end + ATILE - 1) / ATILE;
  const float scale = 1.0f / sqrtf((float)D);
  const float sc = kLog2e * scale;
  const bf16* Kb = base + (a.hl + hd) * D;
  const bf16* Vb = base + (2 * a.hl + hd) * D;
  ATileSrc<D> src;
  src.init(wave, lane);
  unsigned char* ring = lds_raw + grp * (NST * STAGE);
  const uint32_t lds0 = lds_offset_of(ring);
  const int njt = (nt + NG - 1) / NG;
#pragma unroll
  for (int t = 0; t < NST - 1; ++t) {
    const int tc = min(NG * t + grp, nt - 1) * ATILE;
    src.issue(Kb, ld, tc, a.s, lds0 + t * STAGE, wave);
    src.issue(Vb, ld, tc, a.s, lds0 + t * STAGE + TL::BYTES, wave);
  }
  int stage = 0;
  for (int j = 0; j < njt; ++j) {
    const int t = NG * j + grp;
    const int k0 = t * ATILE;
    wait_vmcnt<LPT*(NST - 2)>();
    __builtin_amdgcn_s_barrier();
    // the copies that re-arm the stage of step j - 1 are issued one at a time inside the element-wise pass below
    // (as in the forward kernel: a burst here holds every wave of the CU in front of its first fragment read)
    constexpr bool SPREAD = D <= 96;
    const int pst = stage == 0 ? NST - 1 : stage - 1;
    const int tc_next = min(t + NG * (NST - 1), nt - 1) * ATILE;
    const uint32_t dstK = lds0 + pst * STAGE, dstV = dstK + TL::BYTES;
    auto copy_after = [&](int el) {                  // el: element index 0..31 of the pass (compile time after unrolling)
#pragma unroll
      for (int c = 0; c < LPT; ++c)
        if (el == (32 * c + 16) / LPT) {
          if (c < TL::QPW) src.issue_one(Kb, ld, tc_next, a.s, dstK, wave, c);
          else src.issue_one(Vb, ld, tc_next, a.s, dstV, wave, c - TL::QPW);
        }
    };
    const unsigned char* sK = ring + stage * STAGE;
    const unsigned char* sV = sK + TL::BYTES;
    stage = stage == NST - 1 ? 0 : stage + 1;
    const bool live = t < nt && !(a.causal && k0 > qw0 + 31);
    if (!SPREAD || !live) {
      src.issue(Kb, ld, tc_next, a.s, dstK, wave);
      src.issue(Vb, ld, tc_next, a.s, dstV, wave);
    }
    if (!live) continue;
    uint2 kw = make_uint2(0xFFFFFFFFu, 0xFFFFFFFFu);          // keep bits of this query row, keys k0 .. k0 + 63
    if (DROP) kw = *reinterpret_cast<const uint2*>(kbrow + (k0 >> 5));
    floatx16 sacc[2], pacc[2];
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int e = 0; e < 16; ++e) { sacc[kt][e] = 0.f; pacc[kt][e] = 0.f; }
    // four independent accumulation chains, interleaved
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks)
#pragma unroll
      for (int kt = 0; kt < 2; ++kt) {
        sacc[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(TL::frag_kc(sK, kt * 32, ks, lane), qf[ks], sacc[kt], 0, 0, 0);   // S^T[key][query]
        pacc[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(TL::frag_kc(sV, kt * 32, ks, lane), dof[ks], pacc[kt], 0, 0, 0);  // dP^T[key][query]
      }
    const bool need_mask = (a.causal && k0 + ATILE - 1 > qw0) || (k0 + ATILE > klen);   // wave-uniform
    if (DROP) {
      // gradient w.r.t. the undropped probability: keep o dP / (1 - p)
#pragma unroll
      for (int kt = 0; kt < 2; ++kt) {
        const uint32_t w = (kt == 0 ? kw.x : kw.y) >> (4 * lh);
#pragma unroll
        for (int e = 0; e < 16; ++e)
          pacc[kt][e] = ((w >> (8 * (e >> 2) + (e & 3))) & 1u) ? pacc[kt][e] * a.drop.scale : 0.f;
      }
    }
    if (need_mask) {
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int key = k0 + kt * 32 + 8 * (e >> 2) + 4 * lh + (e & 3);
          const bool off = key >= klen || (a.causal && key > qi);
          const float p = off ? 0.f : __builtin_amdgcn_exp2f(fmaf(sacc[kt][e], sc, -lse2));
          sacc[kt][e] = p * (pacc[kt][e] - dl);     // dS^T
          if (SPREAD) copy_after(kt * 16 + e);
        }
    } else {
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          sacc[kt][e] = __builtin_amdgcn_exp2f(fmaf(sacc[kt][e], sc, -lse2)) * (pacc[kt][e] - dl);
          if (SPREAD) copy_after(kt * 16 + e);
        }
    }
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const bf16x8 dsf = pack8(sacc[c >> 1], 8 * (c & 1));
#pragma unroll
      for (int dt = 0; dt < D / 32; ++dt)
        dq[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(TL::frag_tr(sK, c, dt * 32, lane), dsf, dq[dt], 0, 0, 0);   // dQ^T[dcol][query]
    }
  }
  wait_vmcnt<0>();
  // dQ = group 0's sum + group 1's sum (group 1 parks its accumulators in LDS: [wave][value][lane])
  if (NG == 2) {
    __syncthreads();
    float* park = reinterpret_cast<float*>(lds_raw) + (size_t)wave * (D / 2) * 64 + lane;
    if (grp == 1) {
#pragma unroll
      for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
        for (int e = 0; e < 16; ++e) park[(dt * 16 + e) * 64] = dq[dt][e];
    }
    __syncthreads();
    if (grp == 1) return;
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
      for (int e = 0; e < 16; ++e) dq[dt][e] += park[(dt * 16 + e) * 64];
  }
  if (qi < a.s) {
    bf16* orow = (bf16*)a.dqkv + ((size_t)bi * a.s + qi) * ld + hd * D;
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        bf16x4 ov;
#pragma unroll
        for (int e = 0; e < 4; ++e) ov[e] = (bf16)(dq[dt][4 * g + e] * scale);
        *reinterpret_cast<bf16x4*>(orow + dt * 32 + 8 * g + 4 * lh) = ov;
      }
  }
}

// ------------------------------------------------------------------------------------------ backward: dK, dV
// Workgroup = 128 keys of one (batch, head), a wave owns 32 keys.  Q and dO tiles of 64 queries stream through the DMA
// ring together with the tile's log-sum-exp (log2 units) and delta vectors, which the dQ kernel left in the workspace.
// Per 32-query half tile: S = Q K^T and dP = dO V^T (contraction along D), P = exp2(S sc - lse), dS = P o (dP - delta),
// then dV^T += dO^T P and dK^T += Q^T dS with Q and dO read a second time through the transposing loads.
// Head sizes up to 96 run TWO wave groups (8 waves, two per SIMD): group g takes the query tiles 2 j + g through its own
// ring and the groups' dK / dV sums are added through LDS at the end, which halves the serial chain of the key blocks
// with the most queries (for causal masks block 0 streams every query tile and sets the kernel's duration).  Two waves
// per SIMD leave 256 registers per lane, so the wave's own K and V rows are not held in registers there: the block's
// 128 K and V rows are copied to LDS once and their fragments are read per use.
// Larger heads keep one group (their accumulators alone need more registers) and split the D columns of dK / dV over
// two workgroups instead.
template <int D, bool DROP>
__global__ __launch_bounds__(dkv_groups<D>() * ANT) void attn_bwd_dkv_bf16_kernel(AttnArgs a) {
  typedef ATile<D> TL;
  constexpr int BKB = 32 * ANW, VEC = 2 * ATILE * 4;          // VEC: bytes of the lse + delta vectors of a tile
  constexpr int KBB = DROP ? ATILE * 16 : 0;                  // keep bits of the tile: 64 queries x 128 keys
  constexpr int STAGE = 2 * TL::BYTES + VEC + KBB, LPT = 2 * TL::QPW + 1 + (DROP ? 1 : 0);
  constexpr int NG = dkv_groups<D>(), NST = dkv_stages<D>();
  constexpr bool OWN_LDS = NG == 2 && dkv_own_lds<D>();        // own K / V rows in LDS (after the rings)
  // Large heads: the dK / dV accumulators of all D columns plus the owned K / V rows do not fit the register file
  // (they spilled: 2.3x / 5.6x the d = 96 time at d = 128 / 192).  Two workgroups then share a key block, each
  // accumulating one half of the D columns of dK and dV (the scores are computed by both); this also doubles the
  // number of workgroups where a shard has few heads.
  constexpr int DS = dkv_dsplit<D>(), DH = D / DS;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, lh = lane >> 5;
  // known wave-uniform: mask tests become scalar branches
  const int grp = NG == 1 ? 0 : __builtin_amdgcn_readfirstlane(tid >> 8);   // wave group: even / odd query tiles
  const int wave = __builtin_amdgcn_readfirstlane((tid >> 6) & 3);         // wave inside its group: 32 keys
  const AttnBlock blk = attn_block(((a.s + 32 * ANW - 1) / (32 * ANW)) * DS, a.hl, a.b);
  if (!blk.valid) return;
  const int kb = blk.xb / DS;                      // key block; for causal, block 0 has the most queries: first
  const int dh0 = (blk.xb % DS) * DH;              // first of this workgroup's dK / dV columns
  const int hd = blk.hd, bi = blk.bi;
  const int ld = 3 * a.hl * D;
  const bf16* base = (const bf16*)a.qkv + (size_t)bi * a.s * ld;
  const int klen = attn_key_len(a.key_len, bi, a.s);
  const int kb0 = kb * BKB, kw0 = kb0 + wave * 32, kj = kw0 + l32;
  const int kc = min(kj, a.s - 1);
  ATileSrc<D> src;
  src.init(wave, lane);
  const uint32_t lds0 = lds_offset_of(lds_raw);

  // the block's own K and V rows: registers (one group) or two 64-row tiles each in LDS (two groups; rows past the
  // end of the sequence repeat the last row, exactly as the register path clamps them)
  bf16x8 kf[OWN_LDS ? 1 : D / 16], vf[OWN_LDS ? 1 : D / 16];
  const unsigned char* ownK = lds_raw + NG * NST * STAGE;
  const unsigned char* ownV = ownK + 2 * TL::BYTES;
  if (OWN_LDS) {
    // group 0 copies the K rows, group 1 the V rows (two tiles of 64 rows each)
    const bf16* P = base + ((grp == 0 ? a.hl : 2 * a.hl) + hd) * D;
    const uint32_t dst = lds0 + NG * NST * STAGE + grp * 2 * TL::BYTES;
    src.issue(P, ld, kb0, a.s, dst, wave);
    src.issue(P, ld, kb0 + ATILE, a.s, dst + TL::BYTES, wave);
  } else {
    const bf16* krow = base + (size_t)kc * ld + (a.hl + hd) * D;
    const bf16* vrow = base + (size_t)kc * ld + (2 * a.hl + hd) * D;
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) {
      kf[ks] = *reinterpret_cast<const bf16x8*>(krow + ks * 16 + lh * 8);
      vf[ks] = *reinterpret_cast<const bf16x8*>(vrow + ks * 16 + lh * 8);
    }
  }
  const unsigned char* myK = ownK + (wave >> 1) * TL::BYTES;   // the tile that holds this wave's 32 rows, at (wave & 1) 32
  const unsigned char* myV = ownV + (wave >> 1) * TL::BYTES;
  const int own_r0 = (wave & 1) * 32;
  floatx16 dk[DH / 32], dv[DH / 32];
#pragma unroll
  for (int dt = 0; dt < DH / 32; ++dt)
#pragma unroll
    for (int e = 0; e < 16; ++e) { dk[dt][e] = 0.f; dv[dt][e] = 0.f; }
  const float scale = 1.0f / sqrtf((float)D);
  const float sc = kLog2e * scale;
  const int nqt = (a.s + ATILE - 1) / ATILE;
  int qt0 = a.causal ? kb0 / ATILE : 0;
  if (kb0 >= klen) qt0 = nqt;                     // every key of the block is padding: gradients are zero
  const int nt = nqt - qt0;                       // tiles to stream (block-uniform)
  const int njt = (nt + NG - 1) / NG;             // steps: group g handles tile NG j + g in step j (if it exists)
  const bf16* Qb = base + hd * D;
  const int ldo = a.hl * D;
  const bf16* dOb = (const bf16*)a.dctx + (size_t)bi * a.s * ldo + hd * D;
  // per-query vectors in the workspace: [0] delta, [1] log-sum-exp in log2 units (both written by the dQ kernel)
  const size_t nrow_all = (size_t)a.b * a.hl * a.s;
  const float* vec_b = ((wave & 1) ? a.delta + nrow_all : a.delta) + ((size_t)bi * a.hl + hd) * a.s;
  unsigned char* ring = lds_raw + grp * (NST * STAGE);        // this group's ring
  const uint32_t ring0 = lds0 + grp * (NST * STAGE);
  auto issue_tile = [&](int t, int st) {          // tile index relative to qt0 (clamped), ring stage
    const int r0 = (qt0 + min(t, nt - 1)) * ATILE;
    const uint32_t sb = ring0 + st * STAGE;
    src.issue(Qb, ld, r0, a.s, sb, wave);
    src.issue(dOb, ldo, r0, a.s, sb + TL::BYTES, wave);
    // waves 0, 2 copy the delta vector, waves 1, 3 the log-sum-exp vector (same data twice: uniform copy counts)
    dma4(vec_b + min(r0 + lane, a.s - 1), sb + 2 * TL::BYTES + (wave & 1) * (ATILE * 4));
    if (DROP) {
      // lane t copies the four words of query r0 + t that cover this block's 128 keys (every wave copies the same
      // kilobyte: uniform copy counts)
      const uint32_t* src_bits = a.keep_bits + (((size_t)bi * a.hl + hd) * a.s + min(r0 + lane, a.s - 1)) * a.keep_pitch +
                                 (kb0 >> 5);
      dma16(reinterpret_cast<const bf16*>(src_bits), sb + 2 * TL::BYTES + VEC);
    }
  };
  if (nt > 0) {
#pragma unroll
    for (int t = 0; t < NST - 1; ++t) issue_tile(NG * t + grp, t);
  }
  int stage = 0;
  for (int j = 0; j < njt; ++j) {
    const int t = NG * j + grp;
    const int q0 = (qt0 + t) * ATILE;
    wait_vmcnt<LPT*(NST - 2)>();                   // this wave's copies of step j (and of the own rows) have landed
    __builtin_amdgcn_s_barrier();                 // everyone's have; and everyone is done with step j - 1
    // (issued in one burst: spreading these copies over the element-wise passes, as the forward and dQ kernels do,
    // measured slower here -- the passes read the per-query vectors from LDS and the copies' compiler-level memory
    // barrier pins those reads)
    issue_tile(t + NG * (NST - 1), stage == 0 ? NST - 1 : stage - 1);
    const unsigned char* sQ = ring + stage * STAGE;
    const unsigned char* sdO = sQ + TL::BYTES;
    const float* sDl = reinterpret_cast<const float*>(sdO + TL::BYTES);
    const float* sLse = sDl + ATILE;
    const uint32_t* sBits = reinterpret_cast<const uint32_t*>(sLse + ATILE);   // [64 queries][4 words]
    stage = stage == NST - 1 ? 0 : stage + 1;
    if (t >= nt || (a.causal && q0 + ATILE - 1 < kw0)) continue;   // no such tile / every query precedes this wave's keys
    const bool need_mask = (a.causal && q0 < kw0 + 31) || (kw0 + 32 > klen) || (q0 + ATILE > a.s);   // wave-uniform
#pragma unroll
    for (int qs = 0; qs < 2; ++qs) {
      floatx16 sacc, pacc;
#pragma unroll
      for (int e = 0; e < 16; ++e) { sacc[e] = 0.f; pacc[e] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < D / 16; ++ks) {
        const bf16x8 kk = OWN_LDS ? TL::frag_kc(myK, own_r0, ks, lane) : kf[OWN_LDS ? 0 : ks];
        const bf16x8 vv = OWN_LDS ? TL::frag_kc(myV, own_r0, ks, lane) : vf[OWN_LDS ? 0 : ks];
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(TL::frag_kc(sQ, qs * 32, ks, lane), kk, sacc, 0, 0, 0);    // S[query][key]
        pacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(TL::frag_kc(sdO, qs * 32, ks, lane), vv, pacc, 0, 0, 0);   // dP[query][key]
      }
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int qoff = qs * 32 + 8 * g + 4 * lh;
        const float4 l4 = *reinterpret_cast<const float4*>(sLse + qoff);
        const float4 d4 = *reinterpret_cast<const float4*>(sDl + qoff);
        const float lv4[4] = {l4.x, l4.y, l4.z, l4.w};
        const float dv4[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          float p = __builtin_amdgcn_exp2f(fmaf(sacc[4 * g + e], sc, -lv4[e]));
          if (need_mask) {
            const int q = q0 + qoff + e;
            p = (kj >= klen || q >= a.s || (a.causal && kj > q)) ? 0.f : p;
          }
          if (DROP) {
            const bool keep = (sBits[(qoff + e) * 4 + wave] >> l32) & 1u;
            sacc[4 * g + e] = keep ? p * a.drop.scale : 0.f;                                       // dropped P (for dV)
            pacc[4 * g + e] = p * ((keep ? pacc[4 * g + e] * a.drop.scale : 0.f) - dv4[e]);        // dS
          } else {
            sacc[4 * g + e] = p;                                // P
            pacc[4 * g + e] = p * (pacc[4 * g + e] - dv4[e]);   // dS
          }
        }
      }
#pragma unroll
      for (int cc = 0; cc < 2; ++cc) {
        const int c = 2 * qs + cc;
        const bf16x8 pf = pack8(sacc, 8 * cc);
        const bf16x8 dsf = pack8(pacc, 8 * cc);
#pragma unroll
        for (int dt = 0; dt < DH / 32; ++dt) {
          dv[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(TL::frag_tr(sdO, c, dh0 + dt * 32, lane), pf, dv[dt], 0, 0, 0);    // dV^T[dcol][key]
          dk[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(TL::frag_tr(sQ, c, dh0 + dt * 32, lane), dsf, dk[dt], 0, 0, 0);    // dK^T[dcol][key]
        }
      }
    }
  }
  wait_vmcnt<0>();
  // dK, dV = group 0's sums + group 1's sums (group 1 parks its accumulators in LDS: [wave][value][lane])
  if (NG == 2) {
    __syncthreads();
    constexpr int NV = 2 * (DH / 32) * 16;
    float* park = reinterpret_cast<float*>(lds_raw) + (size_t)wave * NV * 64 + lane;
    if (grp == 1) {
#pragma unroll
      for (int dt = 0; dt < DH / 32; ++dt)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          park[(dt * 16 + e) * 64] = dk[dt][e];
          park[((DH / 32 + dt) * 16 + e) * 64] = dv[dt][e];
        }
    }
    __syncthreads();
    if (grp == 1) return;
#pragma unroll
    for (int dt = 0; dt < DH / 32; ++dt)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        dk[dt][e] += park[(dt * 16 + e) * 64];
        dv[dt][e] += park[((DH / 32 + dt) * 16 + e) * 64];
      }
  }
  if (kj < a.s) {
    bf16* krow = (bf16*)a.dqkv + ((size_t)bi * a.s + kj) * ld + (a.hl + hd) * D;
    bf16* vrow = (bf16*)a.dqkv + ((size_t)bi * a.s + kj) * ld + (2 * a.hl + hd) * D;
#pragma unroll
    for (int dt = 0; dt < DH / 32; ++dt)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        bf16x4 ok, ov;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          ok[e] = (bf16)(dk[dt][4 * g + e] * scale);
          ov[e] = (bf16)dv[dt][4 * g + e];
        }
        *reinterpret_cast<bf16x4*>(krow + dh0 + dt * 32 + 8 * g + 4 * lh) = ok;
        *reinterpret_cast<bf16x4*>(vrow + dh0 + dt * 32 + 8 * g + 4 * lh) = ov;
      }
  }
}

// ------------------------------------------------------------------------------------------ launchers
bool attn_bf16_supported(int d) { return d == 64 || d == 96 || d == 128 || d == 192; }

template <int D, bool DROP>
static hipError_t launch_fwd_dd(const AttnArgs& a, hipStream_t st) {
  const size_t lds = (size_t)attn_groups<D>() * group_stages<D>() * 2 * ATile<D>::BYTES;
  if (lds > 64 * 1024) {
    hipError_t e = hipFuncSetAttribute((const void*)attn_fwd_bf16_kernel<D, DROP>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  const dim3 grid = attn_grid((a.s + 32 * ANW - 1) / (32 * ANW), a.hl, a.b);
  hipLaunchKernelGGL((attn_fwd_bf16_kernel<D, DROP>), grid, dim3(attn_groups<D>() * ANT), lds, st, a);
  return hipGetLastError();
}

template <int D>
static hipError_t launch_fwd_d(const AttnArgs& a, hipStream_t st) {
  return a.drop.enabled ? launch_fwd_dd<D, true>(a, st) : launch_fwd_dd<D, false>(a, st);
}

template <int D, bool DROP>
static hipError_t launch_bwd_dd(const AttnArgs& a, hipStream_t st) {
  const int nblk = (a.s + 32 * ANW - 1) / (32 * ANW);
  const dim3 grid = attn_grid(nblk, a.hl, a.b);
  const size_t lds_q = (size_t)attn_groups<D>() * group_stages<D>() * 2 * ATile<D>::BYTES;
  hipError_t e;
  if (lds_q > 64 * 1024) {
    e = hipFuncSetAttribute((const void*)attn_bwd_dq_bf16_kernel<D, DROP>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)lds_q);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL((attn_bwd_dq_bf16_kernel<D, DROP>), grid, dim3(attn_groups<D>() * ANT), lds_q, st, a);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  constexpr int NGK = dkv_groups<D>(), NSK = dkv_stages<D>();
  constexpr size_t kStageKv = 2 * ATile<D>::BYTES + 2 * ATILE * 4;
  // rings, the owned K / V rows (two groups), and at the end the parked accumulators of group 1
  constexpr size_t kOwn = (NGK == 2 && dkv_own_lds<D>()) ? 4 * ATile<D>::BYTES : 0;
  constexpr size_t kPark = NGK == 2 ? (size_t)ANW * 2 * (D / dkv_dsplit<D>() / 32) * 16 * 64 * 4 : 0;
  static_assert((size_t)NGK * NSK * (kStageKv + ATILE * 16) + kOwn <= 160 * 1024 && kPark <= 160 * 1024, "LDS budget");
  size_t lds_kv = (size_t)NGK * NSK * (kStageKv + (DROP ? ATILE * 16 : 0)) + kOwn;
  if (lds_kv < kPark) lds_kv = kPark;
  if (lds_kv > 64 * 1024) {
    e = hipFuncSetAttribute((const void*)attn_bwd_dkv_bf16_kernel<D, DROP>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)lds_kv);
    if (e != hipSuccess) return e;
  }
  const dim3 grid_kv = attn_grid(nblk * dkv_dsplit<D>(), a.hl, a.b);
  hipLaunchKernelGGL((attn_bwd_dkv_bf16_kernel<D, DROP>), grid_kv, dim3(NGK * ANT), lds_kv, st, a);
  return hipGetLastError();
}

template <int D>
static hipError_t launch_bwd_d(const AttnArgs& a, hipStream_t st) {
  return a.drop.enabled ? launch_bwd_dd<D, true>(a, st) : launch_bwd_dd<D, false>(a, st);
}

hipError_t launch_attn_fwd_bf16(const AttnArgs& a, hipStream_t st) {
  switch (a.d) {
    case 64: return launch_fwd_d<64>(a, st);
    case 96: return launch_fwd_d<96>(a, st);
    case 128: return launch_fwd_d<128>(a, st);
    case 192: return launch_fwd_d<192>(a, st);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_attn_bwd_bf16(const AttnArgs& a, hipStream_t st) {
  switch (a.d) {
    case 64: return launch_bwd_d<64>(a, st);
    case 96: return launch_bwd_d<96>(a, st);
    case 128: return launch_bwd_d<128>(a, st);
    case 192: return launch_bwd_d<192>(a, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace mlm
