// Dispatcher of the bf16 MFMA GEMM: operand layout -> translation unit, problem shape -> tile configuration.
#include <stdlib.h>
#include "gemm_bf16.h"

namespace mlm {

// Tile choice.  256 CUs; a 256x256 or 256x128 workgroup fills a CU's LDS (1 per CU), 128x128 fits twice.
// Cost model: (number of scheduling rounds) x (tile area) / (relative efficiency of the tile shape); the larger
// tiles reuse LDS data more per MFMA but quantise worse on small N.  MLM_GEMM_TILE=0/1/2 forces a configuration
// (used by the tuning sweeps).
int gemm_cu_count();

int pick_tile(int M, int N, int K) {
  (void)K;
  static int forced = -2;
  if (forced == -2) {
    const char* e = getenv("MLM_GEMM_TILE");
    forced = e ? atoi(e) : -1;
  }
  if (forced >= 0 && forced < TILE_COUNT) return forced;
  const int bm[TILE_COUNT] = {256, 256, 128}, bn[TILE_COUNT] = {256, 128, 128};
  const int per_cu[TILE_COUNT] = {1, 1, 2};
  const double eff[TILE_COUNT] = {1.0, 0.9, 0.75};
  int best = 0;
  double best_cost = 1e300;
  for (int t = 0; t < TILE_COUNT; ++t) {
    const long tiles = (long)((M + bm[t] - 1) / bm[t]) * ((N + bn[t] - 1) / bn[t]);
    const long slots = (long)gemm_cu_count() * per_cu[t];
    const long rounds = (tiles + slots - 1) / slots;
    const double cost = (double)rounds * bm[t] * bn[t] * per_cu[t] / eff[t];
    if (cost < best_cost) { best_cost = cost; best = t; }
  }
  return best;
}

// MLM_GEMM_V2=0 switches the direct-to-LDS kernel off (A/B comparisons).
bool gemm_use_v2(const GemmArgs& a) {
  static int enabled = -1;
  if (enabled < 0) {
    const char* e = getenv("MLM_GEMM_V2");
    enabled = (e && atoi(e) == 0) ? 0 : 1;
  }
  return enabled && a.K % 32 == 0 && a.K >= 64;
}

// Waves per workgroup of the 256 x 256 tile: 8 (2 x 4 waves of 128 x 64, two per SIMD) for every operand layout.
// (With the 32 x 32 x 16 MFMA the weight-gradient layout -- both operands read through the transposing loads -- was
// ~3 % faster with 4 waves of 128 x 128; with the 16 x 16 x 32 MFMA, which only the 8-wave variant uses, 8 waves win by
// 10 % on the 3072 x 6400 x 8192 gradient of the output embedding.)  MLM_GEMM_WAVES=4|8 forces one variant.
int gemm_v2_waves(bool a_kc, bool b_kc) {
  (void)a_kc; (void)b_kc;
  static int forced = -1;
  if (forced < 0) {
    const char* e = getenv("MLM_GEMM_WAVES");
    forced = e ? (atoi(e) == 4 ? 4 : 8) : 0;
  }
  return forced ? forced : 8;
}

int gemm_v2_forced_bn() {
  static int forced = -1;
  if (forced < 0) {
    const char* e = getenv("MLM_GEMM_BN");
    const int v = e ? atoi(e) : 0;
    forced = (v == 192 || v == 256) ? v : 0;
  }
  return forced;
}

// Compute units of the current device, capped at the tail-split workspace's bound; one query per device.
int gemm_cu_count() {
  constexpr int kMaxDevices = 64, kCap = 256;
  static int cached[kMaxDevices] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return kCap;
  int n = __atomic_load_n(&cached[dev], __ATOMIC_RELAXED);
  if (n == 0) {
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = kCap;
    if (n > kCap) n = kCap;
    __atomic_store_n(&cached[dev], n, __ATOMIC_RELAXED);
  }
  return n;
}

int gemm_bf16_ce_col_tiles(int M, int N, int K) {
  GemmArgs probe;
  probe.K = K;
  if (gemm_use_v2(probe)) return (N + 255) / 256;
  const int bn = kTileBN[pick_tile(M, N, K)];
  return (N + bn - 1) / bn;
}

hipError_t launch_gemm_bf16(const GemmArgs& a, hipStream_t st) {
  if (a.a_kc && !a.b_kc) return launch_gemm_bf16_fwd(a, st);
  if (a.a_kc && a.b_kc) return launch_gemm_bf16_dgrad(a, st);
  if (!a.a_kc && !a.b_kc) return launch_gemm_bf16_wgrad(a, st);
  return hipErrorInvalidValue;
}

}  // namespace mlm
