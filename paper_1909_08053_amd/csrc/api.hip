// extern "C" entry points of libmlm_shard: host-side validation, workspace carving and the
// per-block kernel sequences.  Every device step runs in this library's own kernels.
#include <string.h>
#include "common.h"
#include "rng.h"

using namespace mlm;

namespace {

struct Local {
  int T, d, hl, Hl, Fl, Vl;
  size_t esz;
};

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

int check_dims(const mlm_dims* dm, Local* L) {
  if (!dm) return MLM_E_NULL;
  if (dm->dtype != MLM_F32 && dm->dtype != MLM_BF16) return MLM_E_DTYPE;
  if (dm->b <= 0 || dm->s <= 0 || dm->H <= 0 || dm->h <= 0 || dm->F <= 0 || dm->V <= 0 || dm->p <= 0)
    return MLM_E_SHAPE;
  if (dm->r < 0 || dm->r >= dm->p) return MLM_E_SHAPE;
  if (dm->H % dm->h || dm->h % dm->p || dm->F % dm->p || dm->V % dm->p) return MLM_E_SHAPE;
  // launch-grid limits: token and column counts index 1-D grids (products below 2^31), row tiles and the batch index
  // 2-D / 3-D grids (below 65536)
  if ((int64_t)dm->b * dm->s > (int64_t)1 << 21 || dm->b > 65535) return MLM_E_SHAPE;
  if (dm->H > (1 << 20) || dm->F / dm->p > (1 << 20) || dm->V / dm->p > (1 << 20)) return MLM_E_SHAPE;
  L->T = dm->b * dm->s;
  L->d = dm->H / dm->h;
  L->hl = dm->h / dm->p;
  L->Hl = L->hl * L->d;
  L->Fl = dm->F / dm->p;
  L->Vl = dm->V / dm->p;
  L->esz = dm->dtype == MLM_BF16 ? 2 : 4;
  if (dm->H % 8 || L->Hl % 8 || L->Fl % 8 || L->Vl % 8 || L->d % 8) return MLM_E_ALIGN;
  return MLM_OK;
}

int ln_supported(const mlm_dims* dm) {
  const int vn = dm->dtype == MLM_BF16 ? 8 : 4;
  return (dm->H / vn + 63) / 64 <= 8 ? MLM_OK : MLM_E_UNSUPPORTED;
}

int attn_supported(const mlm_dims* dm, const Local& L) {
  const bool ok = dm->dtype == MLM_BF16 ? attn_bf16_supported(L.d) : attn_f32_supported(L.d);
  return ok ? MLM_OK : MLM_E_UNSUPPORTED;
}

// fp32 scratch for the k-split of partially filled GEMM rounds (bf16 path only)
constexpr size_t kSplitKBytes = (size_t)256 * 256 * 256 * sizeof(float);

size_t ws_bytes_for(const mlm_dims* dm, const Local& L, int which) {
  const size_t T = (size_t)L.T;
  const size_t cs_rows = (T + kColsumRowsPerBlock - 1) / kColsumRowsPerBlock;
  const size_t sk = dm->dtype == MLM_BF16 ? kSplitKBytes : 0;
  switch (which) {
    case MLM_WS_LAYERNORM_BWD:
      return align256(((T + kLnBwdRowsPerBlock - 1) / kLnBwdRowsPerBlock) * 3 * (size_t)dm->H * 4);
    case MLM_WS_ATTN_FWD: return sk;
    case MLM_WS_ATTN_BWD:
      return align256(T * L.Hl * L.esz) + align256(T * 3 * L.Hl * L.esz) +
             align256((size_t)dm->b * L.hl * dm->s * 8) + align256(cs_rows * 3 * L.Hl * 4) + sk;
    case MLM_WS_MLP_FWD: return sk;
    case MLM_WS_MLP_BWD: return align256(T * L.Fl * L.esz) + align256(cs_rows * L.Fl * 4) + sk;
    case MLM_WS_COLSUM: return align256(cs_rows * (size_t)dm->H * 4);
    case MLM_WS_VOCAB_CE_FWD:
      if (dm->dtype == MLM_BF16) {
        const size_t ntile = ((size_t)L.Vl + 127) / 128;   // upper bound over the tile configurations
        return 2 * align256(ntile * T * 4) + align256(T * 4) + sk;
      }
      return align256(T * L.Vl * 4);
    case MLM_WS_VOCAB_CE_BWD: return align256(T * L.Vl * L.esz) + sk;
    default: return 0;
  }
}

inline int hip_status(hipError_t e) { return e == hipSuccess ? MLM_OK : MLM_E_HIP; }

GemmArgs gemm_args(int M, int N, int K, const void* A, int lda, int a_kc, const void* B, int ldb, int b_kc, void* C,
                   int ldc) {
  GemmArgs g;
  memset(&g, 0, sizeof(g));
  g.M = M; g.N = N; g.K = K;
  g.A = A; g.lda = lda; g.a_kc = a_kc;
  g.B = B; g.ldb = ldb; g.b_kc = b_kc;
  g.C = C; g.ldc = ldc;
  g.epi = EPI_STORE;
  return g;
}

hipError_t run_gemm(int dtype, GemmArgs g, hipStream_t st, float* splitk = nullptr) {
  g.splitk_ws = splitk;
  return dtype == MLM_BF16 ? launch_gemm_bf16(g, st) : launch_gemm_f32(g, st);
}

// forward layout: C[M,N] = X[M,K] W[K,N]
GemmArgs gemm_fwd(int M, int N, int K, const void* X, const void* W, void* C) {
  return gemm_args(M, N, K, X, K, 1, W, N, 0, C, N);
}
// input gradient: dX[M,N] = dY[M,K] W[N,K]^T  (W stored [in=N, out=K])
GemmArgs gemm_dgrad(int M, int N, int K, const void* dY, const void* W, void* dX) {
  return gemm_args(M, N, K, dY, K, 1, W, K, 1, dX, N);
}
// weight gradient: dW[M,N] = X[K,M]^T dY[K,N]
GemmArgs gemm_wgrad(int M, int N, int K, const void* X, const void* dY, void* dW) {
  return gemm_args(M, N, K, X, M, 0, dY, N, 0, dW, N);
}

#define MLM_TRY_HIP(expr)                    \
  do {                                       \
    hipError_t e_ = (expr);                  \
    if (e_ != hipSuccess) return MLM_E_HIP;  \
  } while (0)

}  // namespace

extern "C" {

MLM_API const char* mlm_status_string(int code) {
  switch (code) {
    case MLM_OK: return "MLM_OK";
    case MLM_E_NULL: return "MLM_E_NULL: required pointer is NULL";
    case MLM_E_SHAPE: return "MLM_E_SHAPE: bad size or indivisible shard";
    case MLM_E_DTYPE: return "MLM_E_DTYPE: unknown dtype";
    case MLM_E_WORKSPACE: return "MLM_E_WORKSPACE: workspace too small, or problem larger than the static scratch of a no-allocation call";
    case MLM_E_ALIGN: return "MLM_E_ALIGN: size or pointer alignment";
    case MLM_E_HIP: return "MLM_E_HIP: HIP call or launch failed";
    case MLM_E_UNSUPPORTED: return "MLM_E_UNSUPPORTED: configuration not compiled in";
    default: return "MLM_E_?: unknown status";
  }
}

MLM_API int mlm_shard_range(int64_t n, int32_t p, int32_t r, int64_t* begin, int64_t* end) {
  if (!begin || !end) return MLM_E_NULL;
  if (p <= 0 || r < 0 || r >= p || n < 0 || n % p != 0) return MLM_E_SHAPE;
  const int64_t q = n / p;
  *begin = (int64_t)r * q;
  *end = (int64_t)(r + 1) * q;
  return MLM_OK;
}

MLM_API int mlm_workspace_bytes(const mlm_dims* dims, int32_t which, size_t* bytes) {
  if (!bytes) return MLM_E_NULL;
  Local L;
  int rc = check_dims(dims, &L);
  if (rc) return rc;
  if (which < 0 || which >= MLM_WS_COUNT) return MLM_E_SHAPE;
  *bytes = ws_bytes_for(dims, L, which);
  return MLM_OK;
}

MLM_API int mlm_layernorm_fwd(const mlm_dims* dims, const void* x, const void* gamma, const void* beta, void* y, float* mean,
                      float* rstd, void* stream) {
  Local L;
  int rc = check_dims(dims, &L);
  if (rc) return rc;
  if (!x || !gamma || !beta || !y || !mean || !rstd) return MLM_E_NULL;
  if (!aligned16(x) || !aligned16(gamma) || !aligned16(beta) || !aligned16(y)) return MLM_E_ALIGN;
  if ((rc = ln_supported(dims))) return rc;
  return hip_status(launch_layernorm_fwd(dims->dtype, L.T, dims->H, dims->ln_eps, x, gamma, beta, y, mean, rstd,
                                         (hipStream_t)stream));
}

MLM_API int mlm_layernorm_bwd(const mlm_dims* dims, const void* dy, const void* x, const void* gamma, const float* mean,
                      const float* rstd, const void* residual_grad, void* dx, void* dgamma, void* dbeta, void* ws,
                      size_t ws_bytes, void* stream) {
  Local L;
  int rc = check_dims(dims, &L);
  if (rc) return rc;
  if (!dy || !x || !gamma || !mean || !rstd || !dx || !dgamma || !dbeta || !ws) return MLM_E_NULL;
  if (!aligned16(dy) || !aligned16(x) || !aligned16(gamma) || !aligned16(dx) || !aligned16(ws) ||
      (residual_grad && !aligned16(residual_grad)))
    return MLM_E_ALIGN;
  if ((rc = ln_supported(dims))) return rc;
  if (ws_bytes < ws_bytes_for(dims, L, MLM_WS_LAYERNORM_BWD)) return MLM_E_WORKSPACE;
  return hip_status(launch_layernorm_bwd(dims->dtype, L.T, dims->H, dy, x, gamma, mean, rstd, residual_grad, dx,
                                         dgamma, dbeta, (float*)ws, (hipStream_t)stream));
}

MLM_API int mlm_combine(const mlm_dims* dims, const void* const* partials, int32_t n_partials, const void* bias,
                const void* residual, void* out, void* stream) {
  Local L;
  int rc = check_dims(dims, &L);
  if (rc) return rc;
  if (!partials || !out) return MLM_E_NULL;
  if (n_partials < 1 || n_partials > kMaxPartials) return MLM_E_SHAPE;
  for (int i = 0; i < n_partials; ++i) {
    if (!partials[i]) return MLM_E_NULL;
    if (!aligned16(partials[i])) return MLM_E_ALIGN;
  }
  if (!aligned16(out) || (bias && !aligned16(bias)) || (residual && !aligned16(residual))) return MLM_E_ALIGN;
  return hip_status(launch_combine(dims->dtype, L.T, dims->H, partials, n_partials, bias, 1, residual, out, nullptr,
                                   (hipStream_t)stream));
}

static int check_partials(const void* const* partials, int32_t n) {
  if (!partials) return MLM_E_NULL;
  if (n < 1 || n > kMaxPartials) return MLM_E_SHAPE;
  for (int i = 0; i < n; ++i) {
    if (!partials[i]) return MLM_E_NULL;
    if (!aligned16(partials[i])) return MLM_E_ALIGN;
  }
  return MLM_OK;
}

static int check_drop(const mlm_dropout* drop) {
  if (drop && !(drop->p >= 0.0f && drop->p < 1.0f)) return MLM_E_SHAPE;
  return MLM_OK;
}

static int combine_layernorm_fwd_impl(const mlm_dims* dims, const void* const* partials, int32_t n_partials,
                                      const void* bias, const mlm_dropout* drop, const void* residual, void* x_out,
                                      const void* gamma, const void* beta, void* y, float* mean, float* rstd,
                                      void* stream) {
  Local L;
  int rc = check_dims(dims, &L);
  if (rc) return rc;
  if ((rc = check_partials(partials, n_partials))) return rc;
  if ((rc = check_drop(drop))) return rc;
  if (!x_out || !gamma || !beta || !y || !mean || !rstd) return MLM_E_NULL;
  if (!aligned16(x_out) || !aligned16(gamma) || !aligned16(beta) || !aligned16(y) || (bias && !aligned16(bias)) ||
      (residual && !aligned16(residual)))
    return MLM_E_ALIGN;
  if ((rc = ln_supported(dims))) return rc;
  return hip_status(launch_combine_layernorm_fwd(dims->dtype, L.T, dims->H, dims->ln_eps, partials, n_partials, bias,
                                                 residual, x_out, gamma, beta, y, mean, rstd, drop,
                                                 (hipStream_t)stream));
}

MLM_API int mlm_combine_layernorm_fwd(const mlm_dims* dims, const void* const* partials, int32_t n_partials,
                                      const void* bias, const void* residual, void* x_out, const void* gamma,
                                      const void* beta, void* y, float* mean, float* rstd, void* stream) {
  return combine_layernorm_fwd_impl(dims, partials, n_partials, bias, nullptr, residual, x_out, gamma, beta, y, mean,
                                    rstd, stream);
}

MLM_API int mlm_combine_layernorm_fwd_dropout(const mlm_dims* dims, const void* const* partials, int32_t n_partials,
                                              const void* bias, const mlm_dropout* drop, const void* residual,
                                              void* x_out, const void* gamma, const void* beta, void* y, float* mean,
                                              float* rstd, void* stream) {
  return combine_layernorm_fwd_impl(dims, partials, n_partials, bias, drop, residual, x_out, gamma, beta, y, mean, rstd,
                                    stream);
}

MLM_API int mlm_combine_dropout(const mlm_dims* dims, const void* const* partials, int32_t n_partials, const void* bias,
                                int32_t bias_rows, const mlm_dropout* drop, const void* residual, void* out,
                                void* stream) {
  Local L;
  int rc = check_dims(dims, &L);
  if (rc) return rc;
  if ((rc = check_partials(partials, n_partials))) return rc;
  if ((rc = check_drop(drop))) return rc;
  if (!out) return MLM_E_NULL;
  if (bias && (bias_rows < 1 || bias_rows > L.T)) return MLM_E_SHAPE;
  if (!aligned16(out) || (bias && !aligned16(bias)) || (residual && !aligned16(residual))) return MLM_E_ALIGN;
  return hip_status(launch_combine(dims->dtype, L.T, dims->H, partials, n_partials, bias, bias ? bias_rows : 1,
                                   residual, out, drop, (hipStream_t)stream));
}

static int combine_layernorm_bwd_impl(const mlm_dims* dims, const void* const* partials, int32_t n_partials,
                                      const void* x, const void* gamma, const float* mean, const float* rstd,
                                      const void* residual_grad, const mlm_dropout* drop, void* dy_out, void* dx,
                                      void* dz_out, void* dgamma, void* dbeta, void* dx_colsum, void* ws,
                                      size_t ws_bytes, void* stream) {
  Local L;
  int rc = check_dims(dims, &L);
  if (rc) return rc;
  if ((rc = check_partials(partials, n_partials))) return rc;
  if ((rc = check_drop(drop))) return rc;
  if ((drop && drop->p > 0.0f && !dz_out) || (dz_out && dz_out == dx)) return MLM_E_NULL;
  if (dz_out && !aligned16(dz_out)) return MLM_E_ALIGN;
  if (!x || !gamma || !mean || !rstd || !dx || !dgamma || !dbeta || !ws) return MLM_E_NULL;
  if (!aligned16(x) || !aligned16(gamma) || !aligned16(dx) || !aligned16(ws) ||
      (residual_grad && !aligned16(residual_grad)) || (dy_out && !aligned16(dy_out)))
    return MLM_E_ALIGN;
  if ((rc = ln_supported(dims))) return rc;
  if (ws_bytes < ws_bytes_for(dims, L, MLM_WS_LAYERNORM_BWD)) return MLM_E_WORKSPACE;
  return hip_status(launch_combine_layernorm_bwd(dims->dtype, L.T, dims->H, partials, n_partials, x, gamma, mean, rstd,
                                                 residual_grad, dy_out, dx, dgamma, dbeta, dx_colsum, (float*)ws,
                                                 drop, dz_out, (hipStream_t)stream));
}

MLM_API int mlm_combine_layernorm_bwd(const mlm_dims* dims, const void* const* partials, int32_t n_partials,
                                      const void* x, const void* gamma, const float* mean, const float* rstd,
                                      const void* residual_grad, void* dy_out, void* dx, void* dgamma, void* dbeta,
                                      void* dx_colsum, void* ws, size_t ws_bytes, void* stream) {
  return combine_layernorm_bwd_impl(dims, partials, n_partials, x, gamma, mean, rstd, residual_grad, nullptr, dy_out, dx,
                                    nullptr, dgamma, dbeta, dx_colsum, ws, ws_bytes, stream);
}

MLM_API int mlm_combine_layernorm_bwd_dropout(const mlm_dims* dims, const void* const* partials, int32_t n_partials,
                                              const void* x, const void* gamma, const float* mean, const float* rstd,
                                              const void* residual_grad, const mlm_dropout* drop, void* dy_out,
                                              void* dx, void* dz_out, void* dgamma, void* dbeta, void* dx_colsum,
                                              void* ws, size_t ws_bytes, void* stream) {
  return combine_layernorm_bwd_impl(dims, partials, n_partials, x, gamma, mean, rstd, residual_grad, drop, dy_out, dx,
                                    dz_out, dgamma, dbeta, dx_colsum, ws, ws_bytes, stream);
}

MLM_API int mlm_colsum(const mlm_dims* dims, const void* dy, void* dbias, void* ws, size_t ws_bytes, void* stream) {
  Local L;
  int rc = check_dims(dims, &L);
  if (rc) return rc;
  if (!dy || !dbias || !ws) return MLM_E_NULL;
  if (!aligned16(dy) || !aligned16(ws)) return MLM_E_ALIGN;
  if (ws_bytes < ws_bytes_for(dims, L, MLM_WS_COLSUM)) return MLM_E_WORKSPACE;
  return hip_status(launch_colsum(dims->dtype, L.T, dims->H, dy, dbias, (float*)ws, (hipStream_t)stream));
}

MLM_API int mlm_colsum_noalloc(const mlm_dims* dims, const void* dy, void* dbias, void* stream) {
  Local L;
  int rc = check_dims(dims, &L);
  if (rc) return rc;
  if (!dy || !dbias) return MLM_E_NULL;
  if (!aligned16(dy)) return MLM_E_ALIGN;
  const size_t chunks = ((size_t)L.T + kColsumRowsPerBlock - 1) / kColsumRowsPerBlock;
  if (chunks * (size_t)dims->H > kStaticScratchFloats) return MLM_E_WORKSPACE;   // beyond the static scratch
  return hip_status(launch_colsum_static(dims->dtype, L.T, dims->H, dy, dbias, (hipStream_t)stream));
}

// upper bound of the partial storage of one layer backward + the final layer norm: four layer-norm backwards, the
// two bias column sums inside the attention and MLP calls and two stand-alone [T,H] column sums
static size_t deferred_sums_bytes_for(const mlm_dims* dm, const Local& L) {
  const size_t T = (size_t)L.T;
  const size_t ln = align256(((T + kLnBwdRowsPerBlock - 1) / kLnBwdRowsPerBlock) * 3 * (size_t)dm->H * 4);
  const size_t chunks = (T + kColsumRowsPerBlock - 1) / kColsumRowsPerBlock;
  return 4 * ln + align256(chunks * 3 * L.Hl * 4) + align256(chunks * L.Fl * 4) + 2 * align256(chunks * dm->H * 4);
}

MLM_API int mlm_deferred_sums_bytes(const mlm_dims* dims, size_t* bytes) {
  Local L;
  int rc = check_dims(dims, &L);
  if (rc) return rc;
  if (!bytes) return MLM_E_NULL;
  *bytes = deferred_sums_bytes_for(dims, L);
  return MLM_OK;
}

MLM_API int mlm_deferred_sums_begin(void* buf, size_t buf_bytes) {
  if (!buf) return MLM_E_NULL;
  if (((uintptr_t)buf & 255) != 0) return MLM_E_ALIGN;
  if (deferred_sums_open()) return MLM_E_UNSUPPORTED;      // one open list per host thread
  return hip_status(deferred_sums_begin(buf, buf_bytes));
}

MLM_API int mlm_deferred_sums_flush(void* stream) {
  if (!deferred_sums_open()) return MLM_E_UNSUPPORTED;
  return hip_status(deferred_sums_flush((hipStream_t)stream));
}

static int keep_pitch_words(int s) { return 4 * ((s + 127) / 128); }

// dropout of the attention probabilities requested and active (p > 0)?  Validates the extra arguments.
static int check_attn_drop(const mlm_dims* dims, const mlm_dropout* drop, const void* keep_bits, bool* active) {
  *active = false;
  int rc = check_drop(drop);
  if (rc) return rc;
  if (!drop || drop->p <= 0.0f) return MLM_OK;
  if (!keep_bits) return MLM_E_NULL;
  if (dims->s % 4 != 0 || !aligned16(keep_bits)) return MLM_E_ALIGN;
  *active = true;
  return MLM_OK;
}

static int attn_shard_fwd_impl(const mlm_dims* dims, const void* u, const void* Wqkv_r, const void* bqkv_r,
                               const void* Wo_r, const int32_t* key_len, const mlm_dropout* drop, void* qkv_r,
                               void* ctx_r, float* lse_r, uint32_t* keep_bits_r, void* partial_r, void* ws,
                               size_t ws_bytes, void* stream) {
  Local L;
  int rc = check_dims(dims, &L);
  if (rc) return rc;
  bool dropping;
  if ((rc = check_attn_drop(dims, drop, keep_bits_r, &dropping))) return rc;
  if (!u || !Wqkv_r || !Wo_r || !qkv_r || !ctx_r || !lse_r || !partial_r) return MLM_E_NULL;
  if (!aligned16(u) || !aligned16(Wqkv_r) || !aligned16(Wo_r) || !aligned16(qkv_r) || !aligned16(ctx_r) ||
      !aligned16(partial_r) || (bqkv_r && !aligned16(bqkv_r)))
    return MLM_E_ALIGN;
  if ((rc = attn_supported(dims, L))) return rc;
  if (ws_bytes < ws_bytes_for(dims, L, MLM_WS_ATTN_FWD) || (ws_bytes && !ws)) return MLM_E_WORKSPACE;
  if (ws && !aligned16(ws)) return MLM_E_ALIGN;
  hipStream_t st = (hipStream_t)stream;
  const int dt = dims->dtype;
  float* sk = dt == MLM_BF16 ? (float*)ws : nullptr;
  GemmArgs g = gemm_fwd(L.T, 3 * L.Hl, dims->H, u, Wqkv_r, qkv_r);
  g.bias = bqkv_r;
  MLM_TRY_HIP(run_gemm(dt, g, st, sk));
  AttnArgs a;
  memset(&a, 0, sizeof(a));
  a.b = dims->b; a.s = dims->s; a.hl = L.hl; a.d = L.d; a.causal = dims->causal; a.key_len = key_len;
  a.qkv = qkv_r; a.ctx = ctx_r; a.lse = lse_r;
  a.drop = make_drop_args(dropping ? drop : nullptr);
  a.keep_bits = keep_bits_r; a.keep_pitch = keep_pitch_words(dims->s);
  MLM_TRY_HIP(dt == MLM_BF16 ? launch_attn_fwd_bf16(a, st) : launch_attn_fwd_f32(a, st));
  MLM_TRY_HIP(run_gemm(dt, gemm_fwd(L.T, dims->H, L.Hl, ctx_r, Wo_r, partial_r), st, sk));
  return MLM_OK;
}

MLM_API int mlm_attn_shard_fwd(const mlm_dims* dims, const void* u, const void* Wqkv_r, const void* bqkv_r, const void* Wo_r,
                       const int32_t* key_len, void* qkv_r, void* ctx_r, float* lse_r, void* partial_r, void* ws,
                       size_t ws_bytes, void* stream) {
  return attn_shard_fwd_impl(dims, u, Wqkv_r, bqkv_r, Wo_r, key_len, nullptr, qkv_r, ctx_r, lse_r, nullptr, partial_r, ws,
                             ws_bytes, stream);
}

MLM_API int mlm_attn_shard_fwd_dropout(const mlm_dims* dims, const void* u, const void* Wqkv_r, const void* bqkv_r,
                                       const void* Wo_r, const int32_t* key_len, const mlm_dropout* drop, void* qkv_r,
                                       void* ctx_r, float* lse_r, uint32_t* keep_bits_r, void* partial_r, void* ws,
                                       size_t ws_bytes, void* stream) {
  return attn_shard_fwd_impl(dims, u, Wqkv_r, bqkv_r, Wo_r, key_len, drop, qkv_r, ctx_r, lse_r, keep_bits_r, partial_r,
                             ws, ws_bytes, stream);
}

MLM_API int mlm_attn_keep_words(const mlm_dims* dims, size_t* words) {
  if (!words) return MLM_E_NULL;
  Local L;
  int rc = check_dims(dims, &L);
  if (rc) return rc;
  *words = (size_t)dims->b * L.hl * dims->s * keep_pitch_words(dims->s);
  return MLM_OK;
}

MLM_API int mlm_rng_stream_seed(uint64_t base_seed, int32_t stream, int32_t r, uint64_t* seed) {
  if (!seed) return MLM_E_NULL;
  if (r < 0) return MLM_E_SHAPE;
  if (stream == MLM_STREAM_REPLICATED) { *seed = base_seed; return MLM_OK; }
  if (stream == MLM_STREAM_MODEL_PARALLEL) { *seed = base_seed + 1ull + (uint64_t)r; return MLM_OK; }
  return MLM_E_SHAPE;
}

static int attn_shard_bwd_impl(const mlm_dims* dims, const void* dx1, const void* u, const void* Wqkv_r,
                               const void* Wo_r, const int32_t* key_len, const mlm_dropout* drop, const void* qkv_r,
                               const void* ctx_r, const float* lse_r, const uint32_t* keep_bits_r, void* dWqkv_r,
                               void* dbqkv_r, void* dWo_r, void* du_partial_r, void* ws, size_t ws_bytes,
                               void* stream, void* dqkv_out = nullptr) {
  // dqkv_out != NULL: input-gradient-only form -- the gradient of the QKV activations is left in dqkv_out for a later
  // mlm_layer_shard_wgrads call and the two weight gradients are not computed here (u, dWqkv_r, dWo_r unused)
  const bool defer = dqkv_out != nullptr;
  Local L;
  int rc = check_dims(dims, &L);
  if (rc) return rc;
  bool dropping;
  if ((rc = check_attn_drop(dims, drop, keep_bits_r, &dropping))) return rc;
  if (!dx1 || !Wqkv_r || !Wo_r || !qkv_r || !ctx_r || !lse_r || !dbqkv_r || !du_partial_r || !ws) return MLM_E_NULL;
  if (!defer && (!u || !dWqkv_r || !dWo_r)) return MLM_E_NULL;
  if (!aligned16(dx1) || !aligned16(Wqkv_r) || !aligned16(Wo_r) || !aligned16(qkv_r) || !aligned16(ctx_r) ||
      !aligned16(du_partial_r) || !aligned16(ws) || (defer && !aligned16(dqkv_out)) ||
      (!defer && (!aligned16(u) || !aligned16(dWqkv_r) || !aligned16(dWo_r))))
    return MLM_E_ALIGN;
  if ((rc = attn_supported(dims, L))) return rc;
  if (ws_bytes < ws_bytes_for(dims, L, MLM_WS_ATTN_BWD)) return MLM_E_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  const int dt = dims->dtype;
  const size_t T = (size_t)L.T;
  char* w = (char*)ws;
  void* dctx = w;                 w += align256(T * L.Hl * L.esz);
  void* dqkv = defer ? dqkv_out : (void*)w;   w += align256(T * 3 * L.Hl * L.esz);
  float* delta = (float*)w;       w += align256((size_t)dims->b * L.hl * dims->s * 8);   // delta, and lse in log2 units
  float* csws = (float*)w;        w += align256(((T + kColsumRowsPerBlock - 1) / kColsumRowsPerBlock) * 3 * L.Hl * 4);
  float* sk = dt == MLM_BF16 ? (float*)w : nullptr;
  // output projection: dWo_r = ctx^T dx1, dctx = dx1 Wo_r^T
  if (!defer) MLM_TRY_HIP(run_gemm(dt, gemm_wgrad(L.Hl, dims->H, L.T, ctx_r, dx1, dWo_r), st, sk));
  MLM_TRY_HIP(run_gemm(dt, gemm_dgrad(L.T, L.Hl, dims->H, dx1, Wo_r, dctx), st, sk));
  // attention core
  // bf16: the dQ kernel computes delta itself (and stores it for the dK/dV kernel)
  if (dt != MLM_BF16) MLM_TRY_HIP(launch_attn_delta(dt, L.T, L.hl, L.d, dims->b, dims->s, ctx_r, dctx, delta, st));
  AttnArgs a;
  memset(&a, 0, sizeof(a));
  a.b = dims->b; a.s = dims->s; a.hl = L.hl; a.d = L.d; a.causal = dims->causal; a.key_len = key_len;
  a.qkv = qkv_r; a.ctx = const_cast<void*>(ctx_r); a.lse = const_cast<float*>(lse_r);
  a.dctx = dctx; a.dqkv = dqkv; a.delta = delta;
  a.drop = make_drop_args(dropping ? drop : nullptr);
  a.keep_bits = const_cast<uint32_t*>(keep_bits_r); a.keep_pitch = keep_pitch_words(dims->s);
  MLM_TRY_HIP(dt == MLM_BF16 ? launch_attn_bwd_bf16(a, st) : launch_attn_bwd_f32(a, st));
  // QKV projection: dWqkv_r = u^T dqkv, dbqkv_r = column sums, du_partial_r = dqkv Wqkv_r^T
  if (!defer) MLM_TRY_HIP(run_gemm(dt, gemm_wgrad(dims->H, 3 * L.Hl, L.T, u, dqkv, dWqkv_r), st, sk));
  MLM_TRY_HIP(launch_colsum(dt, L.T, 3 * L.Hl, dqkv, dbqkv_r, csws, st));
  MLM_TRY_HIP(run_gemm(dt, gemm_dgrad(L.T, dims->H, 3 * L.Hl, dqkv, Wqkv_r, du_partial_r), st, sk));
  return MLM_OK;
}

MLM_API int mlm_attn_shard_bwd(const mlm_dims* dims, const void* dx1, const void* u, const void* Wqkv_r, const void* Wo_r,
                       const int32_t* key_len, const void* qkv_r, const void* ctx_r, const float* lse_r, void* dWqkv_r,
                       void* dbqkv_r, void* dWo_r, void* du_partial_r, void* ws, size_t ws_bytes, void* stream) {
  return attn_shard_bwd_impl(dims, dx1, u, Wqkv_r, Wo_r, key_len, nullptr, qkv_r, ctx_r, lse_r, nullptr, dWqkv_r, dbqkv_r,
                             dWo_r, du_partial_r, ws, ws_bytes, stream);
}

MLM_API int mlm_attn_shard_bwd_input(const mlm_dims* dims, const void* dx1, const void* Wqkv_r, const void* Wo_r,
                                     const int32_t* key_len, const mlm_dropout* drop, const void* qkv_r,
                                     const void* ctx_r, const float* lse_r, const uint32_t* keep_bits_r, void* dqkv_r,
                                     void* dbqkv_r, void* du_partial_r, void* ws, size_t ws_bytes, void* stream) {
  if (!dqkv_r) return MLM_E_NULL;
  return attn_shard_bwd_impl(dims, dx1, nullptr, Wqkv_r, Wo_r, key_len, drop, qkv_r, ctx_r, lse_r, keep_bits_r, nullptr,
                             dbqkv_r, nullptr, du_partial_r, ws, ws_bytes, stream, dqkv_r);
}

MLM_API int mlm_attn_shard_bwd_dropout(const mlm_dims* dims, const void* dx1, const void* u, const void* Wqkv_r,
                                       const void* Wo_r, const int32_t* key_len, const mlm_dropout* drop,
                                       const void* qkv_r, const void* ctx_r, const float* lse_r,
                                       const uint32_t* keep_bits_r, void* dWqkv_r, void* dbqkv_r, void* dWo_r,
                                       void* du_partial_r, void* ws, size_t ws_bytes, void* stream) {
  return attn_shard_bwd_impl(dims, dx1, u, Wqkv_r, Wo_r, key_len, drop, qkv_r, ctx_r, lse_r, keep_bits_r, dWqkv_r,
                             dbqkv_r, dWo_r, du_partial_r, ws, ws_bytes, stream);
}

MLM_API int mlm_mlp_shard_fwd(const mlm_dims* dims, const void* u2, const void* A_r, const void* a_r, const void* B_r,
                      void* g_r, void* y_r, void* partial_r, void* ws, size_t ws_bytes, void* stream) {
  Local L;
  int rc = check_dims(dims, &L);
  if (rc) return rc;
  if (!u2 || !A_r || !B_r || !g_r || !y_r || !partial_r) return MLM_E_NULL;
  if (!aligned16(u2) || !aligned16(A_r) || !aligned16(B_r) || !aligned16(g_r) || !aligned16(y_r) ||
      !aligned16(partial_r) || (a_r && !aligned16(a_r)))
    return MLM_E_ALIGN;
  if (ws_bytes < ws_bytes_for(dims, L, MLM_WS_MLP_FWD) || (ws_bytes && !ws)) return MLM_E_WORKSPACE;
  if (ws && !aligned16(ws)) return MLM_E_ALIGN;
  hipStream_t st = (hipStream_t)stream;
  const int dt = dims->dtype;
  float* sk = dt == MLM_BF16 ? (float*)ws : nullptr;
  GemmArgs g = gemm_fwd(L.T, L.Fl, dims->H, u2, A_r, y_r);   // Y_r = GeLU(X A_r + a_r), Eq. 3
  g.epi = EPI_BIAS_GELU;
  g.bias = a_r;
  g.aux = g_r; g.ldaux = L.Fl;
  g.gelu_tanh = dims->gelu_tanh;
  MLM_TRY_HIP(run_gemm(dt, g, st, sk));
  MLM_TRY_HIP(run_gemm(dt, gemm_fwd(L.T, dims->H, L.Fl, y_r, B_r, partial_r), st, sk));   // partial of Z = Y B
  return MLM_OK;
}

static int mlp_shard_bwd_impl(const mlm_dims* dims, const void* dx2, const void* u2, const void* A_r, const void* B_r,
                              const void* g_r, const void* y_r, void* dA_r, void* da_r, void* dB_r,
                              void* du2_partial_r, void* ws, size_t ws_bytes, void* stream, void* dg_out) {
  // dg_out != NULL: input-gradient-only form (dG left in dg_out for mlm_layer_shard_wgrads; u2, y_r, dA_r, dB_r unused)
  const bool defer = dg_out != nullptr;
  Local L;
  int rc = check_dims(dims, &L);
  if (rc) return rc;
  if (!dx2 || !A_r || !B_r || !g_r || !da_r || !du2_partial_r || !ws) return MLM_E_NULL;
  if (!defer && (!u2 || !y_r || !dA_r || !dB_r)) return MLM_E_NULL;
  if (!aligned16(dx2) || !aligned16(A_r) || !aligned16(B_r) || !aligned16(g_r) || !aligned16(du2_partial_r) ||
      !aligned16(ws) || (defer && !aligned16(dg_out)) ||
      (!defer && (!aligned16(u2) || !aligned16(y_r) || !aligned16(dA_r) || !aligned16(dB_r))))
    return MLM_E_ALIGN;
  if (ws_bytes < ws_bytes_for(dims, L, MLM_WS_MLP_BWD)) return MLM_E_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  const int dt = dims->dtype;
  const size_t T = (size_t)L.T;
  char* w = (char*)ws;
  void* dg = defer ? dg_out : (void*)w;   w += align256(T * L.Fl * L.esz);
  float* csws = (float*)w;        w += align256(((T + kColsumRowsPerBlock - 1) / kColsumRowsPerBlock) * L.Fl * 4);
  float* sk = dt == MLM_BF16 ? (float*)w : nullptr;
  if (!defer) MLM_TRY_HIP(run_gemm(dt, gemm_wgrad(L.Fl, dims->H, L.T, y_r, dx2, dB_r), st, sk));
  GemmArgs g = gemm_dgrad(L.T, L.Fl, dims->H, dx2, B_r, dg);   // dG = (dX2 B_r^T) o GeLU'(G)
  g.epi = EPI_DGELU;
  g.aux = const_cast<void*>(g_r); g.ldaux = L.Fl;
  g.gelu_tanh = dims->gelu_tanh;
  MLM_TRY_HIP(run_gemm(dt, g, st, sk));
  MLM_TRY_HIP(launch_colsum(dt, L.T, L.Fl, dg, da_r, csws, st));
  if (!defer) MLM_TRY_HIP(run_gemm(dt, gemm_wgrad(dims->H, L.Fl, L.T, u2, dg, dA_r), st, sk));
  MLM_TRY_HIP(run_gemm(dt, gemm_dgrad(L.T, dims->H, L.Fl, dg, A_r, du2_partial_r), st, sk));
  return MLM_OK;
}

MLM_API int mlm_mlp_shard_bwd(const mlm_dims* dims, const void* dx2, const void* u2, const void* A_r, const void* B_r,
                      const void* g_r, const void* y_r, void* dA_r, void* da_r, void* dB_r, void* du2_partial_r,
                      void* ws, size_t ws_bytes, void* stream) {
  return mlp_shard_bwd_impl(dims, dx2, u2, A_r, B_r, g_r, y_r, dA_r, da_r, dB_r, du2_partial_r, ws, ws_bytes, stream,
                            nullptr);
}

MLM_API int mlm_mlp_shard_bwd_input(const mlm_dims* dims, const void* dx2, const void* A_r, const void* B_r,
                                    const void* g_r, void* dg_r, void* da_r, void* du2_partial_r, void* ws,
                                    size_t ws_bytes, void* stream) {
  if (!dg_r) return MLM_E_NULL;
  return mlp_shard_bwd_impl(dims, dx2, nullptr, A_r, B_r, g_r, nullptr, nullptr, da_r, nullptr, du2_partial_r, ws,
                            ws_bytes, stream, dg_r);
}

MLM_API int mlm_layer_shard_wgrads(const mlm_dims* dims, const void* u, const void* dqkv_r, const void* ctx_r,
                                   const void* dz1, const void* u2, const void* dg_r, const void* y_r, const void* dz2,
                                   void* dWqkv_r, void* dWo_r, void* dA_r, void* dB_r, void* ws, size_t ws_bytes,
                                   void* stream) {
  Local L;
  int rc = check_dims(dims, &L);
  if (rc) return rc;
  const void* in[8] = {u, dqkv_r, ctx_r, dz1, u2, dg_r, y_r, dz2};
  void* out[4] = {dWqkv_r, dWo_r, dA_r, dB_r};
  for (const void* p : in) if (!p) return MLM_E_NULL;
  for (void* p : out) if (!p) return MLM_E_NULL;
  for (const void* p : in) if (!aligned16(p)) return MLM_E_ALIGN;
  for (void* p : out) if (!aligned16(p)) return MLM_E_ALIGN;
  const size_t need = dims->dtype == MLM_BF16 ? kSplitKBytes : 0;
  if (ws_bytes < need || (need && !ws)) return MLM_E_WORKSPACE;
  if (ws && !aligned16(ws)) return MLM_E_ALIGN;
  hipStream_t st = (hipStream_t)stream;
  // k = tokens in all four: dW = X^T dY
  GemmArgs g[4] = {gemm_wgrad(L.Fl, dims->H, L.T, y_r, dz2, dB_r), gemm_wgrad(dims->H, L.Fl, L.T, u2, dg_r, dA_r),
                   gemm_wgrad(dims->H, 3 * L.Hl, L.T, u, dqkv_r, dWqkv_r), gemm_wgrad(L.Hl, dims->H, L.T, ctx_r, dz1, dWo_r)};
  if (dims->dtype == MLM_BF16) return hip_status(launch_gemm_bf16_wgrad_group(g, 4, (float*)ws, st));
  for (int q = 0; q < 4; ++q) MLM_TRY_HIP(launch_gemm_f32(g[q], st));
  return MLM_OK;
}

MLM_API int mlm_vocab_ce_shard_fwd(const mlm_dims* dims, const void* hf, const void* E_r, const int32_t* targets, float* m_r,
                           float* s_r, float* t_r, void* logits_r, void* ws, size_t ws_bytes, void* stream) {
  Local L;
  int rc = check_dims(dims, &L);
  if (rc) return rc;
  if (!hf || !E_r || !targets || !m_r || !s_r || !t_r || !ws) return MLM_E_NULL;
  if (!aligned16(hf) || !aligned16(E_r) || !aligned16(ws) || (logits_r && !aligned16(logits_r))) return MLM_E_ALIGN;
  if (ws_bytes < ws_bytes_for(dims, L, MLM_WS_VOCAB_CE_FWD)) return MLM_E_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  const int v0 = dims->r * L.Vl;
  if (dims->dtype == MLM_BF16) {
    const size_t T = (size_t)L.T;
    const size_t ntile_max = ((size_t)L.Vl + 127) / 128;
    char* w = (char*)ws;
    float* part_m = (float*)w;    w += align256(ntile_max * T * 4);
    float* part_s = (float*)w;    w += align256(ntile_max * T * 4);
    float* t_ws = (float*)w;      w += align256(T * 4);
    GemmArgs g = gemm_fwd(L.T, L.Vl, dims->H, hf, E_r, logits_r);
    g.splitk_ws = (float*)w;
    g.epi = EPI_CE;
    g.targets = targets; g.v0 = v0;
    g.part_m = part_m; g.part_s = part_s; g.t_out = t_ws;
    const int ntiles = gemm_bf16_ce_col_tiles(g.M, g.N, g.K);
    MLM_TRY_HIP(launch_gemm_bf16(g, st));
    MLM_TRY_HIP(launch_ce_tile_merge(L.T, ntiles, part_m, part_s, t_ws, targets, v0, v0 + L.Vl, m_r, s_r, t_r, st));
  } else {
    float* lg = logits_r ? (float*)logits_r : (float*)ws;
    MLM_TRY_HIP(launch_gemm_f32(gemm_fwd(L.T, L.Vl, dims->H, hf, E_r, lg), st));
    MLM_TRY_HIP(launch_ce_rows_f32(L.T, L.Vl, lg, targets, v0, m_r, s_r, t_r, st));
  }
  return MLM_OK;
}

MLM_API int mlm_vocab_ce_merge(const mlm_dims* dims, const float* m, const float* s, const float* t, int32_t n_shards,
                       const float* loss_w, float* ce, float* M, float* S, float* loss_out, void* stream) {
  Local L;
  int rc = check_dims(dims, &L);
  if (rc) return rc;
  if (!m || !s || !t || !ce || !M || !S || !loss_out) return MLM_E_NULL;
  if (n_shards < 1 || n_shards > dims->p) return MLM_E_SHAPE;
  return hip_status(launch_ce_merge(L.T, n_shards, m, s, t, loss_w, ce, M, S, loss_out, (hipStream_t)stream));
}

MLM_API int mlm_vocab_ce_shard_bwd(const mlm_dims* dims, const void* hf, const void* E_r, const int32_t* targets,
                           const float* loss_w, const float* M, const float* S, const float* loss_stats,
                           void* logits_r, void* dE_r, void* dhf_partial_r, void* ws, size_t ws_bytes, void* stream) {
  Local L;
  int rc = check_dims(dims, &L);
  if (rc) return rc;
  if (!hf || !E_r || !targets || !M || !S || !loss_stats || !dE_r || !dhf_partial_r) return MLM_E_NULL;
  if (!ws) return MLM_E_NULL;
  if (!aligned16(hf) || !aligned16(E_r) || !aligned16(dE_r) || !aligned16(dhf_partial_r) ||
      (logits_r && !aligned16(logits_r)) || !aligned16(ws))
    return MLM_E_ALIGN;
  if (ws_bytes < ws_bytes_for(dims, L, MLM_WS_VOCAB_CE_BWD)) return MLM_E_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  const int dt = dims->dtype;
  const int v0 = dims->r * L.Vl;
  float* sk = dt == MLM_BF16 ? (float*)((char*)ws + align256((size_t)L.T * L.Vl * L.esz)) : nullptr;
  void* dL = logits_r;
  if (logits_r) {
    MLM_TRY_HIP(launch_dlogits_inplace(dt, L.T, L.Vl, logits_r, targets, v0, M, S, loss_w, loss_stats, st));
  } else {
    dL = ws;
    GemmArgs g = gemm_fwd(L.T, L.Vl, dims->H, hf, E_r, dL);   // recompute L_r = hf E_r, emit dL_r directly
    g.epi = EPI_DLOGITS;
    g.targets = targets; g.v0 = v0;
    g.Mrow = M; g.Srow = S; g.loss_w = loss_w; g.loss_stats = loss_stats;
    MLM_TRY_HIP(run_gemm(dt, g, st, sk));
  }
  MLM_TRY_HIP(run_gemm(dt, gemm_wgrad(dims->H, L.Vl, L.T, hf, dL, dE_r), st, sk));
  MLM_TRY_HIP(run_gemm(dt, gemm_dgrad(L.T, dims->H, L.Vl, dL, E_r, dhf_partial_r), st, sk));
  return MLM_OK;
}

MLM_API int mlm_embed_shard_fwd(const mlm_dims* dims, const int32_t* ids, const void* E_r, int32_t* perm_r,
                                void* partial_r, void* stream) {
  Local L;
  int rc = check_dims(dims, &L);
  if (rc) return rc;
  if (!ids || !E_r || !perm_r || !partial_r) return MLM_E_NULL;
  if (!aligned16(E_r) || !aligned16(partial_r)) return MLM_E_ALIGN;
  return hip_status(launch_embed_fwd(dims->dtype, L.T, dims->H, L.Vl, dims->r * L.Vl, ids, E_r, perm_r, partial_r,
                                     (hipStream_t)stream));
}

MLM_API int mlm_embed_bwd_replicated(const mlm_dims* dims, const void* dx0, const mlm_dropout* drop, void* dz0,
                                     void* dpos, void* stream) {
  Local L;
  int rc = check_dims(dims, &L);
  if (rc) return rc;
  if ((rc = check_drop(drop))) return rc;
  if (!dx0 || (!dz0 && !dpos)) return MLM_E_NULL;
  if (drop && drop->p > 0.0f && !dz0) return MLM_E_NULL;
  if (!aligned16(dx0) || (dz0 && !aligned16(dz0)) || (dpos && !aligned16(dpos))) return MLM_E_ALIGN;
  return hip_status(launch_embed_bwd_replicated(dims->dtype, dims->b, dims->s, dims->H, dx0, dz0, dpos, drop,
                                                (hipStream_t)stream));
}

MLM_API int mlm_embed_shard_bwd(const mlm_dims* dims, const int32_t* ids, const int32_t* perm_r, const void* dz0,
                                void* dE_r, void* stream) {
  Local L;
  int rc = check_dims(dims, &L);
  if (rc) return rc;
  if (!ids || !perm_r || !dz0 || !dE_r) return MLM_E_NULL;
  if (!aligned16(dz0) || !aligned16(dE_r)) return MLM_E_ALIGN;
  return hip_status(launch_embed_bwd(dims->dtype, L.T, dims->H, L.Vl, dims->r * L.Vl, ids, perm_r, dz0, dE_r,
                                     (hipStream_t)stream));
}

MLM_API int mlm_rows_gather(const mlm_dims* dims, const void* x, const int32_t* row_idx, int32_t n, int32_t n_out,
                            void* out, void* stream) {
  Local L;
  int rc = check_dims(dims, &L);
  if (rc) return rc;
  if (!x || !row_idx || !out) return MLM_E_NULL;
  if (n < 0 || n > L.T || n_out < n || n_out < 1) return MLM_E_SHAPE;
  if (!aligned16(x) || !aligned16(out)) return MLM_E_ALIGN;
  return hip_status(launch_rows_gather(dims->dtype, n, n_out, dims->H, row_idx, x, out, (hipStream_t)stream));
}

MLM_API int mlm_rows_scatter(const mlm_dims* dims, const void* y, const int32_t* row_idx, int32_t n, void* out,
                             void* stream) {
  Local L;
  int rc = check_dims(dims, &L);
  if (rc) return rc;
  if (!y || !row_idx || !out) return MLM_E_NULL;
  if (n < 0 || n > L.T) return MLM_E_SHAPE;
  if (!aligned16(y) || !aligned16(out)) return MLM_E_ALIGN;
  return hip_status(launch_rows_scatter(dims->dtype, n, L.T, dims->H, row_idx, y, out, (hipStream_t)stream));
}

MLM_API int mlm_gemm(int32_t dtype, int32_t trans_a, int32_t trans_b, int64_t M, int64_t N, int64_t K, const void* A,
             const void* B, void* C, const void* bias, void* stream) {
  if (dtype != MLM_F32 && dtype != MLM_BF16) return MLM_E_DTYPE;
  if (!A || !B || !C) return MLM_E_NULL;
  if (M <= 0 || N <= 0 || K <= 0 || M > (1 << 21) || N > (1 << 21) || K > (1 << 24)) return MLM_E_SHAPE;
  if ((trans_a != 0 && trans_a != 1) || (trans_b != 0 && trans_b != 1)) return MLM_E_SHAPE;
  if (trans_a && trans_b) return MLM_E_UNSUPPORTED;
  if (M % 8 || N % 8 || K % 8) return MLM_E_ALIGN;
  if (!aligned16(A) || !aligned16(B) || !aligned16(C) || (bias && !aligned16(bias))) return MLM_E_ALIGN;
  GemmArgs g = gemm_args((int)M, (int)N, (int)K, A, trans_a ? (int)M : (int)K, trans_a ? 0 : 1, B,
                         trans_b ? (int)K : (int)N, trans_b ? 1 : 0, C, (int)N);
  g.bias = bias;
  return hip_status(run_gemm(dtype, g, (hipStream_t)stream));
}

}  // extern "C"
