// Internal declarations shared by the HIP translation units of libmlm_shard (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "mlm_shard.h"

namespace mlm {

typedef __bf16 bf16;
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;

constexpr int kWave = 64;

// hipFuncSetAttribute(kernel, MaxDynamicSharedMemorySize, bytes) once per (kernel instantiation, device): the attribute
// belongs to the device's copy of the kernel, so the "done" state is a bit per device (devices beyond 63 set it on
// every launch).  A race between two host threads only repeats the idempotent call.
struct LdsAttrOnce {
  unsigned long long done = 0;
  hipError_t ensure(const void* kernel, int bytes) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const unsigned long long bit = (dev >= 0 && dev < 64) ? (1ull << dev) : 0ull;
    if (bit && (__atomic_load_n(&done, __ATOMIC_ACQUIRE) & bit)) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess && bit) __atomic_fetch_or(&done, bit, __ATOMIC_RELEASE);
    return e;
  }
};

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16 v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16 from_f32<bf16>(float v) { return (bf16)v; }   // round to nearest even

// 16-byte vector of storage elements: 4 floats or 8 bf16.
template <typename T> struct Vec16;
template <> struct Vec16<float> {
  static constexpr int N = 4;
  float4 raw;
  __device__ __forceinline__ void load(const float* p) { raw = *reinterpret_cast<const float4*>(p); }
  __device__ __forceinline__ void store(float* p) const { *reinterpret_cast<float4*>(p) = raw; }
  __device__ __forceinline__ float get(int i) const { return reinterpret_cast<const float*>(&raw)[i]; }
  __device__ __forceinline__ void set(int i, float v) { reinterpret_cast<float*>(&raw)[i] = v; }
};
template <> struct Vec16<bf16> {
  static constexpr int N = 8;
  bf16x8 raw;
  __device__ __forceinline__ void load(const bf16* p) { raw = *reinterpret_cast<const bf16x8*>(p); }
  __device__ __forceinline__ void store(bf16* p) const { *reinterpret_cast<bf16x8*>(p) = raw; }
  __device__ __forceinline__ float get(int i) const { return (float)raw[i]; }
  __device__ __forceinline__ void set(int i, float v) { raw[i] = (bf16)v; }
};

// Vector of BYTES (16 or 8) bytes of storage elements.  The narrow form exists for kernels in which a lane owns one
// vector of every row: half the elements per lane means twice the waves per row.
template <typename T, int BYTES> struct VecB;
template <typename T> struct VecB<T, 16> : Vec16<T> {};
template <> struct VecB<bf16, 8> {
  static constexpr int N = 4;
  bf16x4 raw;
  __device__ __forceinline__ void load(const bf16* p) { raw = *reinterpret_cast<const bf16x4*>(p); }
  __device__ __forceinline__ void store(bf16* p) const { *reinterpret_cast<bf16x4*>(p) = raw; }
  __device__ __forceinline__ float get(int i) const { return (float)raw[i]; }
  __device__ __forceinline__ void set(int i, float v) { raw[i] = (bf16)v; }
};

// Wave-wide reductions on the data-parallel-primitive path of the vector ALU (row shifts inside 16-lane rows, then two
// row broadcasts): seven dependent VALU operations instead of six round trips through the LDS crossbar that a shuffle
// butterfly costs.  The total ends up in lane 63 and is handed to every lane as a scalar.  The order of the additions
// is fixed, so results are reproducible run to run.
template <int CTRL, int ROW_MASK, int BANK_MASK>
__device__ __forceinline__ float dpp_move(float identity, float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, identity), __builtin_bit_cast(int, v),
                                                               CTRL, ROW_MASK, BANK_MASK, false));
}
// Sum over each row of 16 lanes; the total is in lane 15 of the row (the other lanes hold partial sums).
__device__ __forceinline__ float row16_sum(float v) {
  // lanes the shift leaves without a source, and lanes masked out, take the identity 0
  float a = v + dpp_move<0x111, 0xf, 0xf>(0.f, v);            // row_shr:1
  a += dpp_move<0x112, 0xf, 0xf>(0.f, v);                     // row_shr:2
  a += dpp_move<0x113, 0xf, 0xf>(0.f, v);                     // row_shr:3  -> sums of 4 consecutive lanes
  a += dpp_move<0x114, 0xf, 0xe>(0.f, a);                     // row_shr:4  -> of 8
  a += dpp_move<0x118, 0xf, 0xc>(0.f, a);                     // row_shr:8  -> lane 15 of each row: the row's 16
  return a;
}
__device__ __forceinline__ float lane_value(float v, int lane) {   // lane: compile-time or wave-uniform
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}
__device__ __forceinline__ float wave_sum(float v) {
  float a = row16_sum(v);
  a += dpp_move<0x142, 0xa, 0xf>(0.f, a);                     // row_bcast:15 into rows 1 and 3
  a += dpp_move<0x143, 0xc, 0xf>(0.f, a);                     // row_bcast:31 into rows 2 and 3 -> lane 63: all 64
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, a), 63));
}
__device__ __forceinline__ float wave_max(float v) {
  const float ninf = -INFINITY;
  float a = fmaxf(v, dpp_move<0x111, 0xf, 0xf>(ninf, v));
  a = fmaxf(a, dpp_move<0x112, 0xf, 0xf>(ninf, v));
  a = fmaxf(a, dpp_move<0x113, 0xf, 0xf>(ninf, v));
  a = fmaxf(a, dpp_move<0x114, 0xf, 0xe>(ninf, a));
  a = fmaxf(a, dpp_move<0x118, 0xf, 0xc>(ninf, a));
  a = fmaxf(a, dpp_move<0x142, 0xa, 0xf>(ninf, a));
  a = fmaxf(a, dpp_move<0x143, 0xc, 0xf>(ninf, a));
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, a), 63));
}

// GeLU and its derivative.  tanh form: 0.5 x (1 + tanh(u)) = x sigmoid(2u) with u = sqrt(2/pi)(x + 0.044715 x^3);
// exact form: x Phi(x).  The sigmoid is one exp2 and one reciprocal; it saturates cleanly (exp2 -> 0 or inf).
__device__ __forceinline__ float gelu_sigmoid2u(float x) {
  // 2u log2(e) = x (c0 + c1 x^2)
  const float c0 = 2.0f * 0.7978845608028654f * 1.4426950408889634f;
  const float c1 = c0 * 0.044715f;
  const float w = x * fmaf(c1, x * x, c0);
  return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-w));
}
__device__ __forceinline__ float gelu_fwd(float x, bool tanh_form) {
  if (tanh_form) return x * gelu_sigmoid2u(x);
  return 0.5f * x * (1.0f + erff(x * 0.7071067811865476f));
}
__device__ __forceinline__ float gelu_bwd(float x, bool tanh_form) {
  if (tanh_form) {
    // d/dx [x s(2u)] = s + x s (1 - s) 2 u',  u' = sqrt(2/pi)(1 + 3 * 0.044715 x^2)
    const float sg = gelu_sigmoid2u(x);
    const float du2 = 2.0f * 0.7978845608028654f * fmaf(0.134145f, x * x, 1.0f);
    return sg + x * sg * (1.0f - sg) * du2;
  }
  return 0.5f * (1.0f + erff(x * 0.7071067811865476f)) + x * __expf(-0.5f * x * x) * 0.3989422804014327f;
}

// ---- epilogues a GEMM can fuse --------------------------------------------------
enum Epilogue : int {
  EPI_STORE = 0,      // C = acc (+ bias)
  EPI_BIAS_GELU = 1,  // aux = acc + bias (pre-activation), C = GeLU(aux)
  EPI_DGELU = 2,      // C = acc * GeLU'(aux)
  EPI_CE = 3,         // per-row (max, sum-exp) partials per column tile, target logit; C = logits if C != NULL
  EPI_DLOGITS = 4     // C = coef_row * (exp(acc - Mrow)/Srow - [col + v0 == target_row])
};

struct GemmArgs {
  int M, N, K;
  const void* A; int lda; int a_kc;   // a_kc: element (m,k) at A[m*lda + k]; else at A[k*lda + m]
  const void* B; int ldb; int b_kc;   // b_kc: element (k,n) at B[n*ldb + k]; else at B[k*ldb + n]
  void* C; int ldc;
  int epi;
  const void* bias;                    // [N] storage dtype or NULL
  void* aux; int ldaux;                // EPI_BIAS_GELU: out pre-activation; EPI_DGELU: in pre-activation
  int gelu_tanh;
  // EPI_CE / EPI_DLOGITS
  const int32_t* targets;              // [M] global vocabulary ids
  int v0;                              // first vocabulary id of the shard
  float* part_m; float* part_s;        // [n_col_tiles][M] partials (EPI_CE)
  float* t_out;                        // [M] target logit, written by the owner tile only (EPI_CE)
  const float* Mrow; const float* Srow; const float* loss_w; const float* loss_stats;  // EPI_DLOGITS
  float* splitk_ws;                    // >= 64 MB of scratch for the tail split of the plain-store GEMM, or NULL
};

// Number of column tiles the bf16 CE epilogue produces partials for (depends on the tile config chosen for N).
int gemm_bf16_ce_col_tiles(int M, int N, int K);
hipError_t launch_gemm_bf16(const GemmArgs& a, hipStream_t st);
hipError_t launch_gemm_f32(const GemmArgs& a, hipStream_t st);
// n weight-gradient GEMMs (A m-contiguous, B n-contiguous, plain store) in one launch where that is faster
hipError_t launch_gemm_bf16_wgrad_group(const GemmArgs* probs, int n, float* splitk_ws, hipStream_t st);

// ---- dropout site as the kernels see it (rng.h holds the generator) ---------------
struct DropArgs {
  uint32_t k0, k1;          // key: the stream seed
  uint32_t off_lo, off_hi;  // site offset: counter words 2 and 3
  uint32_t thr;             // keep iff word >= thr = floor(p 2^32)
  float scale;              // 1 / (1 - p)
  int enabled;              // 0: identity (p == 0 or no dropout requested)
};

// ---- attention ------------------------------------------------------------------
struct AttnArgs {
  int b, s, hl, d;          // batch, sequence, local heads, head size
  int causal;
  const int32_t* key_len;   // [b] or NULL
  const void* qkv;          // [T, 3*hl*d]
  void* ctx;                // fwd out / bwd in: [T, hl*d]
  float* lse;               // [b, hl, s]
  const void* dctx;         // bwd: [T, hl*d]
  void* dqkv;               // bwd out: [T, 3*hl*d]
  float* delta;             // bwd scratch: [b, hl, s]
  // dropout of the probabilities: forward draws the mask and saves it as bits, backward reads the bits
  DropArgs drop;            // enabled = 0: no dropout
  uint32_t* keep_bits;      // [b, hl, s, keep_pitch] words; bit (j % 32) of word j / 32 of row (b, head, i): key j kept
  int keep_pitch;           // words per query row: 4 ceil(s / 128)
};
// Number of visible keys of batch row bi: key_len lives in device memory and cannot be validated by the host, so every
// kernel clamps it to [1, s] (0 or a negative length would index tiles before the buffer, a length above s keys that do
// not exist).
__device__ __forceinline__ int attn_key_len(const int32_t* key_len, int bi, int s) {
  return key_len ? max(1, min(key_len[bi], s)) : s;
}
bool attn_bf16_supported(int d);
hipError_t launch_attn_fwd_bf16(const AttnArgs& a, hipStream_t st);
hipError_t launch_attn_bwd_bf16(const AttnArgs& a, hipStream_t st);
bool attn_f32_supported(int d);
hipError_t launch_attn_fwd_f32(const AttnArgs& a, hipStream_t st);
hipError_t launch_attn_bwd_f32(const AttnArgs& a, hipStream_t st);

// ---- row / elementwise kernels (rowops.hip); dtype = MLM_F32 / MLM_BF16 ----------
constexpr int kLnBwdRowsPerBlock = 32;
constexpr int kColsumRowsPerBlock = 64;
constexpr int kMaxPartials = 16;

hipError_t launch_layernorm_fwd(int dtype, int T, int H, float eps, const void* x, const void* gamma,
                                const void* beta, void* y, float* mean, float* rstd, hipStream_t st);
// ws: [ceil(T/kLnBwdRowsPerBlock)][2][H] float (the workspace query reserves 3 parts)
hipError_t launch_layernorm_bwd(int dtype, int T, int H, const void* dy, const void* x, const void* gamma,
                                const float* mean, const float* rstd, const void* residual_grad, void* dx,
                                void* dgamma, void* dbeta, float* ws, hipStream_t st);
// Fused forms: the layer norm reads sum(partials) (+ bias + residual) instead of a stored tensor.
hipError_t launch_combine_layernorm_fwd(int dtype, int T, int H, float eps, const void* const* partials, int n,
                                        const void* bias, const void* residual, void* x_out, const void* gamma,
                                        const void* beta, void* y, float* mean, float* rstd, const mlm_dropout* drop,
                                        hipStream_t st);
// ws: [ceil(T/kLnBwdRowsPerBlock)][3][H] float; dy_out and dx_colsum may be NULL.  With drop and dz_out the kernel
// also emits dz_out = dropout-mask(dx) / (1 - p) and dx_colsum sums dz_out's columns instead of dx's.
hipError_t launch_combine_layernorm_bwd(int dtype, int T, int H, const void* const* partials, int n, const void* x,
                                        const void* gamma, const float* mean, const float* rstd,
                                        const void* residual_grad, void* dy_out, void* dx, void* dgamma, void* dbeta,
                                        void* dx_colsum, float* ws, const mlm_dropout* drop, void* dz_out,
                                        hipStream_t st);
// out = residual + dropout(sum partials + bias[t mod bias_rows])
hipError_t launch_combine(int dtype, int T, int H, const void* const* partials, int n, const void* bias,
                          int bias_rows, const void* residual, void* out, const mlm_dropout* drop, hipStream_t st);
// ws: [ceil(T/kColsumRowsPerBlock)][N] float
hipError_t launch_colsum(int dtype, int T, int N, const void* dy, void* dbias, float* ws, hipStream_t st);
// Deferred finishing sums (per host thread).  Between begin and flush, launch_layernorm_bwd,
// launch_combine_layernorm_bwd and launch_colsum keep their block partials in `buf` and leave dgamma / dbeta /
// dx_colsum / dbias unwritten; flush sums all of them in one launch (bit-identical to finishing inside each call).
// A launch whose partials do not fit the rest of `buf`, or the 17th of a list, finishes inside the call.
hipError_t deferred_sums_begin(void* buf, size_t bytes);
bool deferred_sums_open();
hipError_t deferred_sums_flush(hipStream_t st);
// same with the partials in a static device array of kStaticScratchFloats floats (no workspace argument)
constexpr size_t kStaticScratchFloats = (size_t)1 << 20;      // 4 MiB per GPU
hipError_t launch_colsum_static(int dtype, int T, int N, const void* dy, void* dbias, hipStream_t st);
hipError_t launch_ce_tile_merge(int T, int ntiles, const float* part_m, const float* part_s, const float* t_ws,
                                const int32_t* targets, int v0, int v1, float* m_r, float* s_r, float* t_r,
                                hipStream_t st);
hipError_t launch_ce_rows_f32(int T, int Vl, const float* logits, const int32_t* targets, int v0,
                              float* m_r, float* s_r, float* t_r, hipStream_t st);
hipError_t launch_ce_merge(int T, int n_shards, const float* m, const float* s, const float* t, const float* loss_w,
                           float* ce, float* M, float* S, float* loss_out, hipStream_t st);
hipError_t launch_dlogits_inplace(int dtype, int T, int Vl, void* logits, const int32_t* targets, int v0,
                                  const float* M, const float* S, const float* loss_w, const float* loss_stats,
                                  hipStream_t st);
hipError_t launch_rows_gather(int dtype, int n, int n_out, int H, const int32_t* idx, const void* x, void* out,
                              hipStream_t st);
hipError_t launch_rows_scatter(int dtype, int n, int rows, int H, const int32_t* idx, const void* y, void* out,
                               hipStream_t st);
hipError_t launch_embed_fwd(int dtype, int T, int H, int Vl, int v0, const int32_t* ids, const void* E, int32_t* perm,
                            void* partial, hipStream_t st);
hipError_t launch_embed_bwd(int dtype, int T, int H, int Vl, int v0, const int32_t* ids, const int32_t* perm,
                            const void* dz, void* dE, hipStream_t st);
hipError_t launch_embed_bwd_replicated(int dtype, int b, int s, int H, const void* dx0, void* dz0, void* dpos,
                                       const mlm_dropout* drop, hipStream_t st);
hipError_t launch_attn_delta(int dtype, int T, int hl, int d, int b, int s, const void* ctx, const void* dctx,
                             float* delta, hipStream_t st);

}  // namespace mlm
