/*
 * mlm_shard.h -- C ABI of the MI355X (gfx950) layer-shard library.
 *
 * One GPU's share of a tensor-parallel transformer layer and of the
 * vocabulary-parallel loss, forward and backward, as formulated in Section 3 of
 * "Megatron-LM: Training Multi-Billion Parameter Language Models Using Model
 * Parallelism" (arXiv 1909.08053):
 *   - MLP block:  Y_r = GeLU(X A_r)  with A split by columns (Eq. 1 and Eq. 3),
 *                 Z   = sum_r Y_r B_r with B split by rows (partials, then reduce);
 *   - attention:  Q/K/V GEMMs split by columns so that each head is local to a
 *                 shard, output projection split by rows (Section 3, Fig. 3b);
 *   - loss:       logits split by vocabulary, [Y_1, Y_2] = [X E_1, X E_2], fused
 *                 with the cross entropy so that only b x s scalars are exchanged;
 *   - f / g:      the conjugate operators (identity / all-reduce) are replaced
 *                 on a single GPU by mlm_combine and mlm_vocab_ce_merge.
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers unless the comment says "host".
 *   - Matrices are row-major and dense (leading dimension = number of columns).
 *     Activations are [T, .] with T = b*s and token index t = batch*s + position.
 *     Weights are stored [in, out], exactly as the paper writes X A: a column-
 *     parallel shard is a block of columns, a row-parallel shard a block of rows,
 *     each passed as its own dense matrix.
 *   - dims.dtype selects the storage type of every activation / weight / gradient
 *     tensor: MLM_F32 (float) or MLM_BF16 (bfloat16 storage, fp32 accumulation).
 *     Statistics (mean, rstd, lse, m, s, t, ce, M, S, loss) are always float.
 *   - Ownership: the caller owns every buffer, the workspace included.  The library
 *     allocates nothing, creates no streams and never synchronises; kernels are
 *     enqueued on the given stream (a hipStream_t passed as void*, NULL = default).
 *     Inputs are read-only; outputs are fully overwritten unless stated otherwise.
 *   - Errors: every call returns 0 (MLM_OK) or a negative mlm_status.  Arguments are
 *     validated on the host before anything is launched, so a call that fails
 *     validation has launched nothing; MLM_E_HIP (a launch that the runtime refused)
 *     can leave the earlier kernels of the same call enqueued.  No exceptions cross
 *     the ABI.
 *   - Process-wide state: none that a result depends on.  The library keeps (a) per
 *     kernel and device, whether its dynamic-LDS attribute has been set; (b) the
 *     address of mlm_colsum_noalloc's static scratch per device; (c) per host thread,
 *     the list that mlm_deferred_sums_begin opens and mlm_deferred_sums_flush closes;
 *     (d) five tuning
 *     overrides that are read from the environment ONCE per process, at the first
 *     bf16 GEMM: MLM_GEMM_V2=0 (register-staged kernel instead of the direct-to-LDS
 *     one), MLM_GEMM_TILE=0|1|2 (tile of the register-staged kernel), MLM_GEMM_WAVES=4|8,
 *     MLM_GEMM_BN=192|256 (tile width where both exist), MLM_GEMM_GROUP=0 (weight
 *     gradients launched one by one).  They choose between kernels that compute the
 *     same sums in a different order and exist for A/B measurements; unset, the
 *     library chooses by its cost model.  Calls may come from several host threads.
 *   - H, H/p, F/p, V/p and the head size must be multiples of 8 and pointers 16-byte
 *     aligned (MLM_E_ALIGN otherwise).  Supported head sizes: 64, 96, 128, 192 (MLM_BF16);
 *     any multiple of 16 up to 128 (MLM_F32).  H <= 4096 (MLM_BF16) / 2048 (MLM_F32).
 */
#ifndef MLM_SHARD_H
#define MLM_SHARD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Every entry point is exported from the shared library with default visibility. */
#define MLM_API __attribute__((visibility("default")))

typedef enum mlm_status {
  MLM_OK = 0,
  MLM_E_NULL = -1,       /* a required pointer is NULL                              */
  MLM_E_SHAPE = -2,      /* non-positive size, h % p, F % p, V % p, H % h != 0, r outside [0,p), or a size
                            beyond the launch limits: b*s <= 2^21 tokens, b <= 65535, H, F/p, V/p <= 2^20 */
  MLM_E_DTYPE = -3,      /* dtype is neither MLM_F32 nor MLM_BF16                   */
  MLM_E_WORKSPACE = -4,  /* workspace smaller than mlm_workspace_bytes reports      */
  MLM_E_ALIGN = -5,      /* size or pointer alignment requirement of MLM_BF16 violated */
  MLM_E_HIP = -6,        /* a HIP call or kernel launch failed                      */
  MLM_E_UNSUPPORTED = -7 /* e.g. head size not compiled in                          */
} mlm_status;

enum { MLM_F32 = 0, MLM_BF16 = 1 };

/* Global (unsharded) sizes in the paper's notation plus the shard id. */
typedef struct mlm_dims {
  int32_t b;         /* batch size                                            */
  int32_t s;         /* sequence length                                       */
  int32_t H;         /* hidden size                                           */
  int32_t h;         /* attention heads (global); head size d = H / h         */
  int32_t F;         /* MLP inner width (4H in the paper's models)            */
  int32_t V;         /* padded vocabulary size v                              */
  int32_t p;         /* number of model-parallel shards                       */
  int32_t r;         /* this shard, 0 <= r < p                                */
  int32_t dtype;     /* MLM_F32 or MLM_BF16                                   */
  int32_t causal;    /* 1: key j visible to query i iff j <= i (GPT-2); 0: bidirectional (BERT) */
  int32_t gelu_tanh; /* 1: tanh form of GeLU; 0: exact (erf) form             */
  float ln_eps;      /* layer-norm epsilon                                    */
} mlm_dims;

/* Which call a workspace size is asked for. */
enum {
  MLM_WS_LAYERNORM_BWD = 0,
  MLM_WS_ATTN_FWD = 1,
  MLM_WS_ATTN_BWD = 2,
  MLM_WS_MLP_FWD = 3,
  MLM_WS_MLP_BWD = 4,
  MLM_WS_COLSUM = 5,
  MLM_WS_VOCAB_CE_FWD = 6,
  MLM_WS_VOCAB_CE_BWD = 7,
  MLM_WS_COUNT = 8
};

/* ---- host-side integer helpers ------------------------------------------------ */

/* Shard r's contiguous index range [begin, end) of n items split p ways (Section 3:
 * heads, MLP columns/rows and vocabulary are all split into equal contiguous blocks;
 * Section 5.1 pads the vocabulary so that it divides).  begin/end: host pointers.
 * MLM_E_SHAPE if p <= 0, r outside [0,p), n < 0 or n % p != 0. */
MLM_API int mlm_shard_range(int64_t n, int32_t p, int32_t r, int64_t* begin, int64_t* end);

/* Bytes of workspace call `which` (MLM_WS_*) needs for `dims`; *bytes is a host
 * pointer.  A workspace must be 256-byte aligned.  A size of 0 means the call accepts
 * ws == NULL. */
MLM_API int mlm_workspace_bytes(const mlm_dims* dims, int32_t which, size_t* bytes);

/* Human-readable name of a status code (static storage, never NULL). */
MLM_API const char* mlm_status_string(int code);

/* ---- replicated work (Section 3: layer norm and residual are duplicated on every
 *      GPU rather than computed once and broadcast) ------------------------------- */

/* y = (x - mean) * rstd * gamma + beta per token over H (Section 2.2: layer norm on the
 * input of the attention and MLP blocks).  x, y: [T,H] dtype; gamma, beta: [H] dtype;
 * mean, rstd: [T] float outputs (biased variance, rstd = 1/sqrt(var + ln_eps)). */
MLM_API int mlm_layernorm_fwd(const mlm_dims* dims, const void* x, const void* gamma, const void* beta,
                      void* y, float* mean, float* rstd, void* stream);

/* Backward of mlm_layernorm_fwd fused with the residual branch:
 *   dx = residual_grad + d(LN)/dx applied to dy      (residual_grad may be NULL = 0)
 *   dgamma = sum_t dy * xhat,  dbeta = sum_t dy       ([H] dtype outputs)
 * dy, x, residual_grad, dx: [T,H] dtype (dx may alias residual_grad or dy).
 * ws: MLM_WS_LAYERNORM_BWD bytes. */
MLM_API int mlm_layernorm_bwd(const mlm_dims* dims, const void* dy, const void* x, const void* gamma,
                      const float* mean, const float* rstd, const void* residual_grad,
                      void* dx, void* dgamma, void* dbeta, void* ws, size_t ws_bytes, void* stream);

/* The reduction that stands in for the all-reduce of g (forward) and f (backward) on one
 * GPU (Section 3, Fig. 3): out = sum_i partials[i] + bias + residual.
 * partials: HOST array of n_partials device pointers, each [T,H] dtype (1 <= n_partials <= 16);
 * bias: [H] dtype or NULL -- the row-parallel bias, added once after the sum;
 * residual: [T,H] dtype or NULL; out: [T,H] dtype (may alias residual or a partial). */
MLM_API int mlm_combine(const mlm_dims* dims, const void* const* partials, int32_t n_partials,
                const void* bias, const void* residual, void* out, void* stream);

/* mlm_combine fused with the layer norm that consumes its result (Section 3: the all-reduced
 * block output plus bias and residual is normalised identically on every GPU):
 *   x_out = sum_i partials[i] + bias + residual      (rounded once to dtype and stored)
 *   y = layer norm of x_out with gamma, beta;  mean, rstd as in mlm_layernorm_fwd.
 * Arguments as in mlm_combine and mlm_layernorm_fwd; x_out: [T,H] dtype, may alias residual
 * or a partial; y must not alias an input. */
MLM_API int mlm_combine_layernorm_fwd(const mlm_dims* dims, const void* const* partials, int32_t n_partials,
                              const void* bias, const void* residual, void* x_out, const void* gamma,
                              const void* beta, void* y, float* mean, float* rstd, void* stream);

/* mlm_combine (no bias, no residual) fused with mlm_layernorm_bwd: the layer-norm gradient reads
 *   dy = sum_i partials[i]   (rounded once to dtype; also stored to dy_out unless dy_out is NULL)
 * -- the stand-in for f's backward all-reduce feeding the replicated layer norm -- and produces
 * dx, dgamma, dbeta as mlm_layernorm_bwd does.  If dx_colsum is not NULL it also receives
 * dx_colsum[j] = sum_t dx[t,j] ([H] dtype): the gradient of the replicated bias that was added
 * to form this layer norm's input (output-projection bias, second MLP bias), so no separate
 * mlm_colsum pass over dx is needed.  dx may alias residual_grad; dy_out must not alias an
 * input.  ws: MLM_WS_LAYERNORM_BWD bytes. */
MLM_API int mlm_combine_layernorm_bwd(const mlm_dims* dims, const void* const* partials, int32_t n_partials,
                              const void* x, const void* gamma, const float* mean, const float* rstd,
                              const void* residual_grad, void* dy_out, void* dx, void* dgamma, void* dbeta,
                              void* dx_colsum, void* ws, size_t ws_bytes, void* stream);

/* Column sums over tokens, dbias[j] = sum_t dy[t,j]: the gradient of a replicated bias
 * (output-projection bias, second MLP bias).  dy: [T,H] dtype; dbias: [H] dtype.
 * ws: MLM_WS_COLSUM bytes. */
MLM_API int mlm_colsum(const mlm_dims* dims, const void* dy, void* dbias, void* ws, size_t ws_bytes, void* stream);

/* mlm_colsum for callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): same arguments without the workspace,
 * same kernels, same result bit for bit.  The per-chunk partial sums go to a static device
 * array inside the library (4 MiB per GPU, held until the process ends) instead of a caller
 * workspace; the call allocates and frees nothing.
 * Limit: ceil(T / 64) * H <= 1,048,576 floats (e.g. T = 8192 with H <= 8192); beyond that
 * MLM_E_WORKSPACE is returned and nothing is launched.
 * The first call on a device looks up that device's copy of the array (once per device; make
 * that call outside a graph capture).  All calls on one GPU share the array: calls that
 * overlap in time on the same GPU (different streams) race and must be serialised by the
 * caller.  Nothing in the array has to start at zero (every slot a call reads, it has
 * written first), so it is never cleared. */
MLM_API int mlm_colsum_noalloc(const mlm_dims* dims, const void* dy, void* dbias, void* stream);

/* Deferred finishing sums.  The gradients of the layer-norm weights and of the biases
 * (dgamma, dbeta, dx_colsum of mlm_layernorm_bwd / mlm_combine_layernorm_bwd[_dropout],
 * dbias of mlm_colsum, dbqkv_r of mlm_attn_shard_bwd[_input][_dropout], da_r of
 * mlm_mlp_shard_bwd[_input]) are column sums over all tokens (Section 3: each GPU sums its
 * own tokens; no communication).  Every such call forms per-block partial sums and then
 * launches a small kernel that adds them up; nothing else in a backward pass reads the
 * result.  Between mlm_deferred_sums_begin and mlm_deferred_sums_flush, on the calling host
 * thread, these calls keep their block partials in `buf` (bump-allocated, the calls' own
 * workspaces stay free for reuse) and leave the vectors above UNWRITTEN; flush adds all of
 * them up in ONE launch on `stream`, which must be the stream of those calls (or ordered
 * after them).  The sums are bit-identical to the undeferred ones (same kernel code, same
 * order).  buf: device memory, 256-byte aligned, untouched by the caller until the flush
 * has run; mlm_deferred_sums_bytes gives a size that holds one transformer layer's backward
 * plus the final layer norm (*bytes is a host pointer).  A call whose partials do not fit
 * what is left of buf, or the 17th call of a list, simply finishes inside the call as
 * usual, so a short buffer is never an error.  mlm_colsum_noalloc is never deferred.
 * State: one open list per HOST THREAD (thread-local; the only state in the library that
 * outlives a call besides the items listed at the top).  begin: MLM_E_UNSUPPORTED if the
 * thread already has an open list; flush: MLM_E_UNSUPPORTED if it has none.  flush always
 * closes the list, also when its launch fails.  Under stream capture both calls behave as
 * any other call here (begin launches nothing, flush records one kernel). */
MLM_API int mlm_deferred_sums_bytes(const mlm_dims* dims, size_t* bytes);
MLM_API int mlm_deferred_sums_begin(void* buf, size_t buf_bytes);
MLM_API int mlm_deferred_sums_flush(void* stream);

/* ---- self-attention block of shard r (Section 3, Fig. 3b) ---------------------- */

/* Forward.  h_l = h/p local heads, H_l = h_l * d.
 *   qkv_r = u Wqkv_r + bqkv_r                [T, 3 H_l]  columns = [Q heads | K heads | V heads],
 *                                                        each head d contiguous columns
 *   ctx_r = softmax(mask(Q K^T / sqrt(d))) V  per local head, [T, H_l]
 *   lse_r = log sum_j exp(score_ij) over the allowed keys, [b, h_l, s] float
 *   partial_r = ctx_r Wo_r                    [T, H]  (row-parallel partial sum, NO bias)
 * u: [T,H]; Wqkv_r: [H, 3 H_l]; bqkv_r: [3 H_l] or NULL; Wo_r: [H_l, H];
 * key_len: [b] int32 or NULL -- keys j >= key_len[batch] are excluded for every query
 * (BERT-style padding); with causal also j > i is excluded.  Excluded keys get probability
 * exactly 0.  Every query row must keep at least one key: key_len is device memory the
 * host cannot validate, so every kernel reads it as max(1, min(key_len[batch], s)).
 * qkv_r, ctx_r, lse_r are saved for the backward call.  ws: MLM_WS_ATTN_FWD bytes. */
MLM_API int mlm_attn_shard_fwd(const mlm_dims* dims, const void* u, const void* Wqkv_r, const void* bqkv_r,
                       const void* Wo_r, const int32_t* key_len,
                       void* qkv_r, void* ctx_r, float* lse_r, void* partial_r,
                       void* ws, size_t ws_bytes, void* stream);

/* Backward.  dx1: [T,H] gradient w.r.t. the block's (already combined) output.
 * Outputs: dWqkv_r [H, 3 H_l], dbqkv_r [3 H_l], dWo_r [H_l, H], and
 * du_partial_r [T,H] = d(loss)/du through this shard only (the operand of f's all-reduce).
 * ws: MLM_WS_ATTN_BWD bytes. */
MLM_API int mlm_attn_shard_bwd(const mlm_dims* dims, const void* dx1, const void* u, const void* Wqkv_r,
                       const void* Wo_r, const int32_t* key_len,
                       const void* qkv_r, const void* ctx_r, const float* lse_r,
                       void* dWqkv_r, void* dbqkv_r, void* dWo_r, void* du_partial_r,
                       void* ws, size_t ws_bytes, void* stream);

/* ---- MLP block of shard r (Section 3, Eq. 1 and Eq. 3, Fig. 3a) ---------------- */

/* Forward.  F_l = F/p.
 *   g_r = u2 A_r + a_r       [T, F_l]  pre-activation (saved)
 *   y_r = GeLU(g_r)          [T, F_l]  (saved)
 *   partial_r = y_r B_r      [T, H]    (row-parallel partial sum, NO bias)
 * u2: [T,H]; A_r: [H, F_l]; a_r: [F_l] or NULL; B_r: [F_l, H].  ws: MLM_WS_MLP_FWD bytes. */
MLM_API int mlm_mlp_shard_fwd(const mlm_dims* dims, const void* u2, const void* A_r, const void* a_r,
                      const void* B_r, void* g_r, void* y_r, void* partial_r,
                      void* ws, size_t ws_bytes, void* stream);

/* Backward.  dx2: [T,H] gradient w.r.t. the block's combined output.
 * Outputs: dA_r [H, F_l], da_r [F_l], dB_r [F_l, H], du2_partial_r [T,H].
 * ws: MLM_WS_MLP_BWD bytes. */
MLM_API int mlm_mlp_shard_bwd(const mlm_dims* dims, const void* dx2, const void* u2, const void* A_r,
                      const void* B_r, const void* g_r, const void* y_r,
                      void* dA_r, void* da_r, void* dB_r, void* du2_partial_r,
                      void* ws, size_t ws_bytes, void* stream);

/* ---- vocabulary-parallel output embedding fused with the loss (Section 3) ------ */

/* Forward of shard r.  V_l = V/p, shard r owns vocabulary ids [r V_l, (r+1) V_l).
 *   L_r = hf E_r                               [T, V_l]
 *   m_r[t] = max_j L_r[t,j];  s_r[t] = sum_j exp(L_r[t,j] - m_r[t])
 *   t_r[t] = L_r[t, targets[t] - r V_l] if the target id lies in the shard's range, else 0
 * hf: [T,H]; E_r: [H, V_l]; targets: [T] int32 GLOBAL ids in [0,V);
 * m_r, s_r, t_r: [T] float outputs -- the only values a multi-GPU run would exchange;
 * logits_r: [T, V_l] dtype output kept for the backward call, or NULL (backward then
 * recomputes the logits).  ws: MLM_WS_VOCAB_CE_FWD bytes. */
MLM_API int mlm_vocab_ce_shard_fwd(const mlm_dims* dims, const void* hf, const void* E_r, const int32_t* targets,
                           float* m_r, float* s_r, float* t_r, void* logits_r,
                           void* ws, size_t ws_bytes, void* stream);

/* Merge of the per-shard partials (stands in for the all-reduces of the b x s scalars):
 *   M = max_r m_r;  S = sum_r s_r exp(m_r - M);  ce = log S + M - sum_r t_r;
 *   loss_out[0] = sum_t w_t ce_t / sum_t w_t;  loss_out[1] = sum_t w_t.
 * m, s, t: [n_shards, T] float (shard-major, contiguous); loss_w: [T] float weights in {0,1}
 * or NULL (all ones); ce, M, S: [T] float outputs; loss_out: [2] float output. */
MLM_API int mlm_vocab_ce_merge(const mlm_dims* dims, const float* m, const float* s, const float* t,
                       int32_t n_shards, const float* loss_w, float* ce, float* M, float* S,
                       float* loss_out, void* stream);

/* Backward of shard r.
 *   dL_r[t,j] = w_t / sum(w) * (exp(L_r[t,j] - M[t]) / S[t] - [j == targets[t] - r V_l])
 *   dE_r = hf^T dL_r            [H, V_l]
 *   dhf_partial_r = dL_r E_r^T  [T, H]   (operand of f's all-reduce)
 * M, S: [T] from mlm_vocab_ce_merge; loss_stats: the [2] array loss_out of the merge (device);
 * logits_r: the array saved by the forward call -- it is OVERWRITTEN with dL_r -- or NULL,
 * in which case the logits are recomputed into the workspace.  ws: MLM_WS_VOCAB_CE_BWD bytes. */
MLM_API int mlm_vocab_ce_shard_bwd(const mlm_dims* dims, const void* hf, const void* E_r, const int32_t* targets,
                           const float* loss_w, const float* M, const float* S, const float* loss_stats,
                           void* logits_r, void* dE_r, void* dhf_partial_r,
                           void* ws, size_t ws_bytes, void* stream);

/* ---- optimizer step of one model-parallel worker (Section 4.2: Adam with decoupled weight decay
 *      0.01, global gradient-norm clipping at 1.0, mixed precision; Section 3: every worker
 *      optimises its own parameters, no parameter values are communicated) ----------------- */

/* sqnorm_out[0] = sum over the n_tensors gradient tensors of the sum of squares of their
 * elements (fp32, fixed summation order), plus other_sqnorm[0] if that is not NULL -- the
 * other workers' term of the GLOBAL norm, which on several GPUs is the one scalar all-reduce of
 * the step.  grads: HOST array of n_tensors device pointers (1 <= n_tensors <= 64), counts:
 * HOST array of their element counts (multiples of 8 for MLM_BF16, 4 for MLM_F32);
 * other_sqnorm, sqnorm_out: device.  ws: n_tensors * 4096 bytes, 16-byte aligned. */
MLM_API int mlm_grad_sqnorm(int32_t dtype, const void* const* grads, const int64_t* counts, int32_t n_tensors,
                    const float* other_sqnorm, float* sqnorm_out, void* ws, size_t ws_bytes, void* stream);

/* One AdamW update of one parameter tensor of `count` elements (step is 1-based):
 *   g <- grad * min(1, max_norm / (sqrt(total_sqnorm[0]) + 1e-6))      (max_norm <= 0: no clipping,
 *                                                                        total_sqnorm may be NULL)
 *   m <- beta1 m + (1 - beta1) g;   v <- beta2 v + (1 - beta2) g^2
 *   master <- master - lr ( (m / (1 - beta1^step)) / (sqrt(v / (1 - beta2^step)) + eps)
 *                           + weight_decay * master )
 *   weight_out <- master rounded to dtype        (NULL: not written)
 * grad, weight_out: dtype; master, m, v: fp32, updated in place; total_sqnorm: device (from
 * mlm_grad_sqnorm).  Everything 16-byte aligned; count a multiple of 8 (MLM_BF16) / 4 (MLM_F32). */
MLM_API int mlm_adamw_step(int32_t dtype, int64_t count, const void* grad, float* master, float* m, float* v,
                   void* weight_out, const float* total_sqnorm, float max_norm, float lr, float beta1,
                   float beta2, float eps, float weight_decay, int32_t step, void* stream);

/* mlm_adamw_step over n_tensors parameter tensors in ONE launch per 32 tensors (a worker owns many
 * small tensors -- biases, layer-norm vectors -- whose separate launches would dominate the step).
 * counts, grads, masters, ms, vs, weights_out, weight_decays: HOST arrays of n_tensors entries
 * (1 <= n_tensors <= 64); the device buffers they name are as in mlm_adamw_step; weights_out[t] may
 * be NULL; weight_decays[t] is tensor t's decay (0 for tensors that are not decayed). */
MLM_API int mlm_adamw_step_multi(int32_t dtype, int32_t n_tensors, const int64_t* counts, const void* const* grads,
                         float* const* masters, float* const* ms, float* const* vs, void* const* weights_out,
                         const float* weight_decays, const float* total_sqnorm, float max_norm, float lr,
                         float beta1, float beta2, float eps, int32_t step, void* stream);

/* ---- dropout with the two model-parallel random streams (Appendix B.2; the rate, p = 0.1 everywhere,
 *      is in Section 4.2) and the variants of the calls above that apply it ------------------- */

/* One dropout site.  The paper asks for two random streams: one seeded identically on every
 * model-parallel worker for the dropouts OUTSIDE the model-parallel regions (embedding output, the two
 * block outputs before their residual adds), so that the replicated tensors stay identical, and one
 * seeded uniquely per worker for the dropout INSIDE the attention block.  It fixes neither the
 * generator nor the seed rule; this library uses the counter-based Philox4x32-10 generator:
 * element e (row-major index in the tensor this worker holds) reads 32-bit word e mod 4 of the block
 * with counter (lo32(e/4), hi32(e/4), lo32(offset), hi32(offset)) under key (lo32(seed), hi32(seed)),
 * and is kept iff that word >= floor(p 2^32); kept values are scaled by 1/(1-p).  The decision is
 * integer work and reproducible from (seed, offset, e) alone. */
typedef struct mlm_dropout {
  float p;         /* drop probability, 0 <= p < 1 (MLM_E_SHAPE otherwise); 0 = identity            */
  uint64_t seed;   /* stream seed, see mlm_rng_stream_seed                                          */
  uint64_t offset; /* names the site (layer, call, training step); the caller keeps sites distinct  */
} mlm_dropout;

enum { MLM_STREAM_REPLICATED = 0, MLM_STREAM_MODEL_PARALLEL = 1 };

/* Seed of a stream on worker r (host, integer): the replicated stream's seed is base_seed on every
 * worker; worker r's model-parallel seed is base_seed + 1 + r (mod 2^64), distinct from the replicated
 * one and from every other worker's.  seed: host pointer.  MLM_E_SHAPE for an unknown stream or r < 0. */
MLM_API int mlm_rng_stream_seed(uint64_t base_seed, int32_t stream, int32_t r, uint64_t* seed);

/* mlm_combine with dropout on the reduced block output (Section 3: dropout and the residual add are
 * replicated work on the reduced tensor):  out = residual + dropout(sum_i partials[i] + bias).  bias is [bias_rows, H]
 * (row t uses bias row t mod bias_rows; bias_rows = 1 is the ordinary bias vector, bias_rows = s adds a
 * position embedding) or NULL.  drop NULL or p = 0: no dropout.  Element index of the site: t H + column. */
MLM_API int mlm_combine_dropout(const mlm_dims* dims, const void* const* partials, int32_t n_partials,
                        const void* bias, int32_t bias_rows, const mlm_dropout* drop, const void* residual,
                        void* out, void* stream);

/* mlm_combine_layernorm_fwd with dropout:  x_out = residual + dropout(sum_i partials[i] + bias), then the
 * layer norm of x_out.  Other arguments as in mlm_combine_layernorm_fwd. */
MLM_API int mlm_combine_layernorm_fwd_dropout(const mlm_dims* dims, const void* const* partials, int32_t n_partials,
                                      const void* bias, const mlm_dropout* drop, const void* residual,
                                      void* x_out, const void* gamma, const void* beta, void* y, float* mean,
                                      float* rstd, void* stream);

/* mlm_combine_layernorm_bwd for a layer norm whose input was formed WITH dropout
 * (x = residual + dropout(z)): besides dx it emits dz_out = dropout-mask(dx) / (1-p), the gradient of the
 * block output z before dropout ([T,H] dtype) -- the tensor the row-parallel GEMM's backward consumes --
 * and dx_colsum becomes the column sums of dz_out (the gradient of the bias inside z).  drop must name
 * the same site as the forward call (NULL or p = 0: dz_out = dx).  dz_out must not alias dx. */
MLM_API int mlm_combine_layernorm_bwd_dropout(const mlm_dims* dims, const void* const* partials, int32_t n_partials,
                                      const void* x, const void* gamma, const float* mean, const float* rstd,
                                      const void* residual_grad, const mlm_dropout* drop, void* dy_out, void* dx,
                                      void* dz_out, void* dgamma, void* dbeta, void* dx_colsum, void* ws,
                                      size_t ws_bytes, void* stream);

/* Number of 32-bit words of the keep-bit tensor mlm_attn_shard_fwd_dropout saves: [b, h_l, s, pitch] with
 * pitch = 4 ceil(s / 128) words per query row (bit j mod 32 of word j / 32 = key j kept).  words: host. */
MLM_API int mlm_attn_keep_words(const mlm_dims* dims, size_t* words);

/* mlm_attn_shard_fwd with dropout on the attention probabilities (the dropout inside the model-parallel
 * region; drop->seed is this worker's model-parallel stream):
 *   ctx_r = (keep o softmax(...) / (1-p)) V;  lse_r is the log-sum-exp of the UNdropped scores.
 * Element index of the site: ((batch h_l + local head) s + query) s + key; s must be a multiple of 4
 * (MLM_E_ALIGN).  keep_bits_r: uint32 output of mlm_attn_keep_words words, saved for the backward call;
 * only bits of allowed (query, key) pairs are defined. */
MLM_API int mlm_attn_shard_fwd_dropout(const mlm_dims* dims, const void* u, const void* Wqkv_r, const void* bqkv_r,
                               const void* Wo_r, const int32_t* key_len, const mlm_dropout* drop,
                               void* qkv_r, void* ctx_r, float* lse_r, uint32_t* keep_bits_r, void* partial_r,
                               void* ws, size_t ws_bytes, void* stream);

/* Backward of mlm_attn_shard_fwd_dropout: as mlm_attn_shard_bwd, with the saved keep bits and the same
 * drop->p (the generator is not run again). */
MLM_API int mlm_attn_shard_bwd_dropout(const mlm_dims* dims, const void* dx1, const void* u, const void* Wqkv_r,
                               const void* Wo_r, const int32_t* key_len, const mlm_dropout* drop,
                               const void* qkv_r, const void* ctx_r, const float* lse_r,
                               const uint32_t* keep_bits_r, void* dWqkv_r, void* dbqkv_r, void* dWo_r,
                               void* du_partial_r, void* ws, size_t ws_bytes, void* stream);

/* ---- backward of a layer shard with the weight gradients deferred ---------------
 * Section 3 puts the synchronisation points on the ACTIVATION gradients (the operator f); a weight gradient
 * dW = X^T dY is local to its GPU and nothing but the optimizer waits for it.  The two calls below are the
 * backward calls above without their weight-gradient GEMMs -- they leave the gradients of the column-parallel
 * activations in caller buffers instead -- and mlm_layer_shard_wgrads then computes the four weight gradients
 * of the layer shard together: their GEMMs share one launch, hence one partially filled last round of the
 * 256 compute units instead of four (each with its own k-split and fix-up pass). */

/* mlm_mlp_shard_bwd without dA_r / dB_r.  dg_r: [T, F_l] dtype OUTPUT, dG = (dx2 B_r^T) o GeLU'(g_r). */
MLM_API int mlm_mlp_shard_bwd_input(const mlm_dims* dims, const void* dx2, const void* A_r, const void* B_r,
                            const void* g_r, void* dg_r, void* da_r, void* du2_partial_r,
                            void* ws, size_t ws_bytes, void* stream);

/* mlm_attn_shard_bwd(_dropout) without dWqkv_r / dWo_r.  dqkv_r: [T, 3 H_l] dtype OUTPUT, the gradient of
 * qkv_r.  drop / keep_bits_r as in mlm_attn_shard_bwd_dropout (both NULL: no dropout). */
MLM_API int mlm_attn_shard_bwd_input(const mlm_dims* dims, const void* dx1, const void* Wqkv_r, const void* Wo_r,
                             const int32_t* key_len, const mlm_dropout* drop, const void* qkv_r,
                             const void* ctx_r, const float* lse_r, const uint32_t* keep_bits_r,
                             void* dqkv_r, void* dbqkv_r, void* du_partial_r,
                             void* ws, size_t ws_bytes, void* stream);

/* The four weight gradients of the layer shard:
 *   dWqkv_r = u^T dqkv_r   [H, 3 H_l]      dWo_r = ctx_r^T dz1   [H_l, H]
 *   dA_r    = u2^T dg_r    [H, F_l]        dB_r  = y_r^T dz2     [F_l, H]
 * dz1 / dz2: the [T,H] gradients the two backward calls were given as dx1 / dx2 (still intact).
 * ws: MLM_WS_MLP_BWD bytes is enough. */
MLM_API int mlm_layer_shard_wgrads(const mlm_dims* dims, const void* u, const void* dqkv_r, const void* ctx_r,
                           const void* dz1, const void* u2, const void* dg_r, const void* y_r, const void* dz2,
                           void* dWqkv_r, void* dWo_r, void* dA_r, void* dB_r,
                           void* ws, size_t ws_bytes, void* stream);

/* ---- vocabulary-parallel input embedding (Section 3: the input embedding shares its weights with the
 *      output embedding E [H, v] and is split along the vocabulary like it; a shard holds only its slice of
 *      the table, so the shards' lookups are partial results that the operator g sums) ------------------ */

/* Forward of shard r:  partial_r[t, :] = E_r[:, ids[t] - r V_l] if the id lies in the shard's range,
 * else 0.  ids: [T] int32 GLOBAL ids in [0, V); E_r: [H, V_l] (the matrix of mlm_vocab_ce_shard_fwd);
 * partial_r: [T,H] dtype; perm_r: [T] int32 output saved for the backward call -- the tokens in stable
 * order of their local id (ids outside the shard last); integer work, exact.  The sort is a brute-force
 * rank computation, O(T^2) comparisons: meant for T = b s of a few thousand to a few ten thousand.
 * The partials are reduced with mlm_combine_dropout (bias = position embedding [s,H], bias_rows = s,
 * drop = the replicated stream's embedding site). */
MLM_API int mlm_embed_shard_fwd(const mlm_dims* dims, const int32_t* ids, const void* E_r, int32_t* perm_r,
                        void* partial_r, void* stream);

/* Replicated part of the embedding backward:  dz0 = dropout-mask(dx0) / (1-p)  (drop NULL: dz0 = dx0) and
 * dpos[i, :] = sum over the batch of dz0[batch s + i, :]  ([s,H] dtype; NULL: not computed).
 * dx0, dz0: [T,H] dtype; dz0 may alias dx0. */
MLM_API int mlm_embed_bwd_replicated(const mlm_dims* dims, const void* dx0, const mlm_dropout* drop, void* dz0,
                             void* dpos, void* stream);

/* Backward of shard r:  dE_r[:, c] += sum over the tokens t with ids[t] - r V_l == c of dz0[t, :], added
 * in token order (deterministic) ON TOP of what dE_r holds -- the output embedding's gradient from
 * mlm_vocab_ce_shard_bwd, since the two embeddings are one parameter.  Columns no token names are left
 * untouched.  perm_r: from mlm_embed_shard_fwd for the same ids. */
MLM_API int mlm_embed_shard_bwd(const mlm_dims* dims, const int32_t* ids, const int32_t* perm_r, const void* dz0,
                        void* dE_r, void* stream);

/* ---- loss rows only (Section 4: BERT is trained by language-model masking, so the loss sits on a subset of the
 *      positions; the vocabulary-parallel logits GEMM, the dominant cost, is needed for those rows only) */

/* out[k, :] = x[row_idx[k], :] for k < n and zeros for n <= k < n_out.  x: [T,H] dtype; row_idx: [n] int32
 * DEVICE array of token rows, strictly increasing, each in [0, T) (not checked on the device: the caller
 * builds it from the loss mask); out: [n_out, H] dtype.  The compact tensor is then passed to the
 * mlm_vocab_ce_* calls with dims whose b * s equals n_out (padding rows carry loss weight 0). */
MLM_API int mlm_rows_gather(const mlm_dims* dims, const void* x, const int32_t* row_idx, int32_t n, int32_t n_out,
                    void* out, void* stream);

/* Inverse of mlm_rows_gather for the gradient: out[row_idx[k], :] = y[k, :] for k < n, every other row of
 * out [T,H] is set to zero.  y: [>= n, H] dtype. */
MLM_API int mlm_rows_scatter(const mlm_dims* dims, const void* y, const int32_t* row_idx, int32_t n, void* out,
                     void* stream);

/* ---- the GEMM building block (Section 3: "XA", "YB", "XE") --------------------- */

/* C = op(A) op(B) (+ bias per column), row-major, fp32 accumulation.
 *   trans_a == 0: A is [M,K] (lda = K);  trans_a == 1: A is stored [K,M] (lda = M)
 *   trans_b == 0: B is [K,N] (ldb = N);  trans_b == 1: B is stored [N,K] (ldb = K)
 * C: [M,N]; bias: [N] or NULL.  dtype as in mlm_dims.  This is the kernel the block calls
 * above are built from (forward: 0/0, input gradient: 0/1, weight gradient: 1/0).
 * M, N, K multiples of 8; M, N <= 2^21, K <= 2^24 (MLM_E_SHAPE beyond); both operands
 * transposed is MLM_E_UNSUPPORTED. */
MLM_API int mlm_gemm(int32_t dtype, int32_t trans_a, int32_t trans_b, int64_t M, int64_t N, int64_t K,
             const void* A, const void* B, void* C, const void* bias, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MLM_SHARD_H */
