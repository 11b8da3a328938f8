"""Thin ctypes binding of libmlm_shard.so: same names as include/mlm_shard.h, argument marshalling only.

Tensors are torch CUDA tensors (PyTorch is used for device memory and streams, nothing else); every
call is enqueued on torch's current stream.  There is no fallback: if the HIP library is missing the
import of a function raises, loudly.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import torch

MLM_F32, MLM_BF16 = 0, 1
(WS_LAYERNORM_BWD, WS_ATTN_FWD, WS_ATTN_BWD, WS_MLP_FWD, WS_MLP_BWD, WS_COLSUM,
 WS_VOCAB_CE_FWD, WS_VOCAB_CE_BWD) = range(8)

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libmlm_shard.so")

EXPORTS = ("mlm_shard_range", "mlm_workspace_bytes", "mlm_status_string", "mlm_layernorm_fwd", "mlm_layernorm_bwd",
           "mlm_combine", "mlm_combine_layernorm_fwd", "mlm_combine_layernorm_bwd", "mlm_colsum", "mlm_attn_shard_fwd", "mlm_attn_shard_bwd", "mlm_mlp_shard_fwd",
           "mlm_mlp_shard_bwd", "mlm_vocab_ce_shard_fwd", "mlm_vocab_ce_merge", "mlm_vocab_ce_shard_bwd", "mlm_gemm", "mlm_grad_sqnorm",
           "mlm_adamw_step", "mlm_adamw_step_multi", "mlm_rng_stream_seed", "mlm_combine_dropout",
           "mlm_combine_layernorm_fwd_dropout", "mlm_combine_layernorm_bwd_dropout", "mlm_attn_keep_words",
           "mlm_attn_shard_fwd_dropout", "mlm_attn_shard_bwd_dropout", "mlm_embed_shard_fwd", "mlm_embed_bwd_replicated",
           "mlm_embed_shard_bwd", "mlm_rows_gather", "mlm_rows_scatter", "mlm_mlp_shard_bwd_input",
           "mlm_attn_shard_bwd_input", "mlm_layer_shard_wgrads", "mlm_colsum_noalloc", "mlm_deferred_sums_bytes",
           "mlm_deferred_sums_begin", "mlm_deferred_sums_flush")
STREAM_REPLICATED, STREAM_MODEL_PARALLEL = 0, 1


class MlmError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {status_string(code)} ({code})")


class Dims(ctypes.Structure):
    _fields_ = [("b", ctypes.c_int32), ("s", ctypes.c_int32), ("H", ctypes.c_int32), ("h", ctypes.c_int32),
                ("F", ctypes.c_int32), ("V", ctypes.c_int32), ("p", ctypes.c_int32), ("r", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("causal", ctypes.c_int32), ("gelu_tanh", ctypes.c_int32),
                ("ln_eps", ctypes.c_float)]


class Dropout(ctypes.Structure):
    """One dropout site: probability, stream seed (mlm_rng_stream_seed) and the 64-bit offset that names the site."""
    _fields_ = [("p", ctypes.c_float), ("seed", ctypes.c_uint64), ("offset", ctypes.c_uint64)]


def make_dropout(p: float, seed: int, offset: int) -> Dropout:
    return Dropout(float(p), int(seed) & 0xFFFFFFFFFFFFFFFF, int(offset) & 0xFFFFFFFFFFFFFFFF)


def _d(drop: Optional[Dropout]):
    return ctypes.byref(drop) if drop is not None else ctypes.c_void_p(0)


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is not built; run `python -m paper_1909_08053_amd.build` "
                               "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        L.mlm_status_string.restype = ctypes.c_char_p
        L.mlm_status_string.argtypes = [ctypes.c_int]
        for name in EXPORTS:
            if name != "mlm_status_string":
                getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def status_string(code: int) -> str:
    return lib().mlm_status_string(int(code)).decode()


def make_dims(b, s, H, h, F, V, p, r, dtype, causal=True, gelu_tanh=True, ln_eps=1e-5) -> Dims:
    return Dims(int(b), int(s), int(H), int(h), int(F), int(V), int(p), int(r), int(dtype), int(bool(causal)),
                int(bool(gelu_tanh)), float(ln_eps))


def _p(t: Optional[torch.Tensor]):
    if t is None:
        return ctypes.c_void_p(0)
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous CUDA tensor")
    return ctypes.c_void_p(t.data_ptr())


def _st(stream):
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream
    return ctypes.c_void_p(int(stream))


def _ws(ws: Optional[torch.Tensor]):
    if ws is None:
        return ctypes.c_void_p(0), ctypes.c_size_t(0)
    return _p(ws), ctypes.c_size_t(ws.numel() * ws.element_size())


def _chk(rc: int, where: str):
    if rc != 0:
        raise MlmError(rc, where)


def mlm_shard_range(n: int, p: int, r: int):
    b, e = ctypes.c_int64(0), ctypes.c_int64(0)
    _chk(lib().mlm_shard_range(ctypes.c_int64(n), ctypes.c_int32(p), ctypes.c_int32(r), ctypes.byref(b),
                               ctypes.byref(e)), "mlm_shard_range")
    return b.value, e.value


def mlm_workspace_bytes(dims: Dims, which: int) -> int:
    n = ctypes.c_size_t(0)
    _chk(lib().mlm_workspace_bytes(ctypes.byref(dims), ctypes.c_int32(which), ctypes.byref(n)), "mlm_workspace_bytes")
    return n.value


def mlm_layernorm_fwd(dims, x, gamma, beta, y, mean, rstd, stream=None):
    _chk(lib().mlm_layernorm_fwd(ctypes.byref(dims), _p(x), _p(gamma), _p(beta), _p(y), _p(mean), _p(rstd),
                                 _st(stream)), "mlm_layernorm_fwd")


def mlm_layernorm_bwd(dims, dy, x, gamma, mean, rstd, residual_grad, dx, dgamma, dbeta, ws, stream=None):
    _chk(lib().mlm_layernorm_bwd(ctypes.byref(dims), _p(dy), _p(x), _p(gamma), _p(mean), _p(rstd), _p(residual_grad),
                                 _p(dx), _p(dgamma), _p(dbeta), *_ws(ws), _st(stream)), "mlm_layernorm_bwd")


def mlm_combine(dims, partials: Sequence[torch.Tensor], bias, residual, out, stream=None):
    n = len(partials)
    arr = (ctypes.c_void_p * max(n, 1))(*[t.data_ptr() for t in partials])
    for t in partials:
        _p(t)
    _chk(lib().mlm_combine(ctypes.byref(dims), arr, ctypes.c_int32(n), _p(bias), _p(residual), _p(out), _st(stream)),
         "mlm_combine")


def _partial_array(partials):
    n = len(partials)
    for t in partials:
        _p(t)
    return (ctypes.c_void_p * max(n, 1))(*[t.data_ptr() for t in partials]), n


def mlm_combine_layernorm_fwd(dims, partials: Sequence[torch.Tensor], bias, residual, x_out, gamma, beta, y, mean, rstd,
                              stream=None):
    arr, n = _partial_array(partials)
    _chk(lib().mlm_combine_layernorm_fwd(ctypes.byref(dims), arr, ctypes.c_int32(n), _p(bias), _p(residual), _p(x_out),
                                         _p(gamma), _p(beta), _p(y), _p(mean), _p(rstd), _st(stream)),
         "mlm_combine_layernorm_fwd")


def mlm_combine_layernorm_bwd(dims, partials: Sequence[torch.Tensor], x, gamma, mean, rstd, residual_grad, dy_out, dx,
                              dgamma, dbeta, dx_colsum, ws, stream=None):
    arr, n = _partial_array(partials)
    _chk(lib().mlm_combine_layernorm_bwd(ctypes.byref(dims), arr, ctypes.c_int32(n), _p(x), _p(gamma), _p(mean),
                                         _p(rstd), _p(residual_grad), _p(dy_out), _p(dx), _p(dgamma), _p(dbeta),
                                         _p(dx_colsum), *_ws(ws), _st(stream)), "mlm_combine_layernorm_bwd")


def mlm_colsum(dims, dy, dbias, ws, stream=None):
    _chk(lib().mlm_colsum(ctypes.byref(dims), _p(dy), _p(dbias), *_ws(ws), _st(stream)), "mlm_colsum")


def mlm_colsum_noalloc(dims, dy, dbias, stream=None):
    _chk(lib().mlm_colsum_noalloc(ctypes.byref(dims), _p(dy), _p(dbias), _st(stream)), "mlm_colsum_noalloc")


def mlm_deferred_sums_bytes(dims) -> int:
    n = ctypes.c_size_t(0)
    _chk(lib().mlm_deferred_sums_bytes(ctypes.byref(dims), ctypes.byref(n)), "mlm_deferred_sums_bytes")
    return int(n.value)


def mlm_deferred_sums_begin(buf):
    _chk(lib().mlm_deferred_sums_begin(*_ws(buf)), "mlm_deferred_sums_begin")


def mlm_deferred_sums_flush(stream=None):
    _chk(lib().mlm_deferred_sums_flush(_st(stream)), "mlm_deferred_sums_flush")


def mlm_attn_shard_fwd(dims, u, Wqkv_r, bqkv_r, Wo_r, key_len, qkv_r, ctx_r, lse_r, partial_r, ws=None, stream=None):
    _chk(lib().mlm_attn_shard_fwd(ctypes.byref(dims), _p(u), _p(Wqkv_r), _p(bqkv_r), _p(Wo_r), _p(key_len), _p(qkv_r),
                                  _p(ctx_r), _p(lse_r), _p(partial_r), *_ws(ws), _st(stream)), "mlm_attn_shard_fwd")


def mlm_attn_shard_bwd(dims, dx1, u, Wqkv_r, Wo_r, key_len, qkv_r, ctx_r, lse_r, dWqkv_r, dbqkv_r, dWo_r,
                       du_partial_r, ws, stream=None):
    _chk(lib().mlm_attn_shard_bwd(ctypes.byref(dims), _p(dx1), _p(u), _p(Wqkv_r), _p(Wo_r), _p(key_len), _p(qkv_r),
                                  _p(ctx_r), _p(lse_r), _p(dWqkv_r), _p(dbqkv_r), _p(dWo_r), _p(du_partial_r),
                                  *_ws(ws), _st(stream)), "mlm_attn_shard_bwd")


def mlm_mlp_shard_fwd(dims, u2, A_r, a_r, B_r, g_r, y_r, partial_r, ws=None, stream=None):
    _chk(lib().mlm_mlp_shard_fwd(ctypes.byref(dims), _p(u2), _p(A_r), _p(a_r), _p(B_r), _p(g_r), _p(y_r),
                                 _p(partial_r), *_ws(ws), _st(stream)), "mlm_mlp_shard_fwd")


def mlm_mlp_shard_bwd(dims, dx2, u2, A_r, B_r, g_r, y_r, dA_r, da_r, dB_r, du2_partial_r, ws, stream=None):
    _chk(lib().mlm_mlp_shard_bwd(ctypes.byref(dims), _p(dx2), _p(u2), _p(A_r), _p(B_r), _p(g_r), _p(y_r), _p(dA_r),
                                 _p(da_r), _p(dB_r), _p(du2_partial_r), *_ws(ws), _st(stream)), "mlm_mlp_shard_bwd")


def mlm_vocab_ce_shard_fwd(dims, hf, E_r, targets, m_r, s_r, t_r, logits_r, ws, stream=None):
    _chk(lib().mlm_vocab_ce_shard_fwd(ctypes.byref(dims), _p(hf), _p(E_r), _p(targets), _p(m_r), _p(s_r), _p(t_r),
                                      _p(logits_r), *_ws(ws), _st(stream)), "mlm_vocab_ce_shard_fwd")


def mlm_vocab_ce_merge(dims, m, s, t, n_shards, loss_w, ce, M, S, loss_out, stream=None):
    _chk(lib().mlm_vocab_ce_merge(ctypes.byref(dims), _p(m), _p(s), _p(t), ctypes.c_int32(n_shards), _p(loss_w),
                                  _p(ce), _p(M), _p(S), _p(loss_out), _st(stream)), "mlm_vocab_ce_merge")


def mlm_vocab_ce_shard_bwd(dims, hf, E_r, targets, loss_w, M, S, loss_stats, logits_r, dE_r, dhf_partial_r, ws,
                           stream=None):
    _chk(lib().mlm_vocab_ce_shard_bwd(ctypes.byref(dims), _p(hf), _p(E_r), _p(targets), _p(loss_w), _p(M), _p(S),
                                      _p(loss_stats), _p(logits_r), _p(dE_r), _p(dhf_partial_r), *_ws(ws),
                                      _st(stream)), "mlm_vocab_ce_shard_bwd")


def mlm_gemm(dtype, trans_a, trans_b, M, N, K, A, B, C, bias=None, stream=None):
    _chk(lib().mlm_gemm(ctypes.c_int32(dtype), ctypes.c_int32(trans_a), ctypes.c_int32(trans_b), ctypes.c_int64(M),
                        ctypes.c_int64(N), ctypes.c_int64(K), _p(A), _p(B), _p(C), _p(bias), _st(stream)), "mlm_gemm")


def mlm_grad_sqnorm(dtype, grads: Sequence[torch.Tensor], other_sqnorm, sqnorm_out, ws, stream=None):
    n = len(grads)
    for t in grads:
        _p(t)
    arr = (ctypes.c_void_p * max(n, 1))(*[t.data_ptr() for t in grads])
    cnt = (ctypes.c_int64 * max(n, 1))(*[t.numel() for t in grads])
    _chk(lib().mlm_grad_sqnorm(ctypes.c_int32(dtype), arr, cnt, ctypes.c_int32(n), _p(other_sqnorm), _p(sqnorm_out),
                               *_ws(ws), _st(stream)), "mlm_grad_sqnorm")


def mlm_adamw_step(dtype, grad, master, m, v, weight_out, total_sqnorm, max_norm, lr, beta1, beta2, eps, weight_decay,
                   step, stream=None):
    f = ctypes.c_float
    _chk(lib().mlm_adamw_step(ctypes.c_int32(dtype), ctypes.c_int64(grad.numel()), _p(grad), _p(master), _p(m), _p(v),
                              _p(weight_out), _p(total_sqnorm), f(max_norm), f(lr), f(beta1), f(beta2), f(eps),
                              f(weight_decay), ctypes.c_int32(step), _st(stream)), "mlm_adamw_step")


def mlm_adamw_step_multi(dtype, grads, masters, ms, vs, weights_out, weight_decays, total_sqnorm, max_norm, lr, beta1,
                         beta2, eps, step, stream=None):
    n = len(grads)
    ptrs = lambda ts: (ctypes.c_void_p * n)(*[(_p(t).value or 0) for t in ts])
    cnt = (ctypes.c_int64 * n)(*[t.numel() for t in grads])
    wds = (ctypes.c_float * n)(*[float(x) for x in weight_decays])
    f = ctypes.c_float
    _chk(lib().mlm_adamw_step_multi(ctypes.c_int32(dtype), ctypes.c_int32(n), cnt, ptrs(grads), ptrs(masters), ptrs(ms),
                                    ptrs(vs), ptrs(weights_out), wds, _p(total_sqnorm), f(max_norm), f(lr), f(beta1),
                                    f(beta2), f(eps), ctypes.c_int32(step), _st(stream)), "mlm_adamw_step_multi")


# ---- dropout (two random streams) and the input embedding -------------------------------------------------------
def mlm_rng_stream_seed(base_seed: int, stream: int, r: int) -> int:
    out = ctypes.c_uint64(0)
    _chk(lib().mlm_rng_stream_seed(ctypes.c_uint64(base_seed & 0xFFFFFFFFFFFFFFFF), ctypes.c_int32(stream),
                                   ctypes.c_int32(r), ctypes.byref(out)), "mlm_rng_stream_seed")
    return out.value


def mlm_combine_dropout(dims, partials, bias, bias_rows, drop, residual, out, stream=None):
    arr, n = _partial_array(partials)
    _chk(lib().mlm_combine_dropout(ctypes.byref(dims), arr, ctypes.c_int32(n), _p(bias), ctypes.c_int32(bias_rows),
                                   _d(drop), _p(residual), _p(out), _st(stream)), "mlm_combine_dropout")


def mlm_combine_layernorm_fwd_dropout(dims, partials, bias, drop, residual, x_out, gamma, beta, y, mean, rstd,
                                      stream=None):
    arr, n = _partial_array(partials)
    _chk(lib().mlm_combine_layernorm_fwd_dropout(ctypes.byref(dims), arr, ctypes.c_int32(n), _p(bias), _d(drop),
                                                 _p(residual), _p(x_out), _p(gamma), _p(beta), _p(y), _p(mean),
                                                 _p(rstd), _st(stream)), "mlm_combine_layernorm_fwd_dropout")


def mlm_combine_layernorm_bwd_dropout(dims, partials, x, gamma, mean, rstd, residual_grad, drop, dy_out, dx, dz_out,
                                      dgamma, dbeta, dx_colsum, ws, stream=None):
    arr, n = _partial_array(partials)
    _chk(lib().mlm_combine_layernorm_bwd_dropout(ctypes.byref(dims), arr, ctypes.c_int32(n), _p(x), _p(gamma),
                                                 _p(mean), _p(rstd), _p(residual_grad), _d(drop), _p(dy_out), _p(dx),
                                                 _p(dz_out), _p(dgamma), _p(dbeta), _p(dx_colsum), *_ws(ws),
                                                 _st(stream)), "mlm_combine_layernorm_bwd_dropout")


def mlm_attn_keep_words(dims) -> int:
    n = ctypes.c_size_t(0)
    _chk(lib().mlm_attn_keep_words(ctypes.byref(dims), ctypes.byref(n)), "mlm_attn_keep_words")
    return n.value


def mlm_attn_shard_fwd_dropout(dims, u, Wqkv_r, bqkv_r, Wo_r, key_len, drop, qkv_r, ctx_r, lse_r, keep_bits_r,
                               partial_r, ws=None, stream=None):
    _chk(lib().mlm_attn_shard_fwd_dropout(ctypes.byref(dims), _p(u), _p(Wqkv_r), _p(bqkv_r), _p(Wo_r), _p(key_len),
                                          _d(drop), _p(qkv_r), _p(ctx_r), _p(lse_r), _p(keep_bits_r), _p(partial_r),
                                          *_ws(ws), _st(stream)), "mlm_attn_shard_fwd_dropout")


def mlm_attn_shard_bwd_dropout(dims, dx1, u, Wqkv_r, Wo_r, key_len, drop, qkv_r, ctx_r, lse_r, keep_bits_r, dWqkv_r,
                               dbqkv_r, dWo_r, du_partial_r, ws, stream=None):
    _chk(lib().mlm_attn_shard_bwd_dropout(ctypes.byref(dims), _p(dx1), _p(u), _p(Wqkv_r), _p(Wo_r), _p(key_len),
                                          _d(drop), _p(qkv_r), _p(ctx_r), _p(lse_r), _p(keep_bits_r), _p(dWqkv_r),
                                          _p(dbqkv_r), _p(dWo_r), _p(du_partial_r), *_ws(ws), _st(stream)),
         "mlm_attn_shard_bwd_dropout")


def mlm_embed_shard_fwd(dims, ids, E_r, perm_r, partial_r, stream=None):
    _chk(lib().mlm_embed_shard_fwd(ctypes.byref(dims), _p(ids), _p(E_r), _p(perm_r), _p(partial_r), _st(stream)),
         "mlm_embed_shard_fwd")


def mlm_embed_bwd_replicated(dims, dx0, drop, dz0, dpos, stream=None):
    _chk(lib().mlm_embed_bwd_replicated(ctypes.byref(dims), _p(dx0), _d(drop), _p(dz0), _p(dpos), _st(stream)),
         "mlm_embed_bwd_replicated")


def mlm_embed_shard_bwd(dims, ids, perm_r, dz0, dE_r, stream=None):
    _chk(lib().mlm_embed_shard_bwd(ctypes.byref(dims), _p(ids), _p(perm_r), _p(dz0), _p(dE_r), _st(stream)),
         "mlm_embed_shard_bwd")


def mlm_rows_gather(dims, x, row_idx, n, n_out, out, stream=None):
    _chk(lib().mlm_rows_gather(ctypes.byref(dims), _p(x), _p(row_idx), ctypes.c_int32(n), ctypes.c_int32(n_out), _p(out),
                               _st(stream)), "mlm_rows_gather")


def mlm_rows_scatter(dims, y, row_idx, n, out, stream=None):
    _chk(lib().mlm_rows_scatter(ctypes.byref(dims), _p(y), _p(row_idx), ctypes.c_int32(n), _p(out), _st(stream)),
         "mlm_rows_scatter")


# ---- backward with the weight gradients deferred to one grouped launch -------------------------------------------
def mlm_mlp_shard_bwd_input(dims, dx2, A_r, B_r, g_r, dg_r, da_r, du2_partial_r, ws, stream=None):
    _chk(lib().mlm_mlp_shard_bwd_input(ctypes.byref(dims), _p(dx2), _p(A_r), _p(B_r), _p(g_r), _p(dg_r), _p(da_r),
                                       _p(du2_partial_r), *_ws(ws), _st(stream)), "mlm_mlp_shard_bwd_input")


def mlm_attn_shard_bwd_input(dims, dx1, Wqkv_r, Wo_r, key_len, drop, qkv_r, ctx_r, lse_r, keep_bits_r, dqkv_r, dbqkv_r,
                             du_partial_r, ws, stream=None):
    _chk(lib().mlm_attn_shard_bwd_input(ctypes.byref(dims), _p(dx1), _p(Wqkv_r), _p(Wo_r), _p(key_len), _d(drop),
                                        _p(qkv_r), _p(ctx_r), _p(lse_r), _p(keep_bits_r), _p(dqkv_r), _p(dbqkv_r),
                                        _p(du_partial_r), *_ws(ws), _st(stream)), "mlm_attn_shard_bwd_input")


def mlm_layer_shard_wgrads(dims, u, dqkv_r, ctx_r, dz1, u2, dg_r, y_r, dz2, dWqkv_r, dWo_r, dA_r, dB_r, ws, stream=None):
    _chk(lib().mlm_layer_shard_wgrads(ctypes.byref(dims), _p(u), _p(dqkv_r), _p(ctx_r), _p(dz1), _p(u2), _p(dg_r),
                                      _p(y_r), _p(dz2), _p(dWqkv_r), _p(dWo_r), _p(dA_r), _p(dB_r), *_ws(ws),
                                      _st(stream)), "mlm_layer_shard_wgrads")
