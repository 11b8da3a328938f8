"""fp64 CPU oracle for the model-parallel transformer layer + vocab-parallel loss.

TEST INFRASTRUCTURE ONLY.  This file is the checker, not the product: only
``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import it.  It shares no code with the HIP path and imports
nothing from it.

What it computes.  The paper's claim (Section 3) is that the sharded layer
reaches exactly the unsharded result: a column split of the first MLP GEMM
commutes with GeLU (Eq. 3), a row split of the second GEMM gives partial sums
that add up to the full product, attention heads are independent, and the
vocabulary-split logits fused with the loss reproduce the ordinary cross
entropy.  So the oracle is the plain definition of the *unsharded* pre-LN
transformer layer (Section 2.2: layer norm on the input of the attention and
MLP blocks, GeLU non-linearity) followed by the output-embedding GEMM and the
mean cross entropy (Section 3 for the GEMM, Appendix E Eq. 4 for "average
cross entropy"), with hand-derived analytic gradients, all in numpy float64.
``sharded_reference`` below additionally writes out the sharded formulation
(explicit per-shard partials, explicit all-reduce stand-ins) so that tests can
check the invariants and obtain the expected per-shard tensors by definition.

Readings taken where the paper is silent (each is also listed in the design
notes): tanh-form GeLU by default (erf form available), biases exist and the
row-parallel bias is added once after the reduction, F = 4H, LN eps 1e-5 with
the biased variance, score scale 1/sqrt(d), masked probabilities exactly 0,
final LN before the output embedding (switchable), loss = mean over positions
with weight 1, targets are given per position (no shift).  Dropout is the
identity unless keep masks are handed in (``inp["drop"]``): the masks are
inputs here, the generator that draws them is oracle/rng_embed_oracle.py.

Pins (tests/test_oracle_*.py, all CPU): closed forms and identities for GeLU,
LN, softmax/attention and cross entropy; library routines (torch fp64
layer_norm, scaled_dot_product_attention, gelu, cross_entropy and autograd)
as second opinions; central finite differences for every gradient; brute-force
loops for the integer work; the sharding invariants of Section 3.
Absolute values at the benchmark configs are NOT printed in the paper:
"parity unpinned" by the paper there, pinned only transitively through the
checks above.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Dict, Optional, Tuple

import numpy as np

F64 = np.float64


@dataclass(frozen=True)
class Spec:
    """Unsharded layer dimensions and switches (notation of Section 3: b, s, H, v)."""
    b: int
    s: int
    H: int
    h: int
    F: int
    V: int
    causal: bool = True
    final_ln: bool = True
    gelu_tanh: bool = True
    ln_eps: float = 1e-5

    @property
    def T(self) -> int:
        return self.b * self.s

    @property
    def d(self) -> int:
        return self.H // self.h


# --------------------------------------------------------------------------- GeLU
_SQRT_2_OVER_PI = math.sqrt(2.0 / math.pi)


def gelu_tanh(x):
    """tanh-form GeLU, 0.5 x (1 + tanh(sqrt(2/pi) (x + 0.044715 x^3))) (Section 3, Eq. 1)."""
    x = np.asarray(x, F64)
    return 0.5 * x * (1.0 + np.tanh(_SQRT_2_OVER_PI * (x + 0.044715 * x ** 3)))


def gelu_tanh_grad(x):
    x = np.asarray(x, F64)
    u = _SQRT_2_OVER_PI * (x + 0.044715 * x ** 3)
    t = np.tanh(u)
    du = _SQRT_2_OVER_PI * (1.0 + 3.0 * 0.044715 * x ** 2)
    return 0.5 * (1.0 + t) + 0.5 * x * (1.0 - t * t) * du


def _erf(x):
    return np.vectorize(math.erf, otypes=[F64])(x)


def gelu_erf(x):
    """Exact GeLU x * Phi(x) with Phi the standard normal CDF."""
    x = np.asarray(x, F64)
    return 0.5 * x * (1.0 + _erf(x / math.sqrt(2.0)))


def gelu_erf_grad(x):
    x = np.asarray(x, F64)
    return 0.5 * (1.0 + _erf(x / math.sqrt(2.0))) + x * np.exp(-0.5 * x * x) / math.sqrt(2.0 * math.pi)


def gelu(x, tanh_form: bool = True):
    return gelu_tanh(x) if tanh_form else gelu_erf(x)


def gelu_grad(x, tanh_form: bool = True):
    return gelu_tanh_grad(x) if tanh_form else gelu_erf_grad(x)


# --------------------------------------------------------------------------- layer norm
def layernorm_fwd(x, gamma, beta, eps) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Per-token layer normalisation over the hidden axis (Section 2.2; replicated, Section 3).

    Returns (y, mean, rstd) with the biased (divide by H) variance."""
    x = np.asarray(x, F64)
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    y = (x - mu) * rstd * gamma + beta
    return y, mu[..., 0], rstd[..., 0]


def layernorm_bwd(dy, x, gamma, mu, rstd):
    """Gradient of layernorm_fwd w.r.t. x, gamma, beta (x, dy: [T, H])."""
    xhat = (x - mu[..., None]) * rstd[..., None]
    g = dy * gamma
    dx = rstd[..., None] * (g - g.mean(axis=-1, keepdims=True)
                            - xhat * (g * xhat).mean(axis=-1, keepdims=True))
    dgamma = (dy * xhat).reshape(-1, x.shape[-1]).sum(axis=0)
    dbeta = dy.reshape(-1, x.shape[-1]).sum(axis=0)
    return dx, dgamma, dbeta


# --------------------------------------------------------------------------- attention
def allowed_mask(s: int, causal: bool, key_len: int) -> np.ndarray:
    """Boolean [s, s] table: may query i attend key j?  (integer work, exact).

    causal: j <= i; key padding: j < key_len (applies to every query row)."""
    i = np.arange(s)[:, None]
    j = np.arange(s)[None, :]
    ok = (j < key_len) & (i >= 0)
    if causal:
        ok = ok & (j <= i)
    return ok


def attention_fwd(Q, K, Vv, spec: Spec, key_len: np.ndarray, keep=None, p_drop: float = 0.0):
    """softmax(mask(Q K^T / sqrt(d))) V per head (Section 3: each head's matmuls are local).

    Q, K, Vv: [b, s, H] with head k in columns [k d, (k+1) d).
    keep: optional boolean [b, h, s, s] dropout mask of the attention probabilities (the dropout inside the
    model-parallel region, Appendix B.2): C = (keep * P / (1 - p_drop)) V.  P and LSE are returned undropped.
    Returns C [b, s, H], P [b, h, s, s], LSE [b, h, s] (natural log of the masked row sum of exp(S))."""
    b, s, H, h, d = spec.b, spec.s, spec.H, spec.h, spec.d
    C = np.zeros((b, s, H), F64)
    P = np.zeros((b, h, s, s), F64)
    LSE = np.zeros((b, h, s), F64)
    scale = 1.0 / math.sqrt(d)
    for bi in range(b):
        ok = allowed_mask(s, spec.causal, int(key_len[bi]))
        for k in range(h):
            sl = slice(k * d, (k + 1) * d)
            S = (Q[bi, :, sl] @ K[bi, :, sl].T) * scale
            Sm = np.where(ok, S, -np.inf)
            mx = Sm.max(axis=-1, keepdims=True)
            e = np.where(ok, np.exp(Sm - mx), 0.0)
            den = e.sum(axis=-1, keepdims=True)
            p = e / den
            P[bi, k] = p
            LSE[bi, k] = (mx + np.log(den))[:, 0]
            if keep is not None:
                p = np.where(keep[bi, k], p, 0.0) / (1.0 - p_drop)
            C[bi, :, sl] = p @ Vv[bi, :, sl]
    return C, P, LSE


def attention_bwd(dC, Q, K, Vv, P, spec: Spec, keep=None, p_drop: float = 0.0):
    """Gradients of attention_fwd w.r.t. Q, K, V given dC (masked entries have P = 0, so dS = 0 there).

    With a dropout mask: C = Pd V with Pd = keep * P / (1 - p_drop), so dV = Pd^T dC and
    dP = keep * (dC V^T) / (1 - p_drop); the softmax gradient then acts on the undropped P."""
    b, s, H, h, d = spec.b, spec.s, spec.H, spec.h, spec.d
    dQ = np.zeros_like(Q)
    dK = np.zeros_like(K)
    dV = np.zeros_like(Vv)
    scale = 1.0 / math.sqrt(d)
    for bi in range(b):
        for k in range(h):
            sl = slice(k * d, (k + 1) * d)
            p = P[bi, k]
            if keep is None:
                dV[bi, :, sl] = p.T @ dC[bi, :, sl]
                dP = dC[bi, :, sl] @ Vv[bi, :, sl].T
            else:
                pd = np.where(keep[bi, k], p, 0.0) / (1.0 - p_drop)
                dV[bi, :, sl] = pd.T @ dC[bi, :, sl]
                dP = np.where(keep[bi, k], dC[bi, :, sl] @ Vv[bi, :, sl].T, 0.0) / (1.0 - p_drop)
            dS = p * (dP - (dP * p).sum(axis=-1, keepdims=True))
            dQ[bi, :, sl] = (dS @ K[bi, :, sl]) * scale
            dK[bi, :, sl] = (dS.T @ Q[bi, :, sl]) * scale
    return dQ, dK, dV


# --------------------------------------------------------------------------- cross entropy
def cross_entropy_fwd(L, tgt, w):
    """Per-token cross entropy log sum_j exp(L_tj) - L_t,tgt and its weighted mean.

    L: [T, V], tgt: [T] int, w: [T] in {0,1}.  Returns (loss, ce[T], rowmax[T], sumexp[T])."""
    T = L.shape[0]
    mx = L.max(axis=-1)
    se = np.exp(L - mx[:, None]).sum(axis=-1)
    ce = np.log(se) + mx - L[np.arange(T), tgt]
    loss = float((w * ce).sum() / w.sum())
    return loss, ce, mx, se


def cross_entropy_bwd(L, tgt, w, mx, se):
    """d loss / d L = w_t / sum(w) * (softmax(L) - onehot(tgt))."""
    T = L.shape[0]
    dL = np.exp(L - mx[:, None]) / se[:, None]
    dL[np.arange(T), tgt] -= 1.0
    dL *= (w / w.sum())[:, None]
    return dL


# --------------------------------------------------------------------------- dropout (masks are INPUTS)
def apply_keep(x, keep, p_drop: float):
    """Inverted dropout with a given boolean keep mask: keep * x / (1 - p_drop); identity if keep is None.

    The same function is its own gradient map (d out = keep * d in / (1 - p_drop))."""
    if keep is None:
        return x
    return np.where(np.asarray(keep, bool).reshape(x.shape), x, 0.0) / (1.0 - p_drop)


def _drop_of(inp):
    """(keep_attn [b,h,s,s], keep1 [T,H], keep2 [T,H], p_attn, p_hidden) from the optional ``drop`` entry of the
    inputs; all None / 0 when the layer runs dropout-free (the default)."""
    d = inp.get("drop")
    if d is None:
        return None, None, None, 0.0, 0.0
    return d.get("keep_attn"), d.get("keep1"), d.get("keep2"), float(d.get("p_attn", 0.0)), float(d.get("p_hidden", 0.0))


# --------------------------------------------------------------------------- unsharded layer
def _f64(P: Dict[str, np.ndarray]) -> Dict[str, np.ndarray]:
    return {k: (np.asarray(v, F64) if np.asarray(v).dtype.kind == "f" else np.asarray(v)) for k, v in P.items()
            if k != "drop"}


def forward(inp: Dict[str, np.ndarray], spec: Spec) -> Dict[str, np.ndarray]:
    """Unsharded pre-LN layer + output embedding + mean cross entropy; returns every intermediate.

    inp holds X [b,s,H], the parameters (g1,b1,Wq,Wk,Wv,bq,bk,bv,Wo,bo,g2,b2,A,a,B,c,gf,bf,E),
    tgt [b,s] int, w [b,s] loss weights in {0,1}, key_len [b]; optionally ``drop``: the dropout keep masks of the
    attention probabilities and of the two block outputs before their residual adds (Section 3 / Appendix B.2)."""
    p = _f64(inp)
    keep_attn, keep1, keep2, p_attn, p_hidden = _drop_of(inp)
    b, s, H, T = spec.b, spec.s, spec.H, spec.T
    X = p["X"].reshape(T, H)
    c: Dict[str, np.ndarray] = {}
    # attention block (Section 3: LN replicated, Q/K/V GEMMs, heads, output projection, residual)
    c["U"], c["mu1"], c["rstd1"] = layernorm_fwd(X, p["g1"], p["b1"], spec.ln_eps)
    c["Q"] = c["U"] @ p["Wq"] + p["bq"]
    c["K"] = c["U"] @ p["Wk"] + p["bk"]
    c["Vv"] = c["U"] @ p["Wv"] + p["bv"]
    C, Pm, LSE = attention_fwd(c["Q"].reshape(b, s, H), c["K"].reshape(b, s, H),
                               c["Vv"].reshape(b, s, H), spec, p["key_len"], keep_attn, p_attn)
    c["C"], c["P"], c["LSE"] = C.reshape(T, H), Pm, LSE
    c["X1"] = X + apply_keep(c["C"] @ p["Wo"] + p["bo"], keep1, p_hidden)
    # MLP block (Section 3, Eq. 1: Y = GeLU(X A); then Z = Y B, residual)
    c["U2"], c["mu2"], c["rstd2"] = layernorm_fwd(c["X1"], p["g2"], p["b2"], spec.ln_eps)
    c["G"] = c["U2"] @ p["A"] + p["a"]
    c["Y"] = gelu(c["G"], spec.gelu_tanh)
    c["X2"] = c["X1"] + apply_keep(c["Y"] @ p["B"] + p["c"], keep2, p_hidden)
    # final LN (switch) and the output embedding fused with the loss (Section 3)
    if spec.final_ln:
        c["Hf"], c["muf"], c["rstdf"] = layernorm_fwd(c["X2"], p["gf"], p["bf"], spec.ln_eps)
    else:
        c["Hf"] = c["X2"]
    c["L"] = c["Hf"] @ p["E"]
    tgt = p["tgt"].reshape(T).astype(np.int64)
    w = np.asarray(p["w"], F64).reshape(T)
    c["loss"], c["ce"], c["M"], c["S"] = cross_entropy_fwd(c["L"], tgt, w)
    return c


def backward(inp: Dict[str, np.ndarray], c: Dict[str, np.ndarray], spec: Spec) -> Dict[str, np.ndarray]:
    """Analytic gradients of ``loss`` w.r.t. X and every parameter, plus the intermediate gradients."""
    p = _f64(inp)
    b, s, H, T = spec.b, spec.s, spec.H, spec.T
    X = p["X"].reshape(T, H)
    tgt = p["tgt"].reshape(T).astype(np.int64)
    w = np.asarray(p["w"], F64).reshape(T)
    keep_attn, keep1, keep2, p_attn, p_hidden = _drop_of(inp)
    g: Dict[str, np.ndarray] = {}
    g["dL"] = cross_entropy_bwd(c["L"], tgt, w, c["M"], c["S"])
    g["dE"] = c["Hf"].T @ g["dL"]
    g["dHf"] = g["dL"] @ p["E"].T
    if spec.final_ln:
        g["dX2"], g["dgf"], g["dbf"] = layernorm_bwd(g["dHf"], c["X2"], p["gf"], c["muf"], c["rstdf"])
    else:
        g["dX2"] = g["dHf"]
        g["dgf"] = np.zeros(H, F64)
        g["dbf"] = np.zeros(H, F64)
    # MLP block
    g["dZ2"] = apply_keep(g["dX2"], keep2, p_hidden)       # gradient of the MLP block output before dropout
    g["dc"] = g["dZ2"].sum(axis=0)
    g["dB"] = c["Y"].T @ g["dZ2"]
    g["dY"] = g["dZ2"] @ p["B"].T
    g["dG"] = g["dY"] * gelu_grad(c["G"], spec.gelu_tanh)
    g["da"] = g["dG"].sum(axis=0)
    g["dA"] = c["U2"].T @ g["dG"]
    g["dU2"] = g["dG"] @ p["A"].T
    dx1_ln, g["dg2"], g["db2"] = layernorm_bwd(g["dU2"], c["X1"], p["g2"], c["mu2"], c["rstd2"])
    g["dX1"] = g["dX2"] + dx1_ln
    # attention block
    g["dZ1"] = apply_keep(g["dX1"], keep1, p_hidden)
    g["dbo"] = g["dZ1"].sum(axis=0)
    g["dWo"] = c["C"].T @ g["dZ1"]
    g["dC"] = g["dZ1"] @ p["Wo"].T
    dQ, dK, dV = attention_bwd(g["dC"].reshape(b, s, H), c["Q"].reshape(b, s, H), c["K"].reshape(b, s, H),
                               c["Vv"].reshape(b, s, H), c["P"], spec, keep_attn, p_attn)
    g["dQ"], g["dK"], g["dVv"] = dQ.reshape(T, H), dK.reshape(T, H), dV.reshape(T, H)
    g["dWq"], g["dWk"], g["dWv"] = c["U"].T @ g["dQ"], c["U"].T @ g["dK"], c["U"].T @ g["dVv"]
    g["dbq"], g["dbk"], g["dbv"] = g["dQ"].sum(axis=0), g["dK"].sum(axis=0), g["dVv"].sum(axis=0)
    g["dU"] = g["dQ"] @ p["Wq"].T + g["dK"] @ p["Wk"].T + g["dVv"] @ p["Wv"].T
    dx_ln, g["dg1"], g["db1"] = layernorm_bwd(g["dU"], X, p["g1"], c["mu1"], c["rstd1"])
    g["dX"] = g["dX1"] + dx_ln
    return g


# --------------------------------------------------------------------------- the original (post-LN) arrangement
def forward_post_ln(inp: Dict[str, np.ndarray], spec: Spec) -> Dict[str, np.ndarray]:
    """The layer in the ORIGINAL BERT arrangement that the paper compares against (Section 5.3, architecture (a) of
    its layer-norm figure): layer norm AFTER each residual add, X1 = LN(X + Attn(X)), X2 = LN(X1 + MLP(X1)); the
    logits are taken from X2 directly.  Reading (the figure itself is not in the text): g1/b1 normalise the attention
    block's sum, g2/b2 the MLP block's; gf/bf are unused.  No dropout here."""
    p = _f64(inp)
    b, s, H, T = spec.b, spec.s, spec.H, spec.T
    X = p["X"].reshape(T, H)
    c: Dict[str, np.ndarray] = {}
    c["Q"], c["K"], c["Vv"] = X @ p["Wq"] + p["bq"], X @ p["Wk"] + p["bk"], X @ p["Wv"] + p["bv"]
    C, Pm, LSE = attention_fwd(c["Q"].reshape(b, s, H), c["K"].reshape(b, s, H), c["Vv"].reshape(b, s, H), spec,
                               p["key_len"])
    c["C"], c["P"], c["LSE"] = C.reshape(T, H), Pm, LSE
    c["S1"] = X + c["C"] @ p["Wo"] + p["bo"]
    c["X1"], c["mu1"], c["rstd1"] = layernorm_fwd(c["S1"], p["g1"], p["b1"], spec.ln_eps)
    c["G"] = c["X1"] @ p["A"] + p["a"]
    c["Y"] = gelu(c["G"], spec.gelu_tanh)
    c["S2"] = c["X1"] + c["Y"] @ p["B"] + p["c"]
    c["X2"], c["mu2"], c["rstd2"] = layernorm_fwd(c["S2"], p["g2"], p["b2"], spec.ln_eps)
    c["L"] = c["X2"] @ p["E"]
    tgt = p["tgt"].reshape(T).astype(np.int64)
    w = np.asarray(p["w"], F64).reshape(T)
    c["loss"], c["ce"], c["M"], c["S"] = cross_entropy_fwd(c["L"], tgt, w)
    return c


def backward_post_ln(inp: Dict[str, np.ndarray], c: Dict[str, np.ndarray], spec: Spec) -> Dict[str, np.ndarray]:
    """Analytic gradients of forward_post_ln."""
    p = _f64(inp)
    b, s, H, T = spec.b, spec.s, spec.H, spec.T
    X = p["X"].reshape(T, H)
    tgt = p["tgt"].reshape(T).astype(np.int64)
    w = np.asarray(p["w"], F64).reshape(T)
    g: Dict[str, np.ndarray] = {}
    g["dL"] = cross_entropy_bwd(c["L"], tgt, w, c["M"], c["S"])
    g["dE"] = c["X2"].T @ g["dL"]
    g["dX2"] = g["dL"] @ p["E"].T
    g["dS2"], g["dg2"], g["db2"] = layernorm_bwd(g["dX2"], c["S2"], p["g2"], c["mu2"], c["rstd2"])
    g["dc"] = g["dS2"].sum(axis=0)
    g["dB"] = c["Y"].T @ g["dS2"]
    g["dG"] = (g["dS2"] @ p["B"].T) * gelu_grad(c["G"], spec.gelu_tanh)
    g["da"] = g["dG"].sum(axis=0)
    g["dA"] = c["X1"].T @ g["dG"]
    g["dX1"] = g["dS2"] + g["dG"] @ p["A"].T                 # residual branch + through the MLP
    g["dS1"], g["dg1"], g["db1"] = layernorm_bwd(g["dX1"], c["S1"], p["g1"], c["mu1"], c["rstd1"])
    g["dbo"] = g["dS1"].sum(axis=0)
    g["dWo"] = c["C"].T @ g["dS1"]
    dC = g["dS1"] @ p["Wo"].T
    dQ, dK, dV = attention_bwd(dC.reshape(b, s, H), c["Q"].reshape(b, s, H), c["K"].reshape(b, s, H),
                               c["Vv"].reshape(b, s, H), c["P"], spec)
    dQ, dK, dV = dQ.reshape(T, H), dK.reshape(T, H), dV.reshape(T, H)
    g["dWq"], g["dWk"], g["dWv"] = X.T @ dQ, X.T @ dK, X.T @ dV
    g["dbq"], g["dbk"], g["dbv"] = dQ.sum(axis=0), dK.sum(axis=0), dV.sum(axis=0)
    g["dX"] = g["dS1"] + dQ @ p["Wq"].T + dK @ p["Wk"].T + dV @ p["Wv"].T
    return g


def loss_only(inp: Dict[str, np.ndarray], spec: Spec) -> float:
    return forward(inp, spec)["loss"]


# --------------------------------------------------------------------------- sharded formulation
def shard_range(n: int, p: int, r: int) -> Tuple[int, int]:
    """Contiguous range of shard r of p over n items (n divisible by p, as in Table 1)."""
    if p <= 0 or not (0 <= r < p) or n % p != 0:
        raise ValueError("bad shard request")
    q = n // p
    return r * q, (r + 1) * q


def shard_params(inp: Dict[str, np.ndarray], spec: Spec, p: int, r: int) -> Dict[str, np.ndarray]:
    """Shard r's parameters by index slicing only (Section 3).

    Column-parallel: Q/K/V columns of the local heads, concatenated [Q | K | V]; A columns.
    Row-parallel: Wo rows of the local heads; B rows.  Vocabulary-parallel: E columns."""
    q = _f64(inp)
    c0, c1 = shard_range(spec.H, p, r)       # local heads' columns (h/p heads of d columns each)
    f0, f1 = shard_range(spec.F, p, r)
    v0, v1 = shard_range(spec.V, p, r)
    if spec.h % p != 0:
        raise ValueError("heads not divisible by p")
    return {
        "Wqkv": np.concatenate([q["Wq"][:, c0:c1], q["Wk"][:, c0:c1], q["Wv"][:, c0:c1]], axis=1),
        "bqkv": np.concatenate([q["bq"][c0:c1], q["bk"][c0:c1], q["bv"][c0:c1]]),
        "Wo": q["Wo"][c0:c1, :],
        "A": q["A"][:, f0:f1], "a": q["a"][f0:f1], "B": q["B"][f0:f1, :],
        "E": q["E"][:, v0:v1],
        "cols": (c0, c1), "ffn": (f0, f1), "vocab": (v0, v1),
    }


def sharded_reference(inp: Dict[str, np.ndarray], spec: Spec, p: int) -> Dict[str, object]:
    """The sharded method written out in fp64: per-shard partials and explicit reductions.

    Follows Section 3 step by step: replicated LN; per shard r the column-parallel QKV GEMM,
    local-head attention, row-parallel projection giving a partial sum; the reduction `g`
    (here: a plain sum over r) followed by bias (once) and residual; the same for the MLP
    (Y_r = GeLU(U2 A_r + a_r), partial Y_r B_r); vocabulary-parallel logits L_r = Hf E_r with
    per-row partials (m_r, s_r, t_r) merged into the loss; and the mirror-image backward where
    `f` sums the per-shard input gradients.  Returns combined tensors under their unsharded
    names and a list ``shards`` of per-shard dictionaries."""
    q = _f64(inp)
    b, s, H, T, d = spec.b, spec.s, spec.H, spec.T, spec.d
    hl = spec.h // p
    Hl = H // p
    lspec = Spec(b=b, s=s, H=Hl, h=hl, F=spec.F // p, V=spec.V // p, causal=spec.causal,
                 final_ln=spec.final_ln, gelu_tanh=spec.gelu_tanh, ln_eps=spec.ln_eps)
    X = q["X"].reshape(T, H)
    tgt = q["tgt"].reshape(T).astype(np.int64)
    w = np.asarray(q["w"], F64).reshape(T)
    sh = [shard_params(inp, spec, p, r) for r in range(p)]
    keep_attn, keep1, keep2, p_attn, p_hidden = _drop_of(inp)
    ka = lambda r: None if keep_attn is None else keep_attn[:, r * hl:(r + 1) * hl]   # local heads' masks
    out: Dict[str, object] = {}
    # ---- forward
    U, mu1, rstd1 = layernorm_fwd(X, q["g1"], q["b1"], spec.ln_eps)
    for r in range(p):
        S = sh[r]
        S["qkv"] = U @ S["Wqkv"] + S["bqkv"]
        Qr, Kr, Vr = S["qkv"][:, :Hl], S["qkv"][:, Hl:2 * Hl], S["qkv"][:, 2 * Hl:]
        C, Pm, LSE = attention_fwd(Qr.reshape(b, s, Hl), Kr.reshape(b, s, Hl), Vr.reshape(b, s, Hl),
                                   lspec, q["key_len"], ka(r), p_attn)
        S["ctx"], S["P"], S["lse"] = C.reshape(T, Hl), Pm, LSE
        S["attn_partial"] = S["ctx"] @ S["Wo"]
    # g: all-reduce, then (replicated) bias once, dropout, residual
    X1 = X + apply_keep(q["bo"] + sum(S["attn_partial"] for S in sh), keep1, p_hidden)
    U2, mu2, rstd2 = layernorm_fwd(X1, q["g2"], q["b2"], spec.ln_eps)
    for r in range(p):
        S = sh[r]
        S["g"] = U2 @ S["A"] + S["a"]
        S["y"] = gelu(S["g"], spec.gelu_tanh)
        S["mlp_partial"] = S["y"] @ S["B"]
    X2 = X1 + apply_keep(q["c"] + sum(S["mlp_partial"] for S in sh), keep2, p_hidden)
    if spec.final_ln:
        Hf, muf, rstdf = layernorm_fwd(X2, q["gf"], q["bf"], spec.ln_eps)
    else:
        Hf = X2
    for r in range(p):
        S = sh[r]
        v0, v1 = S["vocab"]
        S["logits"] = Hf @ S["E"]
        S["m"] = S["logits"].max(axis=-1)
        S["s"] = np.exp(S["logits"] - S["m"][:, None]).sum(axis=-1)
        inside = (tgt >= v0) & (tgt < v1)                           # integer test, exact
        loc = np.where(inside, tgt - v0, 0)
        S["t"] = np.where(inside, S["logits"][np.arange(T), loc], 0.0)
        S["tgt_inside"], S["tgt_local"] = inside, loc
    M = np.max(np.stack([S["m"] for S in sh]), axis=0)              # the b x s scalars that are communicated
    Ssum = sum(S["s"] * np.exp(S["m"] - M) for S in sh)
    tsum = sum(S["t"] for S in sh)
    ce = np.log(Ssum) + M - tsum
    loss = float((w * ce).sum() / w.sum())
    # ---- backward
    coef = w / w.sum()
    for r in range(p):
        S = sh[r]
        dL = np.exp(S["logits"] - M[:, None]) / Ssum[:, None]
        dL[np.arange(T)[S["tgt_inside"]], S["tgt_local"][S["tgt_inside"]]] -= 1.0
        S["dlogits"] = dL * coef[:, None]
        S["dE"] = Hf.T @ S["dlogits"]
        S["dhf_partial"] = S["dlogits"] @ S["E"].T
    dHf = sum(S["dhf_partial"] for S in sh)                          # f: all-reduce of the input gradient
    if spec.final_ln:
        dX2, dgf, dbf = layernorm_bwd(dHf, X2, q["gf"], muf, rstdf)
    else:
        dX2, dgf, dbf = dHf, np.zeros(H), np.zeros(H)
    dZ2 = apply_keep(dX2, keep2, p_hidden)
    dc = dZ2.sum(axis=0)
    for r in range(p):
        S = sh[r]
        S["dB"] = S["y"].T @ dZ2
        S["dy"] = dZ2 @ S["B"].T
        S["dg"] = S["dy"] * gelu_grad(S["g"], spec.gelu_tanh)
        S["da"] = S["dg"].sum(axis=0)
        S["dA"] = U2.T @ S["dg"]
        S["du2_partial"] = S["dg"] @ S["A"].T
    dU2 = sum(S["du2_partial"] for S in sh)
    dx1_ln, dg2, db2 = layernorm_bwd(dU2, X1, q["g2"], mu2, rstd2)
    dX1 = dX2 + dx1_ln
    dZ1 = apply_keep(dX1, keep1, p_hidden)
    dbo = dZ1.sum(axis=0)
    for r in range(p):
        S = sh[r]
        S["dWo"] = S["ctx"].T @ dZ1
        S["dctx"] = dZ1 @ S["Wo"].T
        Qr, Kr, Vr = S["qkv"][:, :Hl], S["qkv"][:, Hl:2 * Hl], S["qkv"][:, 2 * Hl:]
        dQ, dK, dV = attention_bwd(S["dctx"].reshape(b, s, Hl), Qr.reshape(b, s, Hl), Kr.reshape(b, s, Hl),
                                   Vr.reshape(b, s, Hl), S["P"], lspec, ka(r), p_attn)
        S["dqkv"] = np.concatenate([dQ.reshape(T, Hl), dK.reshape(T, Hl), dV.reshape(T, Hl)], axis=1)
        S["dWqkv"] = U.T @ S["dqkv"]
        S["dbqkv"] = S["dqkv"].sum(axis=0)
        S["du_partial"] = S["dqkv"] @ S["Wqkv"].T
    dU = sum(S["du_partial"] for S in sh)
    dx_ln, dg1, db1 = layernorm_bwd(dU, X, q["g1"], mu1, rstd1)
    dX = dX1 + dx_ln
    out.update(U=U, mu1=mu1, rstd1=rstd1, X1=X1, U2=U2, mu2=mu2, rstd2=rstd2, X2=X2, Hf=Hf,
               M=M, S=Ssum, tsum=tsum, ce=ce, loss=loss, dHf=dHf, dX2=dX2, dgf=dgf, dbf=dbf, dc=dc,
               dU2=dU2, dg2=dg2, db2=db2, dX1=dX1, dZ1=dZ1, dZ2=dZ2, dbo=dbo, dU=dU, dg1=dg1, db1=db1, dX=dX, shards=sh)
    if spec.final_ln:
        out.update(muf=muf, rstdf=rstdf)
    return out


# --------------------------------------------------------------------------- FLOP convention used for reporting
def model_flops(spec: Spec, p: int = 1, causal_algorithmic: bool = True) -> Dict[str, float]:
    """Model FLOPs of one shard's fwd+bwd: GEMM = 2 M K N, backward = 2 x forward,
    attention forward = two s x d x s matmuls per head (halved for causal when
    ``causal_algorithmic``), backward = four.  Recomputation is not counted."""
    T, H, d = spec.T, spec.H, spec.d
    hl, Fl, Vl = spec.h // p, spec.F // p, spec.V // p
    Hl = hl * d
    gemm = lambda M, K, N: 2.0 * M * K * N
    qkv = gemm(T, H, 3 * Hl)
    proj = gemm(T, Hl, H)
    fc1 = gemm(T, H, Fl)
    fc2 = gemm(T, Fl, H)
    logits = gemm(T, H, Vl)
    att = 2.0 * (2.0 * spec.b * hl * spec.s * spec.s * d)
    if spec.causal and causal_algorithmic:
        att *= 0.5
    layer_fwd = qkv + proj + fc1 + fc2 + att
    return {"qkv": qkv, "proj": proj, "fc1": fc1, "fc2": fc2, "attn": att, "logits": logits,
            "layer_fwd": layer_fwd, "fwd": layer_fwd + logits, "fwd_bwd": 3.0 * (layer_fwd + logits),
            "layer_fwd_bwd": 3.0 * layer_fwd}
