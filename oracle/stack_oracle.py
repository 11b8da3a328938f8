"""fp64 CPU oracle of an N-layer stack: token + position embedding, N pre-LN transformer layers, final layer norm,
output embedding tied to the input embedding, mean cross entropy -- the model whose per-GPU share the paper trains
with activation checkpointing after every layer (Section 4.2).

TEST INFRASTRUCTURE ONLY (see oracle/layer_oracle.py): only tests/, the smoke test and the benchmark's cpu_baseline leg
may import it; it shares no code with the HIP path.

Every step is the definition already written out (and pinned) in oracle/layer_oracle.py and
oracle/rng_embed_oracle.py; this file only chains them: layer l's output is layer l+1's input, the gradient flows
back the same way, and the embedding matrix collects two gradients (input lookup and output GEMM).  Activation
checkpointing changes what is stored, not what is computed, so it has no counterpart here.
Pins (tests/test_stack_pins.py): a one-layer stack equals the single-layer oracle exactly; library autograd and
finite differences on a two-layer stack.
"""
from __future__ import annotations

from typing import Dict, List, Optional

import numpy as np

from . import layer_oracle as O
from . import rng_embed_oracle as R

F64 = np.float64
LAYER_PARAMS = ("g1", "b1", "Wq", "Wk", "Wv", "bq", "bk", "bv", "Wo", "bo", "g2", "b2", "A", "a", "B", "c")


def layer_fwd(p: Dict[str, np.ndarray], X: np.ndarray, spec: O.Spec, key_len, drop=None) -> Dict[str, np.ndarray]:
    """One pre-LN layer (Section 2.2 / Section 3): X [T, H] -> X2 [T, H]; returns every intermediate."""
    b, s, H, T = spec.b, spec.s, spec.H, spec.T
    keep_attn, keep1, keep2, p_attn, p_hidden = O._drop_of({"drop": drop})
    c: Dict[str, np.ndarray] = {"X": X}
    c["U"], c["mu1"], c["rstd1"] = O.layernorm_fwd(X, p["g1"], p["b1"], spec.ln_eps)
    c["Q"] = c["U"] @ p["Wq"] + p["bq"]
    c["K"] = c["U"] @ p["Wk"] + p["bk"]
    c["Vv"] = c["U"] @ p["Wv"] + p["bv"]
    C, Pm, _ = O.attention_fwd(c["Q"].reshape(b, s, H), c["K"].reshape(b, s, H), c["Vv"].reshape(b, s, H), spec,
                               key_len, keep_attn, p_attn)
    c["C"], c["P"] = C.reshape(T, H), Pm
    c["X1"] = X + O.apply_keep(c["C"] @ p["Wo"] + p["bo"], keep1, p_hidden)
    c["U2"], c["mu2"], c["rstd2"] = O.layernorm_fwd(c["X1"], p["g2"], p["b2"], spec.ln_eps)
    c["G"] = c["U2"] @ p["A"] + p["a"]
    c["Y"] = O.gelu(c["G"], spec.gelu_tanh)
    c["X2"] = c["X1"] + O.apply_keep(c["Y"] @ p["B"] + p["c"], keep2, p_hidden)
    return c


def layer_bwd(p: Dict[str, np.ndarray], c: Dict[str, np.ndarray], dX2: np.ndarray, spec: O.Spec, drop=None):
    """Gradients of one layer given the gradient of its output; returns (dX, parameter gradients)."""
    b, s, H, T = spec.b, spec.s, spec.H, spec.T
    keep_attn, keep1, keep2, p_attn, p_hidden = O._drop_of({"drop": drop})
    g: Dict[str, np.ndarray] = {}
    dZ2 = O.apply_keep(dX2, keep2, p_hidden)
    g["c"] = dZ2.sum(axis=0)
    g["B"] = c["Y"].T @ dZ2
    dG = (dZ2 @ p["B"].T) * O.gelu_grad(c["G"], spec.gelu_tanh)
    g["a"] = dG.sum(axis=0)
    g["A"] = c["U2"].T @ dG
    dx1_ln, g["g2"], g["b2"] = O.layernorm_bwd(dG @ p["A"].T, c["X1"], p["g2"], c["mu2"], c["rstd2"])
    dX1 = dX2 + dx1_ln
    dZ1 = O.apply_keep(dX1, keep1, p_hidden)
    g["bo"] = dZ1.sum(axis=0)
    g["Wo"] = c["C"].T @ dZ1
    dC = dZ1 @ p["Wo"].T
    dQ, dK, dV = O.attention_bwd(dC.reshape(b, s, H), c["Q"].reshape(b, s, H), c["K"].reshape(b, s, H),
                                 c["Vv"].reshape(b, s, H), c["P"], spec, keep_attn, p_attn)
    dQ, dK, dV = dQ.reshape(T, H), dK.reshape(T, H), dV.reshape(T, H)
    g["Wq"], g["Wk"], g["Wv"] = c["U"].T @ dQ, c["U"].T @ dK, c["U"].T @ dV
    g["bq"], g["bk"], g["bv"] = dQ.sum(axis=0), dK.sum(axis=0), dV.sum(axis=0)
    dU = dQ @ p["Wq"].T + dK @ p["Wk"].T + dV @ p["Wv"].T
    dx_ln, g["g1"], g["b1"] = O.layernorm_bwd(dU, c["X"], p["g1"], c["mu1"], c["rstd1"])
    return dX1 + dx_ln, g


def _f64(d):
    return {k: (np.asarray(v, F64) if np.asarray(v).dtype.kind == "f" else np.asarray(v)) for k, v in d.items()}


def forward(model: Dict[str, object], spec: O.Spec) -> Dict[str, object]:
    """model: {"layers": [per-layer parameter dicts], "E" [H, V], "pos" [s, H], "gf", "bf", "ids" [b, s], "tgt" [b, s],
    "w" [b, s], "key_len" [b], optional "drop": {"layers": [layer drop dicts], "keep0", "p_hidden"}}."""
    m = {k: v for k, v in model.items() if k not in ("layers", "drop")}
    m = _f64(m)
    layers = [_f64(L) for L in model["layers"]]
    drop = model.get("drop")
    T = spec.T
    keep0 = drop["keep0"] if drop else None
    p0 = float(drop["p_hidden"]) if drop else 0.0
    out: Dict[str, object] = {"layer_caches": []}
    X = R.embedding_fwd(m["E"], m["ids"], m["pos"], keep0, p0)
    out["X0"] = X
    for l, P in enumerate(layers):
        c = layer_fwd(P, X, spec, m["key_len"], drop["layers"][l] if drop else None)
        out["layer_caches"].append(c)
        X = c["X2"]
    out["XL"] = X
    out["Hf"], out["muf"], out["rstdf"] = O.layernorm_fwd(X, m["gf"], m["bf"], spec.ln_eps)
    out["L"] = out["Hf"] @ m["E"]
    tgt = m["tgt"].reshape(T).astype(np.int64)
    w = np.asarray(m["w"], F64).reshape(T)
    out["loss"], out["ce"], out["M"], out["S"] = O.cross_entropy_fwd(out["L"], tgt, w)
    return out


def backward(model: Dict[str, object], fw: Dict[str, object], spec: O.Spec) -> Dict[str, object]:
    m = _f64({k: v for k, v in model.items() if k not in ("layers", "drop")})
    layers = [_f64(L) for L in model["layers"]]
    drop = model.get("drop")
    T = spec.T
    tgt = m["tgt"].reshape(T).astype(np.int64)
    w = np.asarray(m["w"], F64).reshape(T)
    g: Dict[str, object] = {}
    dL = O.cross_entropy_bwd(fw["L"], tgt, w, fw["M"], fw["S"])
    dE_out = fw["Hf"].T @ dL
    dX, g["gf"], g["bf"] = O.layernorm_bwd(dL @ m["E"].T, fw["XL"], m["gf"], fw["muf"], fw["rstdf"])
    g["layers"] = [None] * len(layers)
    g["dX_in"] = [None] * len(layers)
    for l in reversed(range(len(layers))):
        dX, g["layers"][l] = layer_bwd(layers[l], fw["layer_caches"][l], dX, spec, drop["layers"][l] if drop else None)
        g["dX_in"][l] = dX
    keep0 = drop["keep0"] if drop else None
    p0 = float(drop["p_hidden"]) if drop else 0.0
    dE_in, g["pos"] = R.embedding_bwd(dX, m["ids"], spec.V, spec.s, keep0, p0)
    g["E"] = dE_out + dE_in            # one parameter, two uses (Section 3: the embeddings share weights)
    g["E_out"], g["E_in"] = dE_out, dE_in
    return g


def loss_only(model, spec) -> float:
    return forward(model, spec)["loss"]
