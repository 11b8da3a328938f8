"""Seeded synthetic inputs for the tensor-parallel transformer-layer shard path.

This module holds NONE of the method's arithmetic: it only names the workload
shapes (Table 1 and Table 4 of the paper: hidden size, heads, head dim 96 / 64,
padded vocabulary 51,200 / 30,592, batch 8, sequence 1024 / 512) and draws
seeded random tensors with the paper's initial-weight distribution
(Section 4.2: normal, std 0.02).  Both the CPU oracle's tests and the HIP
path's tests/bench consume these arrays; neither side's code lives here.

Draw order is fixed (X, LN params, attention weights, MLP weights, final LN,
E, targets, key lengths, loss mask) so that one seed always means one input.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, List, Optional

import numpy as np


@dataclass(frozen=True)
class LayerConfig:
    """Global (unsharded) dimensions plus the shard count the config is quoted on."""
    name: str
    b: int          # batch
    s: int          # sequence length
    H: int          # hidden size
    h: int          # attention heads (global)
    F: int          # FFN width (4H, pinned by the parameter counts of Tables 1 and 4)
    V: int          # (padded) vocabulary
    p: int          # model-parallel shards
    causal: bool    # GPT-2 style (True) or BERT style bidirectional with key padding (False)
    dtype: str      # "fp32" or "bf16" (bf16 storage, fp32 accumulation)
    final_ln: bool = True
    gelu_tanh: bool = True
    ln_eps: float = 1e-5
    seed: int = 0
    masked_lm: bool = False   # BERT: loss on a seeded 15 % of valid positions, per-row key lengths

    @property
    def T(self) -> int:
        return self.b * self.s

    @property
    def d(self) -> int:
        return self.H // self.h


# The five workloads the build is quoted on (shapes from Table 1 / Table 4 of the paper).
CONFIGS: Dict[str, LayerConfig] = {
    "tiny": LayerConfig("tiny", b=2, s=128, H=256, h=4, F=1024, V=1024, p=2,
                        causal=True, dtype="fp32", seed=0),
    "gpt2_1p2b": LayerConfig("gpt2_1p2b", b=8, s=1024, H=1536, h=16, F=6144, V=51200, p=1,
                             causal=True, dtype="bf16", seed=1),
    "gpt2_2p5b": LayerConfig("gpt2_2p5b", b=8, s=1024, H=1920, h=20, F=7680, V=51200, p=2,
                             causal=True, dtype="bf16", seed=2),
    "gpt2_8p3b": LayerConfig("gpt2_8p3b", b=8, s=1024, H=3072, h=32, F=12288, V=51200, p=8,
                             causal=True, dtype="bf16", seed=3),
    "bert_3p9b": LayerConfig("bert_3p9b", b=8, s=512, H=2560, h=40, F=10240, V=30592, p=4,
                             causal=False, dtype="bf16", seed=4, masked_lm=True),
}


def _variant(base: str, name: str, **kw) -> LayerConfig:
    return replace(CONFIGS[base], name=name, **kw)


# Shape sweeps of the paper's scaling studies, as single-GPU shard workloads:
#  * "heads": the 8.3B configuration, 8-way model parallel, with 16 / 24 / 32 attention heads (Table 7): head sizes
#    192 / 128 / 96, i.e. 2 / 3 / 4 local heads per GPU;
#  * "strong_1p2b": the 1.2B configuration split 1 / 2 / 4 / 8 ways at fixed batch 8 (Table 8): the per-GPU share of
#    the work shrinks with p;
#  * "table1": the four weak-scaling rows of Table 1 (1.2B on 1 GPU ... 8.3B on 8 GPUs): the per-GPU share stays about
#    constant.
SWEEPS: Dict[str, List[LayerConfig]] = {
    "heads": [_variant("gpt2_8p3b", "gpt2_8p3b_h16", h=16), _variant("gpt2_8p3b", "gpt2_8p3b_h24", h=24),
              CONFIGS["gpt2_8p3b"]],
    "strong_1p2b": [CONFIGS["gpt2_1p2b"]] + [_variant("gpt2_1p2b", f"gpt2_1p2b_p{p}", p=p) for p in (2, 4, 8)],
    "table1": [CONFIGS["gpt2_1p2b"], CONFIGS["gpt2_2p5b"],
               _variant("gpt2_8p3b", "gpt2_4p2b", H=2304, h=24, F=9216, p=4, seed=5), CONFIGS["gpt2_8p3b"]],
}
SWEEP_CONFIGS: Dict[str, LayerConfig] = {c.name: c for cs in SWEEPS.values() for c in cs}


def small_config(name: str = "small", **kw) -> LayerConfig:
    """A test-sized config; any field can be overridden."""
    base = dict(b=2, s=32, H=64, h=4, F=256, V=128, p=2, causal=True, dtype="fp32", seed=11)
    base.update(kw)
    return LayerConfig(name, **base)


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round an fp32 array to the nearest bf16 value (ties to even), returned as fp32.

    Storage-format conversion only (no NaN/Inf handling needed: inputs are finite)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """The uint16 bit patterns of an fp32 array whose values are already bf16-representable."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


PARAM_ORDER = ("g1", "b1", "Wq", "Wk", "Wv", "bq", "bk", "bv", "Wo", "bo",
               "g2", "b2", "A", "a", "B", "c", "gf", "bf", "E")


def make_inputs(cfg: LayerConfig, *, nonzero_bias: bool = False, random_ln: bool = False,
                seed: Optional[int] = None) -> Dict[str, np.ndarray]:
    """Draw one full set of unsharded inputs for `cfg` as fp32 numpy arrays.

    Weights ~ N(0, std 0.02); X ~ N(0,1); biases 0 (or N(0,0.02) with nonzero_bias);
    LN gamma 1 / beta 0 (or gamma 1+N(0,0.1), beta N(0,0.1) with random_ln);
    targets uniform over the padded vocabulary; BERT-style configs also get
    per-sequence key lengths uniform in [s/2, s] and a 15 % loss mask over valid
    positions (at least one position kept).  For bf16 configs every floating array
    is rounded once to bf16 here, so both consumers read identical values.
    """
    rng = np.random.default_rng(cfg.seed if seed is None else seed)
    H, F, V, T = cfg.H, cfg.F, cfg.V, cfg.T
    f32 = np.float32

    def normal(shape, std):
        return (rng.standard_normal(shape, dtype=f32) * f32(std)).astype(f32)

    def bias(n):
        return normal((n,), 0.02) if nonzero_bias else np.zeros((n,), f32)

    def ln():
        if random_ln:
            return (1.0 + normal((H,), 0.1)).astype(f32), normal((H,), 0.1)
        return np.ones((H,), f32), np.zeros((H,), f32)

    out: Dict[str, np.ndarray] = {}
    out["X"] = normal((cfg.b, cfg.s, H), 1.0)
    out["g1"], out["b1"] = ln()
    out["Wq"] = normal((H, H), 0.02)
    out["Wk"] = normal((H, H), 0.02)
    out["Wv"] = normal((H, H), 0.02)
    out["bq"], out["bk"], out["bv"] = bias(H), bias(H), bias(H)
    out["Wo"] = normal((H, H), 0.02)
    out["bo"] = bias(H)
    out["g2"], out["b2"] = ln()
    out["A"] = normal((H, F), 0.02)
    out["a"] = bias(F)
    out["B"] = normal((F, H), 0.02)
    out["c"] = bias(H)
    out["gf"], out["bf"] = ln()
    out["E"] = normal((H, V), 0.02)
    out["tgt"] = rng.integers(0, V, size=(cfg.b, cfg.s), dtype=np.int64).astype(np.int32)
    if cfg.masked_lm:
        lo = max(1, cfg.s // 2)
        out["key_len"] = rng.integers(lo, cfg.s + 1, size=(cfg.b,), dtype=np.int64).astype(np.int32)
        valid = np.arange(cfg.s)[None, :] < out["key_len"][:, None]
        w = (rng.random((cfg.b, cfg.s)) < 0.15) & valid
        if not w.any():
            w[0, 0] = True
        out["w"] = w.astype(f32)
    else:
        out["key_len"] = np.full((cfg.b,), cfg.s, np.int32)
        out["w"] = np.ones((cfg.b, cfg.s), f32)
    if cfg.dtype == "bf16":
        for k, v in out.items():
            if v.dtype == np.float32 and k != "w":
                out[k] = round_to_bf16(v)
    return out


def with_batch(cfg: LayerConfig, b: int) -> LayerConfig:
    return replace(cfg, b=b, name=f"{cfg.name}_b{b}")
