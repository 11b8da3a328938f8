"""Sequencer of one model-parallel worker group's training step on one GPU: vocabulary-parallel input embedding,
N transformer layers, final layer norm, vocabulary-parallel loss, backward, optimizer (allocation and call order only;
all arithmetic is in the HIP library).

The paper trains with activation checkpointing after every transformer layer (Section 4.2): with ``checkpoint=True``
only the layer INPUTS are kept by the forward pass, all layers share one set of activation buffers, and the backward
pass re-runs layer l's forward calls from its saved input right before layer l's backward calls.  Dropout masks come
from the counter-based generator, so the recomputed forward reproduces them exactly (Appendix B.2 needs the same:
"identical dropout patterns").  The reductions g / f of Section 3 are the combine kernels fused into the layer norms:
the reduction that ends layer l's MLP block is fused with layer l+1's first layer norm (or the final one).
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

from . import binding as B
from .synth import LayerConfig

LAYER_REP = ("g1", "b1", "bo", "g2", "b2", "c")          # replicated per-layer parameters
LAYER_SHARD = ("Wqkv", "bqkv", "Wo", "A", "a", "B")      # per-shard per-layer parameters
SITES = {"attn": 1, "hidden1": 2, "hidden2": 3}


class ModelShards:
    def __init__(self, cfg: LayerConfig, n_layers: int, shards: Sequence[int], device: str = "cuda:0",
                 dropout: Optional[Dict[str, object]] = None, checkpoint: bool = True, grouped_wgrads: bool = True,
                 deferred_sums: bool = True):
        """dropout: None or {"p_attn", "p_hidden", "base_seed", "step"}; site offsets are derived as
        (step << 32) | (16 * layer + site) with the embedding site at layer index n_layers.
        grouped_wgrads: the layer backward computes input gradients only and each layer shard's four weight
        gradients come from one mlm_layer_shard_wgrads call (one grouped GEMM launch).
        deferred_sums: the finishing reductions of each layer's bias and layer-norm-weight gradients run as one launch
        per layer (mlm_deferred_sums_begin / _flush around the layer's backward calls; bit-identical results)."""
        self.cfg, self.L, self.shards, self.dev = cfg, int(n_layers), list(shards), torch.device(device)
        self.checkpoint, self.dropout, self.grouped_wgrads = checkpoint, dropout, grouped_wgrads
        self.deferred_sums, self._list_open = deferred_sums, False
        self.dt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
        self.code = B.MLM_BF16 if cfg.dtype == "bf16" else B.MLM_F32
        p = cfg.p
        self.T, self.Hl, self.Fl, self.Vl, self.hl = cfg.T, cfg.H // p, cfg.F // p, cfg.V // p, cfg.h // p
        self.dims = {r: B.make_dims(cfg.b, cfg.s, cfg.H, cfg.h, cfg.F, cfg.V, p, r, self.code, cfg.causal,
                                    cfg.gelu_tanh, cfg.ln_eps) for r in range(p)}
        self.d0 = self.dims[self.shards[0]]
        self.rep: Dict[str, object] = {}
        self.w: List[Dict[int, Dict[str, torch.Tensor]]] = []
        self.E: Dict[int, torch.Tensor] = {}
        self._alloc()

    # ------------------------------------------------------------------ dropout sites
    def site_offset(self, layer: int, site: str) -> int:
        step = int(self.dropout.get("step", 0)) if self.dropout else 0
        return (step << 32) | (16 * layer + SITES.get(site, 4))

    def _drop(self, layer: int, site: str, r: int = 0):
        if self.dropout is None:
            return None
        base = int(self.dropout["base_seed"])
        if site == "attn":
            return B.make_dropout(self.dropout["p_attn"], B.mlm_rng_stream_seed(base, B.STREAM_MODEL_PARALLEL, r),
                                  self.site_offset(layer, site))
        return B.make_dropout(self.dropout["p_hidden"], B.mlm_rng_stream_seed(base, B.STREAM_REPLICATED, 0),
                              self.site_offset(layer, site))

    # ------------------------------------------------------------------ inputs
    def load_host(self, model: Dict[str, object]):
        """model: the dictionary oracle-side tests build ("layers": per-layer UNSHARDED parameters, "E", "pos", "gf",
        "bf", "ids", "tgt", "w", "key_len"); weights are sliced with the library's own shard ranges."""
        cfg = self.cfg
        up = lambda a: torch.from_numpy(np.ascontiguousarray(np.asarray(a, np.float32))).to(self.dev).to(self.dt).contiguous()
        self.rep = {"gf": up(model["gf"]), "bf": up(model["bf"]), "pos": up(model["pos"]),
                    "ids": torch.from_numpy(np.asarray(model["ids"]).reshape(-1).astype(np.int32)).to(self.dev),
                    "tgt": torch.from_numpy(np.asarray(model["tgt"]).reshape(-1).astype(np.int32)).to(self.dev),
                    "w": torch.from_numpy(np.asarray(model["w"]).reshape(-1).astype(np.float32)).to(self.dev),
                    "key_len": torch.from_numpy(np.asarray(model["key_len"]).astype(np.int32)).to(self.dev),
                    "layers": [{k: up(P[k]) for k in LAYER_REP} for P in model["layers"]]}
        self.w = []
        for P in model["layers"]:
            per = {}
            for r in self.shards:
                c0, c1 = B.mlm_shard_range(cfg.H, cfg.p, r)
                f0, f1 = B.mlm_shard_range(cfg.F, cfg.p, r)
                per[r] = {"Wqkv": up(np.concatenate([P["Wq"][:, c0:c1], P["Wk"][:, c0:c1], P["Wv"][:, c0:c1]], axis=1)),
                          "bqkv": up(np.concatenate([P["bq"][c0:c1], P["bk"][c0:c1], P["bv"][c0:c1]])),
                          "Wo": up(P["Wo"][c0:c1, :]), "A": up(P["A"][:, f0:f1]), "a": up(P["a"][f0:f1]),
                          "B": up(P["B"][f0:f1, :])}
            self.w.append(per)
        for r in self.shards:
            v0, v1 = B.mlm_shard_range(cfg.V, cfg.p, r)
            self.E[r] = up(np.asarray(model["E"])[:, v0:v1])

    def load_random(self, seed: int = 0):
        """Synthetic parameters and inputs drawn on the device (weights N(0, std 0.02), Section 4.2)."""
        cfg, H = self.cfg, self.cfg.H
        g = torch.Generator(device=self.dev)
        g.manual_seed(seed)
        rn = lambda *shape, std=0.02: (torch.randn(*shape, generator=g, device=self.dev) * std).to(self.dt)
        ones = lambda n: torch.ones(n, device=self.dev, dtype=self.dt)
        zeros = lambda n: torch.zeros(n, device=self.dev, dtype=self.dt)
        ri = lambda: torch.randint(0, cfg.V, (cfg.T,), generator=g, device=self.dev, dtype=torch.int32)
        self.rep = {"gf": ones(H), "bf": zeros(H), "pos": rn(cfg.s, H), "ids": ri(), "tgt": ri(),
                    "w": torch.ones(cfg.T, device=self.dev),
                    "key_len": torch.full((cfg.b,), cfg.s, device=self.dev, dtype=torch.int32),
                    "layers": [dict(g1=ones(H), b1=zeros(H), bo=zeros(H), g2=ones(H), b2=zeros(H), c=zeros(H))
                               for _ in range(self.L)]}
        self.w = [{r: {"Wqkv": rn(H, 3 * self.Hl), "bqkv": zeros(3 * self.Hl), "Wo": rn(self.Hl, H),
                       "A": rn(H, self.Fl), "a": zeros(self.Fl), "B": rn(self.Fl, H)} for r in self.shards}
                  for _ in range(self.L)]
        self.E = {r: rn(H, self.Vl) for r in self.shards}

    # ------------------------------------------------------------------ buffers
    def _act_set(self):
        cfg, T, H = self.cfg, self.T, self.cfg.H
        e = lambda *shape, dtype=None: torch.empty(*shape, device=self.dev, dtype=dtype or self.dt)
        f32 = torch.float32
        a = {"U": e(T, H), "mu1": e(T, dtype=f32), "rstd1": e(T, dtype=f32), "X1": e(T, H), "U2": e(T, H),
             "mu2": e(T, dtype=f32), "rstd2": e(T, dtype=f32), "sh": {}}
        for r in self.shards:
            a["sh"][r] = {"qkv": e(T, 3 * self.Hl), "ctx": e(T, self.Hl), "lse": e(cfg.b, self.hl, cfg.s, dtype=f32),
                          "attn_partial": e(T, H), "g": e(T, self.Fl), "y": e(T, self.Fl), "mlp_partial": e(T, H)}
            if self.dropout is not None:
                a["sh"][r]["keep_bits"] = torch.zeros(B.mlm_attn_keep_words(self.dims[r]), device=self.dev,
                                                      dtype=torch.int32)
        return a

    def _alloc(self):
        cfg, T, H, L = self.cfg, self.T, self.cfg.H, self.L
        e = lambda *shape, dtype=None: torch.empty(*shape, device=self.dev, dtype=dtype or self.dt)
        f32 = torch.float32
        self.X = [e(T, H) for _ in range(L + 1)]                       # layer inputs; X[L] = the stack's output
        shared = self._act_set() if self.checkpoint else None
        self.acts = [shared if self.checkpoint else self._act_set() for _ in range(L)]
        n = len(self.shards)
        self.head = {"Hf": e(T, H), "muf": e(T, dtype=f32), "rstdf": e(T, dtype=f32), "m": e(n, T, dtype=f32),
                     "s": e(n, T, dtype=f32), "t": e(n, T, dtype=f32), "ce": e(T, dtype=f32), "M": e(T, dtype=f32),
                     "S": e(T, dtype=f32), "loss": e(2, dtype=f32), "dgf": e(H), "dbf": e(H), "dpos": e(cfg.s, H)}
        self.hsh = {r: {"logits": e(T, self.Vl), "dE": e(H, self.Vl), "dhf_partial": e(T, H), "perm": e(T, dtype=torch.int32),
                        "embed_partial": e(T, H)} for r in self.shards}
        # activation gradients of the chain: dX2 of the current layer, its dX1, and the layer's input gradient rotate
        # through three buffers, so that both block-output gradients are still intact when the layer's weight
        # gradients are computed at the end of its backward pass
        self.dXbuf = [e(T, H) for _ in range(3)]
        self.dX = self.dXbuf[0]
        self.dZ = {k: e(T, H) for k in (("dZ1", "dZ2", "dZ0") if self.dropout is not None else ())}
        self.gsh = [{r: {"dWqkv": e(H, 3 * self.Hl), "dbqkv": e(3 * self.Hl), "dWo": e(self.Hl, H), "dA": e(H, self.Fl),
                         "da": e(self.Fl), "dB": e(self.Fl, H)} for r in self.shards} for _ in range(L)]
        self.grep = [{k: e(H) for k in ("dg1", "db1", "dbo", "dg2", "db2", "dc")} for _ in range(L)]
        self.part = {r: {"du_partial": e(T, H), "du2_partial": e(T, H)} for r in self.shards}
        if self.grouped_wgrads:
            for r in self.shards:
                self.part[r]["dg"], self.part[r]["dqkv"] = e(T, self.Fl), e(T, 3 * self.Hl)
        wsb = max(B.mlm_workspace_bytes(self.d0, k) for k in range(8))
        self.ws = torch.empty(max(wsb, 256), device=self.dev, dtype=torch.uint8)
        self.defer_ws = (torch.empty(B.mlm_deferred_sums_bytes(self.d0) * len(self.shards), device=self.dev,
                                     dtype=torch.uint8) if self.deferred_sums else None)

    # ------------------------------------------------------------------ forward
    def _layer_body(self, l: int):
        """Attention shards, reduction + dropout + residual + LN2, MLP shards of layer l; U / mu1 / rstd1 of the layer
        must already be in its activation set."""
        a, rp, ws, d0 = self.acts[l], self.rep["layers"][l], self.ws, self.d0
        kl = self.rep["key_len"] if self.cfg.masked_lm else None
        for r in self.shards:
            w, s = self.w[l][r], a["sh"][r]
            if self.dropout is not None:
                B.mlm_attn_shard_fwd_dropout(self.dims[r], a["U"], w["Wqkv"], w["bqkv"], w["Wo"], kl,
                                             self._drop(l, "attn", r), s["qkv"], s["ctx"], s["lse"], s["keep_bits"],
                                             s["attn_partial"], ws)
            else:
                B.mlm_attn_shard_fwd(self.dims[r], a["U"], w["Wqkv"], w["bqkv"], w["Wo"], kl, s["qkv"], s["ctx"],
                                     s["lse"], s["attn_partial"], ws)
        B.mlm_combine_layernorm_fwd_dropout(d0, [a["sh"][r]["attn_partial"] for r in self.shards], rp["bo"],
                                            self._drop(l, "hidden1"), self.X[l], a["X1"], rp["g2"], rp["b2"], a["U2"],
                                            a["mu2"], a["rstd2"])
        for r in self.shards:
            w, s = self.w[l][r], a["sh"][r]
            B.mlm_mlp_shard_fwd(self.dims[r], a["U2"], w["A"], w["a"], w["B"], s["g"], s["y"], s["mlp_partial"], ws)

    def forward(self):
        rep, d0, ws, hd = self.rep, self.d0, self.ws, self.head
        for r in self.shards:
            B.mlm_embed_shard_fwd(self.dims[r], rep["ids"], self.E[r], self.hsh[r]["perm"], self.hsh[r]["embed_partial"])
        B.mlm_combine_dropout(d0, [self.hsh[r]["embed_partial"] for r in self.shards], rep["pos"], self.cfg.s,
                              self._drop(self.L, "embed"), None, self.X[0])
        a0, r0 = self.acts[0], rep["layers"][0]
        B.mlm_layernorm_fwd(d0, self.X[0], r0["g1"], r0["b1"], a0["U"], a0["mu1"], a0["rstd1"])
        for l in range(self.L):
            self._layer_body(l)
            a, rp = self.acts[l], rep["layers"][l]
            partials = [a["sh"][r]["mlp_partial"] for r in self.shards]
            # the reduction that ends the layer, fused with the NEXT layer norm (layer l+1's first, or the final one)
            if l + 1 < self.L:
                an, rn = self.acts[l + 1], rep["layers"][l + 1]
                B.mlm_combine_layernorm_fwd_dropout(d0, partials, rp["c"], self._drop(l, "hidden2"), a["X1"],
                                                    self.X[l + 1], rn["g1"], rn["b1"], an["U"], an["mu1"], an["rstd1"])
            else:
                B.mlm_combine_layernorm_fwd_dropout(d0, partials, rp["c"], self._drop(l, "hidden2"), a["X1"],
                                                    self.X[self.L], rep["gf"], rep["bf"], hd["Hf"], hd["muf"], hd["rstdf"])
        for i, r in enumerate(self.shards):
            B.mlm_vocab_ce_shard_fwd(self.dims[r], hd["Hf"], self.E[r], rep["tgt"], hd["m"][i], hd["s"][i], hd["t"][i],
                                     self.hsh[r]["logits"], ws)
        B.mlm_vocab_ce_merge(d0, hd["m"], hd["s"], hd["t"], len(self.shards), rep["w"], hd["ce"], hd["M"], hd["S"],
                             hd["loss"])

    # ------------------------------------------------------------------ backward
    def recompute_layer(self, l: int):
        a, rp = self.acts[l], self.rep["layers"][l]
        B.mlm_layernorm_fwd(self.d0, self.X[l], rp["g1"], rp["b1"], a["U"], a["mu1"], a["rstd1"])
        self._layer_body(l)

    def _sums_open(self):
        if self.deferred_sums and not self._list_open:
            B.mlm_deferred_sums_begin(self.defer_ws)
            self._list_open = True

    def _sums_flush(self):
        if self._list_open:
            self._list_open = False
            B.mlm_deferred_sums_flush()

    def backward(self):
        self._sums_open()
        try:
            self._backward_calls()
        finally:
            self._sums_flush()

    def _backward_calls(self):
        rep, d0, ws, hd = self.rep, self.d0, self.ws, self.head
        drop = self.dropout is not None
        kl = rep["key_len"] if self.cfg.masked_lm else None
        dZ = self.dZ
        b2, b1, b0 = self.dXbuf                     # dX2 of the layer at hand, its dX1, the gradient of its input
        for r in self.shards:
            s = self.hsh[r]
            B.mlm_vocab_ce_shard_bwd(self.dims[r], hd["Hf"], self.E[r], rep["tgt"], rep["w"], hd["M"], hd["S"], hd["loss"],
                                     s["logits"], s["dE"], s["dhf_partial"], ws)
        last = self.L - 1
        B.mlm_combine_layernorm_bwd_dropout(d0, [self.hsh[r]["dhf_partial"] for r in self.shards], self.X[self.L],
                                            rep["gf"], hd["muf"], hd["rstdf"], None, self._drop(last, "hidden2"), None, b2,
                                            dZ.get("dZ2"), hd["dgf"], hd["dbf"], self.grep[last]["dc"], ws)
        for l in reversed(range(self.L)):
            if self.checkpoint:
                self.recompute_layer(l)
            a, rp, gr = self.acts[l], rep["layers"][l], self.grep[l]
            dz2 = dZ["dZ2"] if drop else b2
            for r in self.shards:
                w, s, g = self.w[l][r], a["sh"][r], self.gsh[l][r]
                if self.grouped_wgrads:
                    B.mlm_mlp_shard_bwd_input(self.dims[r], dz2, w["A"], w["B"], s["g"], self.part[r]["dg"], g["da"],
                                              self.part[r]["du2_partial"], ws)
                else:
                    B.mlm_mlp_shard_bwd(self.dims[r], dz2, a["U2"], w["A"], w["B"], s["g"], s["y"], g["dA"], g["da"],
                                        g["dB"], self.part[r]["du2_partial"], ws)
            B.mlm_combine_layernorm_bwd_dropout(d0, [self.part[r]["du2_partial"] for r in self.shards], a["X1"], rp["g2"],
                                                a["mu2"], a["rstd2"], b2, self._drop(l, "hidden1"), None, b1,
                                                dZ.get("dZ1"), gr["dg2"], gr["db2"], gr["dbo"], ws)
            dz1 = dZ["dZ1"] if drop else b1
            for r in self.shards:
                w, s, g, pt = self.w[l][r], a["sh"][r], self.gsh[l][r], self.part[r]
                if self.grouped_wgrads:
                    B.mlm_attn_shard_bwd_input(self.dims[r], dz1, w["Wqkv"], w["Wo"], kl,
                                               self._drop(l, "attn", r), s["qkv"], s["ctx"], s["lse"],
                                               s["keep_bits"] if drop else None, pt["dqkv"], g["dbqkv"], pt["du_partial"], ws)
                    # both block-output gradients of this layer are still intact here (the next call overwrites dZ2)
                    B.mlm_layer_shard_wgrads(self.dims[r], a["U"], pt["dqkv"], s["ctx"], dz1, a["U2"], pt["dg"], s["y"],
                                             dz2, g["dWqkv"], g["dWo"], g["dA"], g["dB"], ws)
                elif drop:
                    B.mlm_attn_shard_bwd_dropout(self.dims[r], dz1, a["U"], w["Wqkv"], w["Wo"], kl,
                                                 self._drop(l, "attn", r), s["qkv"], s["ctx"], s["lse"], s["keep_bits"],
                                                 g["dWqkv"], g["dbqkv"], g["dWo"], pt["du_partial"], ws)
                else:
                    B.mlm_attn_shard_bwd(self.dims[r], dz1, a["U"], w["Wqkv"], w["Wo"], kl, s["qkv"], s["ctx"], s["lse"],
                                         g["dWqkv"], g["dbqkv"], g["dWo"], pt["du_partial"], ws)
            du = [self.part[r]["du_partial"] for r in self.shards]
            if l > 0:
                # LN1 of layer l consumed the output of layer l-1's MLP block: its backward also yields that block's
                # pre-dropout gradient and bias gradient
                B.mlm_combine_layernorm_bwd_dropout(d0, du, self.X[l], rp["g1"], a["mu1"], a["rstd1"], b1,
                                                    self._drop(l - 1, "hidden2"), None, b0, dZ.get("dZ2"), gr["dg1"],
                                                    gr["db1"], self.grep[l - 1]["dc"], ws)
            else:
                B.mlm_combine_layernorm_bwd(d0, du, self.X[0], rp["g1"], a["mu1"], a["rstd1"], b1, None, b0, gr["dg1"],
                                            gr["db1"], None, ws)
            b2, b1, b0 = b0, b2, b1                 # the input gradient is the next (lower) layer's dX2
            self._sums_flush()                      # one finishing launch per layer; the list's buffer is reused
            self._sums_open()
        dX = self.dX = b2
        B.mlm_embed_bwd_replicated(d0, dX, self._drop(self.L, "embed"), dZ["dZ0"] if drop else dX, hd["dpos"])
        for r in self.shards:
            B.mlm_embed_shard_bwd(self.dims[r], rep["ids"], self.hsh[r]["perm"], dZ["dZ0"] if drop else dX,
                                  self.hsh[r]["dE"])

    def step(self):
        self.forward()
        self.backward()

    # ------------------------------------------------------------------ optimizer (this worker group's parameters)
    def parameters(self):
        out = []
        for l in range(self.L):
            for r in self.shards:
                for k in LAYER_SHARD:
                    out.append((f"{l}.{r}.{k}", self.w[l][r][k], self.gsh[l][r]["d" + k]))
            for k in LAYER_REP:
                out.append((f"{l}.{k}", self.rep["layers"][l][k], self.grep[l]["d" + k]))
        for r in self.shards:
            out.append((f"E.{r}", self.E[r], self.hsh[r]["dE"]))
        out += [("gf", self.rep["gf"], self.head["dgf"]), ("bf", self.rep["bf"], self.head["dbf"]),
                ("pos", self.rep["pos"], self.head["dpos"])]
        return out

    def optimizer_step(self, step: int, lr: float, max_norm: float = 1.0, beta1: float = 0.9, beta2: float = 0.999,
                       eps: float = 1e-8, weight_decay: float = 0.01):
        """Global gradient-norm clip + AdamW over every parameter, 64 tensors per library call (the squared norm is
        chained through the calls' `other_sqnorm` input)."""
        params = self.parameters()
        if not hasattr(self, "opt"):
            self.opt = {n: {"master": w.float().clone(), "m": torch.zeros_like(w, dtype=torch.float32),
                            "v": torch.zeros_like(w, dtype=torch.float32)} for n, w, _ in params}
            self.opt_ws = torch.empty(64 * 4096, device=self.dev, dtype=torch.uint8)
            self.sqnorm = [torch.zeros(1, device=self.dev, dtype=torch.float32) for _ in range(2)]
        prev = None
        chunks = [params[i:i + 64] for i in range(0, len(params), 64)]
        for i, ch in enumerate(chunks):
            B.mlm_grad_sqnorm(self.code, [g for _, _, g in ch], prev, self.sqnorm[i & 1], self.opt_ws)
            prev = self.sqnorm[i & 1]
        for ch in chunks:
            st = [self.opt[n] for n, _, _ in ch]
            B.mlm_adamw_step_multi(self.code, [g for _, _, g in ch], [x["master"] for x in st], [x["m"] for x in st],
                                   [x["v"] for x in st], [w for _, w, _ in ch], [weight_decay] * len(ch), prev,
                                   max_norm, lr, beta1, beta2, eps, step)

    # ------------------------------------------------------------------ results
    def fetch(self) -> Dict[str, object]:
        torch.cuda.synchronize(self.dev)
        cp = lambda t: t.detach().float().cpu().numpy().astype(np.float64)
        out: Dict[str, object] = {"X": [cp(x) for x in self.X], "Hf": cp(self.head["Hf"]), "ce": cp(self.head["ce"]),
                                  "loss": float(self.head["loss"][0].item()), "dX0": cp(self.dX),
                                  "dgf": cp(self.head["dgf"]), "dbf": cp(self.head["dbf"]), "dpos": cp(self.head["dpos"]),
                                  "dE": {r: cp(self.hsh[r]["dE"]) for r in self.shards},
                                  "layers": [{"rep": {k: cp(v) for k, v in self.grep[l].items()},
                                              "sh": {r: {k: cp(v) for k, v in self.gsh[l][r].items()} for r in self.shards}}
                                             for l in range(self.L)]}
        return out
