"""Sequencer of the layer-shard path on one GPU (allocation and call order only; all arithmetic is in the HIP library).

Runs the forward and backward pass of a model-parallel transformer layer plus the vocabulary-parallel loss for a
chosen set of shards, stage by stage, because shard r's MLP consumes the *combined* attention output (Section 3 of
the paper: two reductions forward, two backward per layer; here ``mlm_combine`` / ``mlm_vocab_ce_merge`` stand in
for them).  With ``shards = range(p)`` the result is the full layer (used to prove the sharding exact); with
``shards = [0]`` it is one GPU's share at its real shape (what the benchmark times).
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

from . import binding as B
from .synth import LayerConfig


def _tdtype(cfg: LayerConfig):
    return torch.bfloat16 if cfg.dtype == "bf16" else torch.float32


class LayerShards:
    def __init__(self, cfg: LayerConfig, shards: Sequence[int], device: str = "cuda:0", store_logits: bool = True,
                 fused: bool = True, store_combined: bool = False, dropout: Optional[Dict[str, object]] = None,
                 embed: bool = False, loss_rows: bool = False, grouped_wgrads: bool = True, post_ln: bool = False,
                 deferred_sums: bool = True):
        """fused: the combine that stands in for an all-reduce runs inside the layer-norm kernel that consumes it
        (and the layer-norm backward also emits the row-parallel bias gradient); store_combined: in fused mode,
        also store the combined gradients dHf / dU2 / dU (nothing in the path reads them).
        dropout: None, or {"p_attn", "p_hidden", "base_seed", "offsets": {"attn", "hidden1", "hidden2", "embed"}} --
        the two-stream dropout of Appendix B.2 (fused mode only): the attention-probability site of shard r draws
        from worker r's model-parallel stream, the hidden sites from the replicated stream.
        embed: the layer input is produced by the vocabulary-parallel input embedding (token ids + position
        embedding) instead of being given, and its backward adds into the tied dE.
        loss_rows: the rows of the final hidden state that carry loss weight are gathered first and the vocabulary-
        parallel logits / loss / gradient calls run on that compact tensor only (BERT-style masked-LM loss: ~15 % of
        the positions); the input gradient is scattered back with zeros elsewhere.  Same loss and gradients.
        grouped_wgrads: the backward calls compute input gradients only and the four weight gradients of each layer
        shard are computed afterwards by one mlm_layer_shard_wgrads call (one grouped GEMM launch).
        deferred_sums: the backward pass runs between mlm_deferred_sums_begin and mlm_deferred_sums_flush, so the
        finishing reductions of the bias and layer-norm-weight gradients are one launch at its end instead of one per
        call (bit-identical results).
        post_ln: the ORIGINAL BERT arrangement the paper compares against (Section 5.3): layer norm after each
        residual add, X1 = LN(X + Attn(X)), X2 = LN(X1 + MLP(X1)), logits from X2; same entry points, other call order."""
        self.cfg, self.shards, self.dev = cfg, list(shards), torch.device(device)
        self.fused, self.store_combined = fused, store_combined
        self.dropout, self.embed, self.loss_rows = dropout, embed, loss_rows
        self.grouped_wgrads = grouped_wgrads
        self.deferred_sums = deferred_sums
        self.post_ln = post_ln
        if post_ln and (dropout is not None or embed or loss_rows or not fused):
            raise ValueError("the post-LN arrangement is wired for the plain fused path only")
        if dropout is not None and not fused:
            raise ValueError("dropout is wired into the fused combine + layer-norm calls only")
        self.dt = _tdtype(cfg)
        self.code = B.MLM_BF16 if cfg.dtype == "bf16" else B.MLM_F32
        self.store_logits = store_logits
        p = cfg.p
        self.T = cfg.T
        self.d = cfg.H // cfg.h
        self.Hl, self.Fl, self.Vl = cfg.H // p, cfg.F // p, cfg.V // p
        self.hl = cfg.h // p
        self.dims = {r: B.make_dims(cfg.b, cfg.s, cfg.H, cfg.h, cfg.F, cfg.V, p, r, self.code, cfg.causal,
                                    cfg.gelu_tanh, cfg.ln_eps) for r in range(p)}
        self.drop: Dict[str, object] = {}
        if dropout is not None:
            off, base = dropout["offsets"], int(dropout["base_seed"])
            rep_seed = B.mlm_rng_stream_seed(base, B.STREAM_REPLICATED, 0)
            for site in ("hidden1", "hidden2", "embed"):
                self.drop[site] = B.make_dropout(dropout["p_hidden"], rep_seed, off[site])
            self.drop["attn"] = {r: B.make_dropout(dropout["p_attn"], B.mlm_rng_stream_seed(base, B.STREAM_MODEL_PARALLEL, r),
                                                   off["attn"]) for r in range(p)}
        self.rep: Dict[str, torch.Tensor] = {}       # replicated parameters and inputs
        self.w: Dict[int, Dict[str, torch.Tensor]] = {}   # per-shard parameters
        self.act: Dict[str, torch.Tensor] = {}       # replicated activations / gradients
        self.sh: Dict[int, Dict[str, torch.Tensor]] = {}  # per-shard activations / gradients
        self._alloc()

    # ------------------------------------------------------------------ inputs
    def load_host_inputs(self, inp: Dict[str, np.ndarray]):
        """Upload unsharded host arrays; weights are sliced with the library's own shard ranges."""
        cfg = self.cfg
        up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(self.dev).to(self.dt).contiguous()
        for k in ("g1", "b1", "bo", "g2", "b2", "c", "gf", "bf"):
            self.rep[k] = up(inp[k])
        if self.embed:
            self.rep["ids"] = torch.from_numpy(inp["ids"].reshape(-1).astype(np.int32)).to(self.dev)
            self.rep["pos"] = up(inp["pos"])
            self.rep["X"] = torch.empty(cfg.T, cfg.H, device=self.dev, dtype=self.dt)
        else:
            self.rep["X"] = up(inp["X"].reshape(cfg.T, cfg.H))
        self.rep["tgt"] = torch.from_numpy(inp["tgt"].reshape(-1).astype(np.int32)).to(self.dev)
        self.rep["w"] = torch.from_numpy(inp["w"].reshape(-1).astype(np.float32)).to(self.dev)
        self.rep["key_len"] = torch.from_numpy(inp["key_len"].astype(np.int32)).to(self.dev)
        for r in self.shards:
            c0, c1 = B.mlm_shard_range(cfg.H, cfg.p, r)
            f0, f1 = B.mlm_shard_range(cfg.F, cfg.p, r)
            v0, v1 = B.mlm_shard_range(cfg.V, cfg.p, r)
            self.w[r] = {
                "Wqkv": up(np.concatenate([inp["Wq"][:, c0:c1], inp["Wk"][:, c0:c1], inp["Wv"][:, c0:c1]], axis=1)),
                "bqkv": up(np.concatenate([inp["bq"][c0:c1], inp["bk"][c0:c1], inp["bv"][c0:c1]])),
                "Wo": up(inp["Wo"][c0:c1, :]),
                "A": up(inp["A"][:, f0:f1]), "a": up(inp["a"][f0:f1]), "B": up(inp["B"][f0:f1, :]),
                "E": up(inp["E"][:, v0:v1]),
            }
        self._prepare_loss_rows()

    def _prepare_loss_rows(self):
        """Row list of the positions with loss weight 1 and the compact targets / weights / buffers (input plumbing:
        an index list built from the given loss mask)."""
        if not self.loss_rows:
            return
        cfg, dev, dt, f32 = self.cfg, self.dev, self.dt, torch.float32
        idx = torch.nonzero(self.rep["w"] > 0).reshape(-1).to(torch.int32)
        n = int(idx.numel())
        n_pad = max(64, (n + 63) // 64 * 64)      # k of the dE GEMM: a multiple of 32 keeps it on the direct-to-LDS kernel
        self.n_rows, self.n_pad = n, n_pad
        self.rep["row_idx"] = idx.contiguous()
        tgt_c = torch.zeros(n_pad, device=dev, dtype=torch.int32)
        tgt_c[:n] = self.rep["tgt"][idx.long()]
        w_c = torch.zeros(n_pad, device=dev, dtype=f32)
        w_c[:n] = 1.0
        self.rep["tgt_c"], self.rep["w_c"] = tgt_c, w_c
        self.dims_c = {r: B.make_dims(1, n_pad, cfg.H, cfg.h, cfg.F, cfg.V, cfg.p, r, self.code, cfg.causal,
                                      cfg.gelu_tanh, cfg.ln_eps) for r in range(cfg.p)}
        e = lambda *shape, dtype=dt: torch.empty(*shape, device=dev, dtype=dtype)
        a, ns = self.act, len(self.shards)
        a["Hf_c"], a["dHf_c"] = e(n_pad, cfg.H), e(n_pad, cfg.H)
        a["m"], a["s"], a["t"] = e(ns, n_pad, dtype=f32), e(ns, n_pad, dtype=f32), e(ns, n_pad, dtype=f32)
        a["ce"], a["M"], a["S"] = e(n_pad, dtype=f32), e(n_pad, dtype=f32), e(n_pad, dtype=f32)
        for r in self.shards:
            self.sh[r]["logits"] = e(n_pad, self.Vl) if self.store_logits else None
            self.sh[r]["dhf_partial"] = e(n_pad, cfg.H)

    def load_random(self, seed: int = 0):
        """Synthetic inputs drawn on the device (benchmark use: same shapes and distributions as synth.make_inputs)."""
        cfg = self.cfg
        g = torch.Generator(device=self.dev)
        g.manual_seed(seed)
        rn = lambda *shape, std=0.02: (torch.randn(*shape, generator=g, device=self.dev) * std).to(self.dt)
        ones = lambda n: torch.ones(n, device=self.dev, dtype=self.dt)
        zeros = lambda n: torch.zeros(n, device=self.dev, dtype=self.dt)
        H = cfg.H
        self.rep.update(X=rn(cfg.T, H, std=1.0), g1=ones(H), b1=zeros(H), g2=ones(H), b2=zeros(H), gf=ones(H),
                        bf=zeros(H), bo=zeros(H), c=zeros(H))
        self.rep["tgt"] = torch.randint(0, cfg.V, (cfg.T,), generator=g, device=self.dev, dtype=torch.int32)
        if self.embed:
            self.rep["ids"] = torch.randint(0, cfg.V, (cfg.T,), generator=g, device=self.dev, dtype=torch.int32)
            self.rep["pos"] = rn(cfg.s, H)
        if cfg.masked_lm:
            kl = torch.randint(max(1, cfg.s // 2), cfg.s + 1, (cfg.b,), generator=g, device=self.dev, dtype=torch.int32)
            pos = torch.arange(cfg.s, device=self.dev)[None, :]
            w = (torch.rand(cfg.b, cfg.s, generator=g, device=self.dev) < 0.15) & (pos < kl[:, None])
            w[0, 0] = True
            self.rep["key_len"], self.rep["w"] = kl, w.reshape(-1).float()
        else:
            self.rep["key_len"] = torch.full((cfg.b,), cfg.s, device=self.dev, dtype=torch.int32)
            self.rep["w"] = torch.ones(cfg.T, device=self.dev)
        for r in self.shards:
            self.w[r] = {"Wqkv": rn(H, 3 * self.Hl), "bqkv": zeros(3 * self.Hl), "Wo": rn(self.Hl, H),
                         "A": rn(H, self.Fl), "a": zeros(self.Fl), "B": rn(self.Fl, H), "E": rn(H, self.Vl)}
        self._prepare_loss_rows()

    # ------------------------------------------------------------------ buffers
    def _alloc(self):
        cfg, T, H, dev, dt = self.cfg, self.T, self.cfg.H, self.dev, self.dt
        e = lambda *shape, dtype=dt: torch.empty(*shape, device=dev, dtype=dtype)
        f32 = torch.float32
        a = self.act
        for k in ("U", "X1", "U2", "X2", "Hf", "dHf", "dX2", "dU2", "dX1", "dU", "dX"):
            a[k] = e(T, H)
        for k in ("mu1", "rstd1", "mu2", "rstd2", "muf", "rstdf", "ce", "M", "S"):
            a[k] = e(T, dtype=f32)
        for k in ("dg1", "db1", "dg2", "db2", "dgf", "dbf", "dbo", "dc"):
            a[k] = e(H)
        n = len(self.shards)
        a["m"], a["s"], a["t"] = e(n, T, dtype=f32), e(n, T, dtype=f32), e(n, T, dtype=f32)
        a["loss"] = e(2, dtype=f32)
        d0 = self.dims[self.shards[0]]
        wsb = max(B.mlm_workspace_bytes(d0, k) for k in range(8))
        self.ws = torch.empty(max(wsb, 256), device=dev, dtype=torch.uint8)
        self.defer_ws = (torch.empty(B.mlm_deferred_sums_bytes(d0) * len(self.shards), device=dev, dtype=torch.uint8)
                         if self.deferred_sums else None)
        if self.dropout is not None:
            a["dZ1"], a["dZ2"] = e(T, H), e(T, H)
        if self.embed:
            a["dZ0"], a["dpos"] = e(T, H), e(cfg.s, H)
        for r in self.shards:
            self.sh[r] = {
                "qkv": e(T, 3 * self.Hl), "ctx": e(T, self.Hl), "lse": e(cfg.b, self.hl, cfg.s, dtype=f32),
                "attn_partial": e(T, H), "g": e(T, self.Fl), "y": e(T, self.Fl), "mlp_partial": e(T, H),
                "logits": e(T, self.Vl) if self.store_logits else None,
                "dE": e(H, self.Vl), "dhf_partial": e(T, H),
                "dA": e(H, self.Fl), "da": e(self.Fl), "dB": e(self.Fl, H), "du2_partial": e(T, H),
                "dWqkv": e(H, 3 * self.Hl), "dbqkv": e(3 * self.Hl), "dWo": e(self.Hl, H), "du_partial": e(T, H),
            }
            if self.grouped_wgrads:
                self.sh[r]["dg"], self.sh[r]["dqkv"] = e(T, self.Fl), e(T, 3 * self.Hl)
            if self.dropout is not None:
                self.sh[r]["keep_bits"] = torch.zeros(B.mlm_attn_keep_words(self.dims[r]), device=dev, dtype=torch.int32)
            if self.embed:
                self.sh[r]["perm"] = e(T, dtype=torch.int32)
                self.sh[r]["embed_partial"] = e(T, H)

    # ------------------------------------------------------------------ the path
    def _embed_forward(self):
        """X = dropout(sum_r E_r[:, id] + position embedding): per-shard lookups, then the stand-in for g."""
        d0, rep = self.dims[self.shards[0]], self.rep
        for r in self.shards:
            B.mlm_embed_shard_fwd(self.dims[r], rep["ids"], self.w[r]["E"], self.sh[r]["perm"],
                                  self.sh[r]["embed_partial"])
        B.mlm_combine_dropout(d0, [self.sh[r]["embed_partial"] for r in self.shards], rep["pos"], self.cfg.s,
                              self.drop.get("embed"), None, rep["X"])

    def _layer_forward(self):
        """LN1, attention shards, combine (+dropout) + LN2, MLP shards: everything up to the MLP partial sums."""
        cfg, a, rep, ws = self.cfg, self.act, self.rep, self.ws
        d0 = self.dims[self.shards[0]]
        kl = rep["key_len"] if cfg.masked_lm else None
        B.mlm_layernorm_fwd(d0, rep["X"], rep["g1"], rep["b1"], a["U"], a["mu1"], a["rstd1"])
        for r in self.shards:
            w, s = self.w[r], self.sh[r]
            if self.dropout is not None:
                B.mlm_attn_shard_fwd_dropout(self.dims[r], a["U"], w["Wqkv"], w["bqkv"], w["Wo"], kl, self.drop["attn"][r],
                                             s["qkv"], s["ctx"], s["lse"], s["keep_bits"], s["attn_partial"], ws)
            else:
                B.mlm_attn_shard_fwd(self.dims[r], a["U"], w["Wqkv"], w["bqkv"], w["Wo"], kl, s["qkv"], s["ctx"],
                                     s["lse"], s["attn_partial"], ws)
        attn_partials = [self.sh[r]["attn_partial"] for r in self.shards]
        if self.dropout is not None:
            B.mlm_combine_layernorm_fwd_dropout(d0, attn_partials, rep["bo"], self.drop["hidden1"], rep["X"], a["X1"],
                                                rep["g2"], rep["b2"], a["U2"], a["mu2"], a["rstd2"])
        elif self.fused:
            B.mlm_combine_layernorm_fwd(d0, attn_partials, rep["bo"], rep["X"], a["X1"], rep["g2"], rep["b2"], a["U2"],
                                        a["mu2"], a["rstd2"])
        else:
            B.mlm_combine(d0, attn_partials, rep["bo"], rep["X"], a["X1"])
            B.mlm_layernorm_fwd(d0, a["X1"], rep["g2"], rep["b2"], a["U2"], a["mu2"], a["rstd2"])
        for r in self.shards:
            w, s = self.w[r], self.sh[r]
            B.mlm_mlp_shard_fwd(self.dims[r], a["U2"], w["A"], w["a"], w["B"], s["g"], s["y"], s["mlp_partial"], ws)

    # ---- the original (post-LN) arrangement: a["X1"] / a["X2"] hold the SUMS before the layer norms (the tensors the
    #      norms' backward needs), a["U2"] the normalised attention-block output (= the MLP's input and residual) and
    #      a["Hf"] the normalised layer output
    def _forward_post_ln(self):
        cfg, a, rep, ws = self.cfg, self.act, self.rep, self.ws
        d0 = self.dims[self.shards[0]]
        kl = rep["key_len"] if cfg.masked_lm else None
        for r in self.shards:
            w, s = self.w[r], self.sh[r]
            B.mlm_attn_shard_fwd(self.dims[r], rep["X"], w["Wqkv"], w["bqkv"], w["Wo"], kl, s["qkv"], s["ctx"], s["lse"],
                                 s["attn_partial"], ws)
        B.mlm_combine_layernorm_fwd(d0, [self.sh[r]["attn_partial"] for r in self.shards], rep["bo"], rep["X"], a["X1"],
                                    rep["g1"], rep["b1"], a["U2"], a["mu1"], a["rstd1"])
        for r in self.shards:
            w, s = self.w[r], self.sh[r]
            B.mlm_mlp_shard_fwd(self.dims[r], a["U2"], w["A"], w["a"], w["B"], s["g"], s["y"], s["mlp_partial"], ws)
        B.mlm_combine_layernorm_fwd(d0, [self.sh[r]["mlp_partial"] for r in self.shards], rep["c"], a["U2"], a["X2"],
                                    rep["g2"], rep["b2"], a["Hf"], a["mu2"], a["rstd2"])
        self._hf = a["Hf"]
        for i, r in enumerate(self.shards):
            B.mlm_vocab_ce_shard_fwd(self.dims[r], a["Hf"], self.w[r]["E"], rep["tgt"], a["m"][i], a["s"][i], a["t"][i],
                                     self.sh[r]["logits"], ws)
        B.mlm_vocab_ce_merge(d0, a["m"], a["s"], a["t"], len(self.shards), rep["w"], a["ce"], a["M"], a["S"], a["loss"])

    def _backward_post_ln(self):
        cfg, a, rep, ws = self.cfg, self.act, self.rep, self.ws
        d0 = self.dims[self.shards[0]]
        kl = rep["key_len"] if cfg.masked_lm else None
        for r in self.shards:
            w, s = self.w[r], self.sh[r]
            B.mlm_vocab_ce_shard_bwd(self.dims[r], a["Hf"], w["E"], rep["tgt"], rep["w"], a["M"], a["S"], a["loss"],
                                     s["logits"], s["dE"], s["dhf_partial"], ws)
        # LN2 backward on dX2 = sum of the logits input-gradient partials: gradient of the MLP block's sum S2
        B.mlm_combine_layernorm_bwd(d0, [self.sh[r]["dhf_partial"] for r in self.shards], a["X2"], rep["g2"], a["mu2"],
                                    a["rstd2"], None, None, a["dX2"], a["dg2"], a["db2"], a["dc"], ws)
        for r in self.shards:
            w, s = self.w[r], self.sh[r]
            B.mlm_mlp_shard_bwd(self.dims[r], a["dX2"], a["U2"], w["A"], w["B"], s["g"], s["y"], s["dA"], s["da"],
                                s["dB"], s["du2_partial"], ws)
        # the attention block's normalised output fed the MLP AND its residual: its gradient is the MLP input-gradient
        # partials plus dS2 -- one more term of the same sum -- and LN1's backward turns it into the gradient of S1
        B.mlm_combine_layernorm_bwd(d0, [self.sh[r]["du2_partial"] for r in self.shards] + [a["dX2"]], a["X1"], rep["g1"],
                                    a["mu1"], a["rstd1"], None, None, a["dX1"], a["dg1"], a["db1"], a["dbo"], ws)
        for r in self.shards:
            w, s = self.w[r], self.sh[r]
            B.mlm_attn_shard_bwd(self.dims[r], a["dX1"], rep["X"], w["Wqkv"], w["Wo"], kl, s["qkv"], s["ctx"], s["lse"],
                                 s["dWqkv"], s["dbqkv"], s["dWo"], s["du_partial"], ws)
        B.mlm_combine(d0, [self.sh[r]["du_partial"] for r in self.shards], None, a["dX1"], a["dX"])
        self._dx2 = a["dX2"]

    def forward(self):
        if self.post_ln:
            return self._forward_post_ln()
        cfg, a, rep, ws = self.cfg, self.act, self.rep, self.ws
        d0 = self.dims[self.shards[0]]
        if self.embed:
            self._embed_forward()
        self._layer_forward()
        mlp_partials = [self.sh[r]["mlp_partial"] for r in self.shards]
        if self.dropout is not None and cfg.final_ln:
            B.mlm_combine_layernorm_fwd_dropout(d0, mlp_partials, rep["c"], self.drop["hidden2"], a["X1"], a["X2"],
                                                rep["gf"], rep["bf"], a["Hf"], a["muf"], a["rstdf"])
            hf = a["Hf"]
        elif self.dropout is not None:
            B.mlm_combine_dropout(d0, mlp_partials, rep["c"], 1, self.drop["hidden2"], a["X1"], a["X2"])
            hf = a["X2"]
        elif cfg.final_ln and self.fused:
            B.mlm_combine_layernorm_fwd(d0, mlp_partials, rep["c"], a["X1"], a["X2"], rep["gf"], rep["bf"], a["Hf"],
                                        a["muf"], a["rstdf"])
            hf = a["Hf"]
        elif cfg.final_ln:
            B.mlm_combine(d0, mlp_partials, rep["c"], a["X1"], a["X2"])
            B.mlm_layernorm_fwd(d0, a["X2"], rep["gf"], rep["bf"], a["Hf"], a["muf"], a["rstdf"])
            hf = a["Hf"]
        else:
            B.mlm_combine(d0, mlp_partials, rep["c"], a["X1"], a["X2"])
            hf = a["X2"]
        self._hf = hf
        cdims, tgt, lw, dc0 = self.dims, rep["tgt"], rep["w"], d0
        if self.loss_rows:
            B.mlm_rows_gather(d0, hf, rep["row_idx"], self.n_rows, self.n_pad, a["Hf_c"])
            hf, cdims, tgt, lw = a["Hf_c"], self.dims_c, rep["tgt_c"], rep["w_c"]
            dc0 = cdims[self.shards[0]]
        for i, r in enumerate(self.shards):
            w, s = self.w[r], self.sh[r]
            B.mlm_vocab_ce_shard_fwd(cdims[r], hf, w["E"], tgt, a["m"][i], a["s"][i], a["t"][i], s["logits"], ws)
        B.mlm_vocab_ce_merge(dc0, a["m"], a["s"], a["t"], len(self.shards), lw, a["ce"], a["M"], a["S"], a["loss"])

    def backward(self):
        if not self.deferred_sums:
            return self._backward_calls()
        B.mlm_deferred_sums_begin(self.defer_ws)
        try:
            self._backward_calls()
        finally:
            B.mlm_deferred_sums_flush()

    def _backward_calls(self):
        if self.post_ln:
            return self._backward_post_ln()
        cfg, a, rep, ws = self.cfg, self.act, self.rep, self.ws
        d0 = self.dims[self.shards[0]]
        kl = rep["key_len"] if cfg.masked_lm else None
        hf = self._hf
        cdims, tgt, lw = self.dims, rep["tgt"], rep["w"]
        if self.loss_rows:
            hf, cdims, tgt, lw = a["Hf_c"], self.dims_c, rep["tgt_c"], rep["w_c"]
        for r in self.shards:
            w, s = self.w[r], self.sh[r]
            B.mlm_vocab_ce_shard_bwd(cdims[r], hf, w["E"], tgt, lw, a["M"], a["S"], a["loss"], s["logits"], s["dE"],
                                     s["dhf_partial"], ws)
        fused = self.fused
        # (with loss_rows the combined dHf IS the one partial: it must not also be the kernel's dy_out)
        keep = (lambda k: None if (k == "dHf" and self.loss_rows) else a[k]) if self.store_combined else (lambda k: None)
        dhf_partials = [self.sh[r]["dhf_partial"] for r in self.shards]
        if self.loss_rows:
            # reduce the compact partials, then put the rows back (zeros elsewhere): one [T,H] "partial" for what follows
            B.mlm_combine(cdims[self.shards[0]], dhf_partials, None, None, a["dHf_c"])
            B.mlm_rows_scatter(d0, a["dHf_c"], rep["row_idx"], self.n_rows, a["dHf"])
            dhf_partials = [a["dHf"]]
        drop = self.dropout is not None
        dz2 = dz1 = None          # gradients of the block outputs BEFORE their dropout (what the shards' backward reads)
        if drop and cfg.final_ln:
            B.mlm_combine_layernorm_bwd_dropout(d0, dhf_partials, a["X2"], rep["gf"], a["muf"], a["rstdf"], None,
                                                self.drop["hidden2"], keep("dHf"), a["dX2"], a["dZ2"], a["dgf"],
                                                a["dbf"], a["dc"], ws)
            dx2, dz2 = a["dX2"], a["dZ2"]
        elif drop:
            B.mlm_combine(d0, dhf_partials, None, None, a["dHf"])
            B.mlm_combine_dropout(d0, dhf_partials, None, 1, self.drop["hidden2"], None, a["dZ2"])
            B.mlm_colsum(d0, a["dZ2"], a["dc"], ws)
            dx2, dz2 = a["dHf"], a["dZ2"]
        elif cfg.final_ln and fused:
            B.mlm_combine_layernorm_bwd(d0, dhf_partials, a["X2"], rep["gf"], a["muf"], a["rstdf"], None, keep("dHf"),
                                        a["dX2"], a["dgf"], a["dbf"], a["dc"], ws)
            dx2 = a["dX2"]
        else:
            B.mlm_combine(d0, dhf_partials, None, None, a["dHf"])
            if cfg.final_ln:
                B.mlm_layernorm_bwd(d0, a["dHf"], a["X2"], rep["gf"], a["muf"], a["rstdf"], None, a["dX2"], a["dgf"],
                                    a["dbf"], ws)
                dx2 = a["dX2"]
            else:
                dx2 = a["dHf"]
            B.mlm_colsum(d0, dx2, a["dc"], ws)
        for r in self.shards:
            w, s = self.w[r], self.sh[r]
            if self.grouped_wgrads:
                B.mlm_mlp_shard_bwd_input(self.dims[r], dz2 if drop else dx2, w["A"], w["B"], s["g"], s["dg"], s["da"],
                                          s["du2_partial"], ws)
            else:
                B.mlm_mlp_shard_bwd(self.dims[r], dz2 if drop else dx2, a["U2"], w["A"], w["B"], s["g"], s["y"],
                                    s["dA"], s["da"], s["dB"], s["du2_partial"], ws)
        du2_partials = [self.sh[r]["du2_partial"] for r in self.shards]
        if drop:
            B.mlm_combine_layernorm_bwd_dropout(d0, du2_partials, a["X1"], rep["g2"], a["mu2"], a["rstd2"], dx2,
                                                self.drop["hidden1"], keep("dU2"), a["dX1"], a["dZ1"], a["dg2"],
                                                a["db2"], a["dbo"], ws)
            dz1 = a["dZ1"]
        elif fused:
            B.mlm_combine_layernorm_bwd(d0, du2_partials, a["X1"], rep["g2"], a["mu2"], a["rstd2"], dx2, keep("dU2"),
                                        a["dX1"], a["dg2"], a["db2"], a["dbo"], ws)
        else:
            B.mlm_combine(d0, du2_partials, None, None, a["dU2"])
            B.mlm_layernorm_bwd(d0, a["dU2"], a["X1"], rep["g2"], a["mu2"], a["rstd2"], dx2, a["dX1"], a["dg2"],
                                a["db2"], ws)
            B.mlm_colsum(d0, a["dX1"], a["dbo"], ws)
        for r in self.shards:
            w, s = self.w[r], self.sh[r]
            if self.grouped_wgrads:
                B.mlm_attn_shard_bwd_input(self.dims[r], dz1 if drop else a["dX1"], w["Wqkv"], w["Wo"], kl,
                                           self.drop["attn"][r] if drop else None, s["qkv"], s["ctx"], s["lse"],
                                           s["keep_bits"] if drop else None, s["dqkv"], s["dbqkv"], s["du_partial"], ws)
                B.mlm_layer_shard_wgrads(self.dims[r], a["U"], s["dqkv"], s["ctx"], dz1 if drop else a["dX1"], a["U2"],
                                         s["dg"], s["y"], dz2 if drop else dx2, s["dWqkv"], s["dWo"], s["dA"], s["dB"],
                                         ws)
            elif drop:
                B.mlm_attn_shard_bwd_dropout(self.dims[r], dz1, a["U"], w["Wqkv"], w["Wo"], kl, self.drop["attn"][r],
                                             s["qkv"], s["ctx"], s["lse"], s["keep_bits"], s["dWqkv"], s["dbqkv"],
                                             s["dWo"], s["du_partial"], ws)
            else:
                B.mlm_attn_shard_bwd(self.dims[r], a["dX1"], a["U"], w["Wqkv"], w["Wo"], kl, s["qkv"], s["ctx"],
                                     s["lse"], s["dWqkv"], s["dbqkv"], s["dWo"], s["du_partial"], ws)
        du_partials = [self.sh[r]["du_partial"] for r in self.shards]
        if fused:
            B.mlm_combine_layernorm_bwd(d0, du_partials, rep["X"], rep["g1"], a["mu1"], a["rstd1"], a["dX1"],
                                        keep("dU"), a["dX"], a["dg1"], a["db1"], None, ws)
        else:
            B.mlm_combine(d0, du_partials, None, None, a["dU"])
            B.mlm_layernorm_bwd(d0, a["dU"], rep["X"], rep["g1"], a["mu1"], a["rstd1"], a["dX1"], a["dX"], a["dg1"],
                                a["db1"], ws)
        self._dx2 = dx2
        if self.embed:
            # replicated part (dropout mask, position-embedding gradient), then each shard's columns of the tied dE
            B.mlm_embed_bwd_replicated(d0, a["dX"], self.drop.get("embed"), a["dZ0"], a["dpos"])
            for r in self.shards:
                B.mlm_embed_shard_bwd(self.dims[r], rep["ids"], self.sh[r]["perm"], a["dZ0"], self.sh[r]["dE"])

    # Activation recomputation (the paper checkpoints activations after every transformer layer, Section 4.2): only the
    # layer input X is kept; everything the layer's backward reads is produced again by re-running the layer's forward
    # calls (not the final layer norm / loss, which belong to the model's head) right before the backward.
    LAYER_ACTIVATIONS = ("U", "mu1", "rstd1", "X1", "U2", "mu2", "rstd2")
    SHARD_ACTIVATIONS = ("qkv", "ctx", "lse", "attn_partial", "g", "y", "mlp_partial")

    def drop_layer_activations(self):
        """Poison what a checkpointing run would not have kept (tests use it to prove the backward reads recomputed
        values only)."""
        for k in self.LAYER_ACTIVATIONS:
            self.act[k].fill_(float("nan"))
        for r in self.shards:
            for k in self.SHARD_ACTIVATIONS:
                self.sh[r][k].fill_(float("nan"))

    def recompute_layer(self):
        self._layer_forward()

    # ------------------------------------------------------------------ optimizer (this worker's parameters)
    def parameters(self):
        """(name, weight tensor, gradient tensor) of everything this object owns: the shards' weights and, once, the
        replicated layer-norm / bias parameters."""
        out = []
        for r in self.shards:
            w, s = self.w[r], self.sh[r]
            for k, gk in (("Wqkv", "dWqkv"), ("bqkv", "dbqkv"), ("Wo", "dWo"), ("A", "dA"), ("a", "da"), ("B", "dB"),
                          ("E", "dE")):
                out.append((f"{r}.{k}", w[k], s[gk]))
        rep, a = self.rep, self.act
        pairs = [("g1", "dg1"), ("b1", "db1"), ("g2", "dg2"), ("b2", "db2"), ("bo", "dbo"), ("c", "dc")]
        if self.cfg.final_ln:
            pairs += [("gf", "dgf"), ("bf", "dbf")]
        for k, gk in pairs:
            out.append((k, rep[k], a[gk]))
        return out

    def optimizer_step(self, step: int, lr: float, max_norm: float = 1.0, beta1: float = 0.9, beta2: float = 0.999,
                       eps: float = 1e-8, weight_decay: float = 0.01, other_sqnorm=None):
        """Global-norm clip + AdamW on every parameter (fp32 master weights and moments are created on first use)."""
        params = self.parameters()
        if not hasattr(self, "opt"):
            self.opt = {n: {"master": w.float().clone(), "m": torch.zeros_like(w, dtype=torch.float32),
                            "v": torch.zeros_like(w, dtype=torch.float32)} for n, w, _ in params}
            self.opt_ws = torch.empty(len(params) * 4096, device=self.dev, dtype=torch.uint8)
            self.sqnorm = torch.zeros(1, device=self.dev, dtype=torch.float32)
        B.mlm_grad_sqnorm(self.code, [g for _, _, g in params], other_sqnorm, self.sqnorm, self.opt_ws)
        st = [self.opt[n] for n, _, _ in params]
        B.mlm_adamw_step_multi(self.code, [g for _, _, g in params], [x["master"] for x in st], [x["m"] for x in st],
                               [x["v"] for x in st], [w for _, w, _ in params], [weight_decay] * len(params),
                               self.sqnorm, max_norm, lr, beta1, beta2, eps, step)

    def step(self, recompute: bool = False):
        self.forward()
        if recompute:
            self.recompute_layer()
        self.backward()

    # ------------------------------------------------------------------ results (host copies, fp64)
    def fetch(self) -> Dict[str, object]:
        torch.cuda.synchronize(self.dev)
        def cp(t):
            # buffers a mode never writes are copied too; their uninitialised bit patterns may be signalling NaNs
            with np.errstate(invalid="ignore"):
                return t.detach().float().cpu().numpy().astype(np.float64)
        skip = ()
        if self.fused and not self.store_combined:      # never written in this mode
            skip = ("dU2", "dU") + (("dHf",) if self.cfg.final_ln else ())
        out: Dict[str, object] = {k: cp(v) for k, v in self.act.items() if k not in skip}
        if getattr(self, "_dx2", None) is not None:
            out["dX2"] = cp(self._dx2)
        if getattr(self, "_hf", None) is not None:
            out["Hf"] = cp(self._hf)
        out["loss"] = float(self.act["loss"][0].item())
        out["wsum"] = float(self.act["loss"][1].item())
        out["shards"] = {r: {k: (cp(v) if v is not None else None) for k, v in self.sh[r].items()} for r in self.shards}
        return out
