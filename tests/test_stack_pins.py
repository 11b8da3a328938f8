"""CPU pins of oracle/stack_oracle.py (embedding + N layers + tied output embedding + loss)."""
import numpy as np
import torch
import torch.nn.functional as TF

from helpers import make_stack_model as make_model, spec_of
from oracle import layer_oracle as O
from oracle import rng_embed_oracle as R
from oracle import stack_oracle as S
from paper_1909_08053_amd import synth


def test_one_layer_stack_equals_the_single_layer_oracle():
    cfg = synth.small_config(b=2, s=12, H=32, h=4, F=128, V=48)
    model = make_model(cfg, 1)
    spec = spec_of(cfg)
    fw = S.forward(model, spec)
    g = S.backward(model, fw, spec)
    inp = dict(model["layers"][0])
    inp.update({k: model[k] for k in ("E", "gf", "bf", "tgt", "w", "key_len")})
    inp["X"] = fw["X0"].reshape(cfg.b, cfg.s, cfg.H)
    c = O.forward(inp, spec)
    gl = O.backward(inp, c, spec)
    assert c["loss"] == fw["loss"]
    assert np.array_equal(gl["dX"], g["dX_in"][0]) and np.array_equal(gl["dE"], g["E_out"])
    for k, gk in (("Wq", "dWq"), ("A", "dA"), ("bo", "dbo"), ("g1", "dg1"), ("c", "dc")):
        assert np.array_equal(g["layers"][0][k], gl[gk]), k
    assert np.array_equal(g["gf"], gl["dgf"])


def _torch_stack_loss(model, spec):
    tt = lambda v: torch.tensor(np.asarray(v, np.float64), requires_grad=True)
    L = [{k: tt(v) for k, v in P.items()} for P in model["layers"]]
    E, pos, gf, bf = tt(model["E"]), tt(model["pos"]), tt(model["gf"]), tt(model["bf"])
    b, s, H, h, d, T = spec.b, spec.s, spec.H, spec.h, spec.d, spec.T
    drop = model.get("drop")
    keepf = lambda x, k, p: x if k is None else x * torch.tensor(np.asarray(k)) / (1.0 - p)
    ph = drop["p_hidden"] if drop else 0.0
    X = keepf(TF.embedding(torch.tensor(model["ids"].reshape(-1).astype(np.int64)), E.T) + pos.repeat(b, 1),
              drop["keep0"] if drop else None, ph)
    heads = lambda z: z.reshape(b, s, h, d).permute(0, 2, 1, 3)
    mask = torch.tensor(np.stack([O.allowed_mask(s, spec.causal, int(k)) for k in model["key_len"]]))[:, None]
    for l, P in enumerate(L):
        dl = drop["layers"][l] if drop else {}
        U = TF.layer_norm(X, (H,), P["g1"], P["b1"], spec.ln_eps)
        Sc = heads(U @ P["Wq"] + P["bq"]) @ heads(U @ P["Wk"] + P["bk"]).transpose(-1, -2) / np.sqrt(d)
        Pm = torch.softmax(Sc.masked_fill(~mask, float("-inf")), dim=-1)
        Pm = keepf(Pm, dl.get("keep_attn"), dl.get("p_attn", 0.0))
        C = (Pm @ heads(U @ P["Wv"] + P["bv"])).permute(0, 2, 1, 3).reshape(T, H)
        X1 = X + keepf(C @ P["Wo"] + P["bo"], dl.get("keep1"), ph)
        U2 = TF.layer_norm(X1, (H,), P["g2"], P["b2"], spec.ln_eps)
        X = X1 + keepf(TF.gelu(U2 @ P["A"] + P["a"], approximate="tanh") @ P["B"] + P["c"], dl.get("keep2"), ph)
    Hf = TF.layer_norm(X, (H,), gf, bf, spec.ln_eps)
    w = np.asarray(model["w"]).reshape(T)
    tgt = torch.tensor(np.where(w > 0, np.asarray(model["tgt"]).reshape(T), -100).astype(np.int64))
    return TF.cross_entropy(Hf @ E, tgt, ignore_index=-100), L, E, pos, gf


def test_two_layer_stack_against_library_autograd():
    for dropout in (None, (0.25, 0.125)):
        cfg = synth.small_config(b=2, s=12, H=32, h=4, F=128, V=48, p=2)
        model = make_model(cfg, 2, dropout=dropout)
        spec = spec_of(cfg)
        fw = S.forward(model, spec)
        g = S.backward(model, fw, spec)
        loss, L, E, pos, gf = _torch_stack_loss(model, spec)
        assert abs(loss.item() - fw["loss"]) < 1e-12
        loss.backward()
        close = lambda a, t: np.max(np.abs(a - t.grad.numpy().reshape(a.shape))) <= 1e-10 * max(np.max(np.abs(a)), 1e-6)
        assert close(g["E"], E) and close(g["pos"], pos) and close(g["gf"], gf)
        for l in range(2):
            for k in S.LAYER_PARAMS:
                if k == "bk":
                    assert np.max(np.abs(g["layers"][l][k])) < 1e-14      # identically zero
                    continue
                assert close(g["layers"][l][k], L[l][k]), (l, k)


def test_two_layer_stack_finite_differences_of_the_tied_embedding():
    cfg = synth.small_config(b=1, s=8, H=16, h=2, F=64, V=32, p=1)
    model = make_model(cfg, 2, scale=10.0, dropout=(0.25, 0.25))
    spec = spec_of(cfg)
    g = S.backward(model, S.forward(model, spec), spec)
    rng = np.random.default_rng(0)
    step = 1e-6
    used = int(model["ids"][0, 0])
    for idx in [(int(rng.integers(0, cfg.H)), used)] + [tuple(rng.integers(0, n) for n in model["E"].shape) for _ in range(4)]:
        hi = dict(model); lo = dict(model)
        a = model["E"].copy(); a[idx] += step; hi["E"] = a
        a = model["E"].copy(); a[idx] -= step; lo["E"] = a
        fd = (S.loss_only(hi, spec) - S.loss_only(lo, spec)) / (2 * step)
        assert abs(fd - g["E"][idx]) <= 1e-6 * max(1.0, abs(g["E"][idx])) + 1e-8, (idx, fd, g["E"][idx])
