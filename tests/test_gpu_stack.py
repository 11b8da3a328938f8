"""GPU parity of the N-layer training step (embedding, layers with or without activation checkpointing, tied output
embedding, loss, backward) against the stack oracle, and of the optimizer step over all of its parameters."""
import numpy as np
import pytest
import torch

from helpers import TOL, check, make_stack_model, spec_of
from oracle import optimizer_oracle as OO
from oracle import stack_oracle as S
from paper_1909_08053_amd import binding as B
from paper_1909_08053_amd import synth
from paper_1909_08053_amd.stack import ModelShards

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
BASE_SEED = 0xABCDEF0123


def run_stack(cfg, n_layers, dropout, checkpoint, scale=3.0):
    M = ModelShards(cfg, n_layers, list(range(cfg.p)), DEV,
                    dropout=dict(p_attn=dropout[0], p_hidden=dropout[1], base_seed=BASE_SEED, step=7) if dropout else None,
                    checkpoint=checkpoint)
    model = make_stack_model(cfg, n_layers, scale=scale, dropout=dropout, base_seed=BASE_SEED, offsets=M.site_offset,
                             round_bf16=cfg.dtype == "bf16")
    spec = spec_of(cfg)
    fw = S.forward(model, spec)
    g = S.backward(model, fw, spec)
    M.load_host(model)
    M.step()
    out = M.fetch()
    tol = TOL[cfg.dtype]
    errs = []
    assert abs(out["loss"] - fw["loss"]) <= tol * abs(fw["loss"]), (out["loss"], fw["loss"])
    check("X0", out["X"][0], fw["X0"], tol, errs)
    for l in range(n_layers):
        check(f"X[{l + 1}]", out["X"][l + 1], fw["layer_caches"][l]["X2"], tol, errs)
    check("Hf", out["Hf"], fw["Hf"], tol, errs)
    check("ce", out["ce"], fw["ce"], tol, errs)
    check("dX0", out["dX0"], g["dX_in"][0], tol, errs)
    check("dgf", out["dgf"], g["gf"], tol, errs)
    check("dbf", out["dbf"], g["bf"], tol, errs)
    check("dpos", out["dpos"], g["pos"], tol, errs)
    Hl, Fl, Vl = cfg.H // cfg.p, cfg.F // cfg.p, cfg.V // cfg.p
    for r in range(cfg.p):
        check(f"dE[{r}] (tied)", out["dE"][r], g["E"][:, r * Vl:(r + 1) * Vl], tol, errs)
    for l in range(n_layers):
        gl = g["layers"][l]
        for k in ("g1", "b1", "bo", "g2", "b2", "c"):
            check(f"layer{l}.d{k}", out["layers"][l]["rep"]["d" + k], gl[k], tol, errs)
        for r in range(cfg.p):
            c = slice(r * Hl, (r + 1) * Hl)
            f = slice(r * Fl, (r + 1) * Fl)
            sh = out["layers"][l]["sh"][r]
            check(f"layer{l}.{r}.dWqkv", sh["dWqkv"], np.concatenate([gl["Wq"][:, c], gl["Wk"][:, c], gl["Wv"][:, c]], axis=1), tol, errs)
            check(f"layer{l}.{r}.dbqkv", sh["dbqkv"], np.concatenate([gl["bq"][c], gl["bk"][c], gl["bv"][c]]), tol, errs)
            check(f"layer{l}.{r}.dWo", sh["dWo"], gl["Wo"][c, :], tol, errs)
            check(f"layer{l}.{r}.dA", sh["dA"], gl["A"][:, f], tol, errs)
            check(f"layer{l}.{r}.da", sh["da"], gl["a"][f], tol, errs)
            check(f"layer{l}.{r}.dB", sh["dB"], gl["B"][f, :], tol, errs)
    return M, model, g, errs


@pytest.mark.parametrize("dtype,dropout,checkpoint", [("fp32", None, False), ("fp32", (0.25, 0.125), True),
                                                      ("bf16", None, True), ("bf16", (0.1, 0.1), True),
                                                      ("bf16", (0.1, 0.1), False)])
def test_three_layer_stack_all_shards(dtype, dropout, checkpoint):
    cfg = synth.small_config(dtype=dtype, b=2, s=136, H=128, h=2, F=512, V=384, p=2)
    _, _, _, errs = run_stack(cfg, 3, dropout, checkpoint)
    print("worst:", sorted(errs, key=lambda e: -e[1])[:4])


def test_checkpointed_gradients_are_bit_identical_to_stored_activations():
    cfg = synth.small_config(dtype="bf16", b=2, s=200, H=256, h=4, F=1024, V=1024, p=2)
    grads = []
    for checkpoint in (False, True):
        M = ModelShards(cfg, 3, [0, 1], DEV, dropout=dict(p_attn=0.1, p_hidden=0.1, base_seed=11, step=1),
                        checkpoint=checkpoint)
        M.load_random(seed=3)
        M.step()
        torch.cuda.synchronize()
        grads.append({n: g.clone() for n, _, g in M.parameters()})
    for n, v in grads[0].items():
        assert torch.isfinite(v.float()).all(), n
        assert torch.equal(v, grads[1][n]), f"{n}: checkpointing changed a gradient"


def test_stack_deferred_sums_are_bit_identical_to_sums_finished_in_each_call():
    """One finishing launch per layer (mlm_deferred_sums_begin / _flush around each layer's backward calls, the list's
    buffer reused from layer to layer) against one per call: every parameter gradient bit for bit."""
    cfg = synth.small_config(dtype="bf16", b=2, s=200, H=256, h=4, F=1024, V=1024, p=2)
    grads = []
    for deferred in (False, True):
        M = ModelShards(cfg, 3, [0, 1], DEV, dropout=dict(p_attn=0.1, p_hidden=0.1, base_seed=11, step=1),
                        deferred_sums=deferred)
        M.load_random(seed=3)
        M.step()
        torch.cuda.synchronize()
        grads.append({n: g.clone() for n, _, g in M.parameters()})
    for n, v in grads[0].items():
        assert torch.isfinite(v.float()).all(), n
        assert torch.equal(v, grads[1][n]), f"{n}: deferred sum differs"


def test_stack_optimizer_step_matches_oracle():
    """One AdamW step with global-norm clipping over all parameters of a 5-layer stack (more than 64 tensors: the
    squared norm is chained over two library calls), against the optimizer oracle fed the GPU's own gradients."""
    cfg = synth.small_config(dtype="bf16", b=2, s=72, H=128, h=2, F=512, V=256, p=2)
    M = ModelShards(cfg, 5, [0, 1], DEV, checkpoint=True)
    M.load_random(seed=5)
    M.step()
    torch.cuda.synchronize()
    params = M.parameters()
    assert len(params) > 64
    dn = lambda t: t.detach().float().cpu().numpy().astype(np.float64)
    w0 = {n: dn(w) for n, w, _ in params}
    gr = {n: dn(g) for n, _, g in params}
    f32 = lambda x: float(np.float32(x))
    hp = dict(lr=f32(1e-3), beta1=f32(0.9), beta2=f32(0.999), eps=f32(1e-8), weight_decay=f32(0.01))
    M.optimizer_step(1, lr=1e-3, max_norm=0.05)
    torch.cuda.synchronize()
    total = sum(float((g_ ** 2).sum()) for g_ in gr.values())
    assert abs(float(M.sqnorm[(len(params) - 1) // 64 & 1].item()) - total) <= 1e-4 * total
    coef = OO.clip_coefficient(total, 0.05)
    assert coef < 1.0
    for n, w, _ in params:
        ref = OO.adamw_step(w0[n], gr[n], np.zeros_like(w0[n]), np.zeros_like(w0[n]), 1, clip=coef, **hp)[0]
        got = dn(M.opt[n]["master"])
        assert np.max(np.abs(got - ref)) <= 1e-5 * max(np.max(np.abs(ref)), 1e-3), n
