"""Shared helpers of the test-suite (no arithmetic of the method lives here)."""
import numpy as np

from oracle import layer_oracle as O
from oracle import rng_embed_oracle as R
from oracle import stack_oracle as S
from paper_1909_08053_amd import synth

TOL = {"fp32": 1e-4, "bf16": 2e-2}   # max-norm relative error bound per storage type (stated by the build's target)


def spec_of(cfg, **kw):
    d = dict(b=cfg.b, s=cfg.s, H=cfg.H, h=cfg.h, F=cfg.F, V=cfg.V, causal=cfg.causal,
             final_ln=cfg.final_ln, gelu_tanh=cfg.gelu_tanh, ln_eps=cfg.ln_eps)
    d.update(kw)
    return O.Spec(**d)


def relerr(got, ref):
    """max_i |got_i - ref_i| / max_i |ref_i|  (max-norm relative error of a whole tensor)."""
    got = np.asarray(got, np.float64).reshape(-1)
    ref = np.asarray(ref, np.float64).reshape(-1)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.all(np.isfinite(got)), "non-finite values in GPU result"
    den = max(float(np.max(np.abs(ref))), 1e-30)
    return float(np.max(np.abs(got - ref))) / den


# Per-block check next to the whole-tensor bound: a tensor is cut into blocks of BLOCK_ROWS x BLOCK_COLS (the last axis
# is the column axis), and every block whose own largest magnitude is at least BLOCK_MIN_FRAC of the tensor's must keep
# max|got - ref| / max|ref| OVER THE BLOCK within BLOCK_OWN_MULT x tol.  A wrong ragged edge tile of a weight gradient or
# a wrong padded row has a block-relative error of order 1 and fails this even where its values are small against the
# tensor's maximum; rounding noise, which scales with the tensor's typical magnitude, stays far below it.
BLOCK_ROWS, BLOCK_COLS = 64, 256
BLOCK_OWN_MULT = 4.0
BLOCK_MIN_FRAC = 0.02


def _block_max(a2, br, bc):
    r = np.maximum.reduceat(a2, np.arange(0, a2.shape[0], br), axis=0)
    return np.maximum.reduceat(r, np.arange(0, a2.shape[1], bc), axis=1)


def block_relerr(got, ref):
    """Largest block-relative error max_block(max|got - ref| / max|ref| over the block) over the blocks that carry
    signal, and the RMS-relative error of the whole tensor."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    g2 = got.reshape(1, -1) if got.ndim < 2 else got.reshape(-1, got.shape[-1])
    r2 = ref.reshape(g2.shape)
    diff = np.abs(g2 - r2)
    rms = float(np.sqrt(np.mean(diff * diff)) / max(np.sqrt(np.mean(r2 * r2)), 1e-30))
    eb = _block_max(diff, BLOCK_ROWS, BLOCK_COLS)
    mb = _block_max(np.abs(r2), BLOCK_ROWS, BLOCK_COLS)
    live = mb >= BLOCK_MIN_FRAC * max(float(mb.max()), 1e-30)
    worst = float(np.max(eb[live] / mb[live])) if np.any(live) else 0.0
    return worst, rms


def check(name, got, ref, tol, errors):
    """Gate: whole-tensor max-norm relative error <= tol.  Hardening: every block with signal within BLOCK_OWN_MULT x tol
    of its own maximum.  Logged in `errors`: (name, max-norm relative, worst block-relative, RMS-relative)."""
    e = relerr(got, ref)
    eb, rms = block_relerr(got, ref)
    errors.append((name, e, eb, rms))
    assert e <= tol, f"{name}: max-norm relative error {e:.3e} > {tol:.1e}"
    assert eb <= BLOCK_OWN_MULT * tol, (f"{name}: a {BLOCK_ROWS}x{BLOCK_COLS} block is off by {eb:.3e} of its own "
                                        f"maximum (> {BLOCK_OWN_MULT:g} x {tol:.1e}); whole-tensor error {e:.3e}")


def make_stack_model(cfg, n_layers, scale=8.0, dropout=None, seed=0, base_seed=5, offsets=None, round_bf16=False):
    """Unsharded parameters and inputs of an N-layer stack (synthetic, seeded); dropout = (p_attn, p_hidden) adds the
    keep masks, drawn by the oracle's generator at the site offsets `offsets(layer, site)`."""
    rng = np.random.default_rng(1000 + seed)
    layers = []
    first = None
    for l in range(n_layers):
        inp = synth.make_inputs(cfg, nonzero_bias=True, random_ln=True, seed=cfg.seed + 17 * l)
        first = first or inp
        P = {k: inp[k].astype(np.float64) for k in S.LAYER_PARAMS}
        for k in ("Wq", "Wk", "Wv", "Wo", "A", "B"):
            P[k] = P[k] * scale
        layers.append(P)
    model = {"layers": layers, "E": first["E"].astype(np.float64) * scale, "gf": first["gf"].astype(np.float64),
             "bf": first["bf"].astype(np.float64), "tgt": first["tgt"], "w": first["w"], "key_len": first["key_len"],
             "ids": rng.integers(0, cfg.V, size=(cfg.b, cfg.s)).astype(np.int32),
             "pos": rng.standard_normal((cfg.s, cfg.H)) * 0.5}
    model["ids"][0, :3] = model["ids"][0, 0]
    if round_bf16:
        for P in layers:
            for k in P:
                P[k] = synth.round_to_bf16(P[k].astype(np.float32)).astype(np.float64)
        for k in ("E", "gf", "bf", "pos"):
            model[k] = synth.round_to_bf16(np.asarray(model[k], np.float32)).astype(np.float64)
    if offsets is None:
        offsets = lambda l, site: 16 * l + {"attn": 1, "hidden1": 2, "hidden2": 3}.get(site, 4)
    if dropout:
        p_attn, p_hidden = dropout
        model["drop"] = {
            "layers": [R.layer_dropout_masks(cfg.b, cfg.s, cfg.H, cfg.h, cfg.p, base_seed,
                                             {k: offsets(l, k) for k in ("attn", "hidden1", "hidden2")}, p_attn, p_hidden)
                       for l in range(n_layers)],
            "keep0": R.keep_mask(R.stream_seed(base_seed, R.STREAM_REPLICATED, 0), offsets(n_layers, "embed"),
                                 (cfg.T, cfg.H), p_hidden),
            "p_hidden": float(np.float32(p_hidden))}
    return model


