"""Shared helpers of the test-suite (no arithmetic of the method lives here)."""
import numpy as np

from oracle import layer_oracle as O

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


def check(name, got, ref, tol, errors):
    e = relerr(got, ref)
    errors.append((name, e))
    assert e <= tol, f"{name}: max-norm relative error {e:.3e} > {tol:.1e}"
