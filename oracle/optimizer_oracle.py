"""fp64 CPU oracle for one model-parallel worker's optimizer step.

TEST INFRASTRUCTURE ONLY.  This file is the checker, not the product: only ``tests/``,
``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may import it.  It shares
no code with the HIP path and imports nothing from it.

What it computes.  Section 4.2 of the paper ("Training Optimization and Hyperparameters"): Adam with
decoupled weight decay (lambda = 0.01), global gradient-norm clipping at 1.0, mixed precision (the
weights used by the GEMMs are a low-precision copy of fp32 master weights).  Section 3: every
model-parallel worker optimises its own parameters, no parameter communication -- the only number
that crosses workers is the squared gradient norm (the clipping is GLOBAL).

The update is the published AdamW algorithm (decoupled weight decay: the decay term multiplies the
weight directly and is not part of the gradient), written out step by step:
    g   <- g * min(1, max_norm / (||g||_global + 1e-6))
    m   <- beta1 m + (1 - beta1) g
    v   <- beta2 v + (1 - beta2) g^2
    mh  = m / (1 - beta1^t),  vh = v / (1 - beta2^t)
    w   <- w - lr (mh / (sqrt(vh) + eps) + lambda w)
Readings where the paper is silent (also listed in the design notes): beta1 = 0.9, beta2 = 0.999,
eps = 1e-8 as defaults; bias correction on; the clip coefficient uses norm + 1e-6 in the
denominator and is capped at 1; the decay uses the weight BEFORE the step; every tensor is decayed
unless the caller passes lambda = 0 for it.

Pins (tests/test_optimizer_pins.py, CPU): closed forms (first step with eps -> 0 moves every weight
by exactly lr against the gradient's sign; zero gradient leaves pure exponential decay
w (1 - lr lambda)^t; clipping leaves small gradients untouched and scales large ones to the bound),
a two-step scalar example worked by hand, and torch.optim.AdamW in float64 as a second opinion over
several steps.
"""
from __future__ import annotations

import math
from typing import Dict, Iterable, Tuple

import numpy as np

F64 = np.float64


def global_sqnorm(grads: Iterable[np.ndarray]) -> float:
    """Sum of squares over every gradient tensor of the worker (the per-worker term of the global norm)."""
    return float(sum(np.sum(np.asarray(g, F64) ** 2) for g in grads))


def clip_coefficient(total_sqnorm: float, max_norm: float) -> float:
    """min(1, max_norm / (norm + 1e-6)); max_norm <= 0 disables clipping."""
    if max_norm <= 0.0:
        return 1.0
    return min(1.0, max_norm / (math.sqrt(total_sqnorm) + 1e-6))


def adamw_step(w: np.ndarray, g: np.ndarray, m: np.ndarray, v: np.ndarray, step: int, lr: float, beta1: float = 0.9,
               beta2: float = 0.999, eps: float = 1e-8, weight_decay: float = 0.01,
               clip: float = 1.0) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """One AdamW update of one tensor; `step` is 1-based, `clip` the already computed global clip coefficient.
    Returns the new (w, m, v) in float64."""
    w, g, m, v = (np.asarray(a, F64) for a in (w, g, m, v))
    g = g * clip
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    mh = m / (1.0 - beta1 ** step)
    vh = v / (1.0 - beta2 ** step)
    w = w - lr * (mh / (np.sqrt(vh) + eps) + weight_decay * w)
    return w, m, v


def worker_step(params: Dict[str, np.ndarray], grads: Dict[str, np.ndarray], state: Dict[str, Dict[str, np.ndarray]],
                step: int, lr: float, max_norm: float = 1.0, other_workers_sqnorm: float = 0.0, **hyper):
    """Clip by the GLOBAL norm (this worker's squared norm plus the other workers') and update every tensor."""
    coef = clip_coefficient(global_sqnorm(grads.values()) + other_workers_sqnorm, max_norm)
    out = {}
    for k in params:
        st = state.setdefault(k, {"m": np.zeros_like(params[k], F64), "v": np.zeros_like(params[k], F64)})
        out[k], st["m"], st["v"] = adamw_step(params[k], grads[k], st["m"], st["v"], step, lr, clip=coef, **hyper)
    return out, coef
