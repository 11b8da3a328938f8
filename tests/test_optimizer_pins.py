"""CPU pins of the optimizer oracle (Section 4.2 of the paper: Adam with decoupled weight decay 0.01, global gradient
norm clipping at 1.0).  None of these re-types the oracle's formula: they are closed forms, a hand-worked example
and a library routine."""
import math

import numpy as np
import torch

from oracle import optimizer_oracle as OO


def test_first_step_moves_by_lr_against_the_sign():
    # t = 1: mh = g, vh = g^2, so the step is lr * g / (|g| + eps): with eps tiny every weight moves by lr
    rng = np.random.default_rng(0)
    w = rng.standard_normal(1000)
    g = rng.standard_normal(1000) * 10.0 ** rng.integers(-3, 3, 1000)
    w1, m1, v1 = OO.adamw_step(w, g, np.zeros(1000), np.zeros(1000), step=1, lr=1e-3, eps=1e-30, weight_decay=0.0)
    assert np.allclose(w1 - w, -1e-3 * np.sign(g), rtol=1e-12, atol=0)
    assert np.allclose(m1, 0.1 * g) and np.allclose(v1, 0.001 * g * g)


def test_zero_gradient_is_pure_decoupled_decay():
    # decoupled decay: with g = 0 the moments stay 0 and w shrinks geometrically, independent of Adam's scaling
    w = np.array([2.0, -3.0, 0.5])
    m = np.zeros(3); v = np.zeros(3)
    cur = w
    for t in range(1, 11):
        cur, m, v = OO.adamw_step(cur, np.zeros(3), m, v, step=t, lr=0.1, weight_decay=0.01)
    assert np.allclose(cur, w * (1 - 0.1 * 0.01) ** 10, rtol=1e-14)
    assert not m.any() and not v.any()


def test_decay_is_not_part_of_the_gradient():
    # L2-in-the-gradient would be rescaled by 1/sqrt(v): here doubling lambda changes the step by exactly lr*lambda*w
    w = np.array([4.0]); g = np.array([0.3])
    a, _, _ = OO.adamw_step(w, g, np.zeros(1), np.zeros(1), 1, lr=0.01, weight_decay=0.01)
    b, _, _ = OO.adamw_step(w, g, np.zeros(1), np.zeros(1), 1, lr=0.01, weight_decay=0.02)
    assert math.isclose(float(a[0] - b[0]), 0.01 * 0.01 * 4.0, rel_tol=1e-12)


def test_hand_worked_two_steps():
    # scalar, beta1 = 0.5, beta2 = 0.75, eps = 0, lr = 0.1, no decay, g1 = 2, g2 = -1, w0 = 1
    # t=1: m = 1, v = 1; mh = 1/(1-0.5) = 2, vh = 1/(1-0.75) = 4 -> w = 1 - 0.1 * 2/2 = 0.9
    # t=2: m = 0.5*1 + 0.5*(-1) = 0, v = 0.75*1 + 0.25*1 = 1 -> mh = 0 -> w stays 0.9
    w, m, v = OO.adamw_step(np.array([1.0]), np.array([2.0]), np.zeros(1), np.zeros(1), 1, 0.1, 0.5, 0.75, 0.0, 0.0)
    assert math.isclose(w[0], 0.9, rel_tol=1e-15) and m[0] == 1.0 and v[0] == 1.0
    w, m, v = OO.adamw_step(w, np.array([-1.0]), m, v, 2, 0.1, 0.5, 0.75, 0.0, 0.0)
    assert math.isclose(w[0], 0.9, rel_tol=1e-15) and m[0] == 0.0 and v[0] == 1.0


def test_clip_coefficient_bounds():
    assert OO.clip_coefficient(0.25, 1.0) == 1.0                     # norm 0.5 < 1: untouched
    c = OO.clip_coefficient(16.0, 1.0)                               # norm 4 -> scaled to (just under) 1
    assert math.isclose(c * 4.0, 1.0, rel_tol=1e-6) and c * 4.0 <= 1.0
    assert OO.clip_coefficient(1e12, 0.0) == 1.0                     # disabled
    g = [np.full(9, 2.0), np.full(16, -1.0)]                         # sqnorm 36 + 16 = 52
    assert OO.global_sqnorm(g) == 52.0


def test_global_norm_includes_other_workers():
    p = {"a": np.ones(4)}; g = {"a": np.full(4, 0.5)}                # own norm 1
    _, c_alone = OO.worker_step(p, g, {}, 1, 1e-3, max_norm=1.0)
    _, c_global = OO.worker_step(p, g, {}, 1, 1e-3, max_norm=1.0, other_workers_sqnorm=3.0)   # global norm 2
    assert math.isclose(c_alone, 1.0 / (1.0 + 1e-6), rel_tol=1e-12) and math.isclose(c_global, 0.5, rel_tol=1e-6)


def test_against_torch_adamw_fp64():
    rng = np.random.default_rng(3)
    w0 = rng.standard_normal((7, 5)); wt = torch.tensor(w0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.AdamW([wt], lr=3e-3, betas=(0.9, 0.999), eps=1e-8, weight_decay=0.01)
    w, m, v = w0.copy(), np.zeros_like(w0), np.zeros_like(w0)
    for t in range(1, 8):
        g = rng.standard_normal((7, 5)) * 3.0
        coef = OO.clip_coefficient(OO.global_sqnorm([g]), 1.0)
        wt.grad = torch.tensor(g)
        torch.nn.utils.clip_grad_norm_([wt], 1.0)
        opt.step()
        w, m, v = OO.adamw_step(w, g, m, v, t, 3e-3, clip=coef)
        assert np.allclose(w, wt.detach().numpy(), rtol=1e-12, atol=1e-14), t
