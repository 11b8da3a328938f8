"""GPU parity of the optimizer entry points (mlm_grad_sqnorm, mlm_adamw_step) against the fp64 oracle, through the
C-ABI.  Floating point: max-norm relative error <= 1e-5 on the fp32 state (the path's stated fp32 bar is 1e-4); the
low-precision weight copy is byte work: it must equal the rounded master bit for bit."""
import numpy as np
import pytest
import torch

from helpers import relerr
from oracle import optimizer_oracle as OO
from paper_1909_08053_amd import binding as B
from paper_1909_08053_amd import synth
from paper_1909_08053_amd.pipeline import LayerShards

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
# the C-ABI takes the hyper-parameters as floats: the oracle is given the same (float32-representable) values
F = lambda x: float(np.float32(x))
LR, B1, B2, EPS, WD = F(3e-3), F(0.9), F(0.999), F(1e-8), F(0.01)


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
@pytest.mark.parametrize("clipped", [False, True])
def test_adamw_three_steps_against_oracle(dtype, clipped):
    rng = np.random.default_rng(17 + clipped)
    code = B.MLM_BF16 if dtype == "bf16" else B.MLM_F32
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    shapes = [(8,), (1152,), (384, 3072), (1000, 1016)]            # one vector .. 1 M elements, ragged against 256-thread blocks
    gscale = 5.0 if clipped else 1e-4                               # global norm far above / far below the bound of 1
    w0 = [rng.standard_normal(s).astype(np.float32) * 0.02 for s in shapes]
    if dtype == "bf16":
        w0 = [synth.round_to_bf16(w) for w in w0]
    dev_w = [torch.from_numpy(w).to(DEV).to(tdt).contiguous() for w in w0]
    master = [torch.from_numpy(w).to(DEV).clone() for w in w0]
    m = [torch.zeros_like(x) for x in master]
    v = [torch.zeros_like(x) for x in master]
    ow, om, ov = [w.astype(np.float64) for w in w0], [np.zeros(s) for s in shapes], [np.zeros(s) for s in shapes]
    ws = torch.empty(len(shapes) * 4096, device=DEV, dtype=torch.uint8)
    sq = torch.zeros(1, device=DEV)
    other = torch.tensor([0.75], device=DEV)
    for step in range(1, 4):
        g = [rng.standard_normal(s).astype(np.float32) * gscale for s in shapes]
        if dtype == "bf16":
            g = [synth.round_to_bf16(x) for x in g]
        dev_g = [torch.from_numpy(x).to(DEV).to(tdt).contiguous() for x in g]
        B.mlm_grad_sqnorm(code, dev_g, other, sq, ws)
        ref_sq = OO.global_sqnorm(g) + 0.75
        assert abs(float(sq.item()) - ref_sq) <= 1e-5 * ref_sq
        coef = OO.clip_coefficient(ref_sq, 1.0)
        assert (coef < 1.0) == clipped
        for i in range(len(shapes)):
            B.mlm_adamw_step(code, dev_g[i], master[i], m[i], v[i], dev_w[i], sq, 1.0, LR, B1, B2, EPS, WD, step)
            ow[i], om[i], ov[i] = OO.adamw_step(ow[i], g[i], om[i], ov[i], step, LR, B1, B2, EPS, WD, clip=coef)
        torch.cuda.synchronize()
        for i in range(len(shapes)):
            assert relerr(master[i].cpu().numpy(), ow[i]) <= 1e-5, (step, i)
            assert relerr(m[i].cpu().numpy(), om[i]) <= 1e-5 and relerr(v[i].cpu().numpy(), ov[i]) <= 1e-5, (step, i)
            # the weight the GEMMs read is the master rounded once to the storage type: bit-exact
            assert torch.equal(dev_w[i], master[i].to(tdt))
    # no clipping requested: total_sqnorm may be NULL and the gradient is used as is
    mm, vv = torch.zeros_like(master[0]), torch.zeros_like(master[0])
    w_before = master[0].clone()
    B.mlm_adamw_step(code, dev_g[0], master[0], mm, vv, None, None, 0.0, F(1e-3), B1, B2, EPS, 0.0, 1)
    exp, _, _ = OO.adamw_step(w_before.cpu().numpy(), g[0], np.zeros(8), np.zeros(8), 1, F(1e-3), B1, B2, EPS, 0.0, clip=1.0)
    assert relerr(master[0].cpu().numpy(), exp) <= 1e-5


def test_multi_tensor_launch_matches_single_launches():
    """The one-launch form gives bit-identical state to per-tensor calls (same arithmetic per element), with a
    different decay per tensor and one tensor without a low-precision copy."""
    rng = np.random.default_rng(5)
    shapes = [(8,), (3072,), (384, 1152), (40,) , (257, 8)] * 8          # 40 tensors: two groups of launches
    mk = lambda: [torch.from_numpy(rng.standard_normal(s).astype(np.float32)).to(DEV) for s in shapes]
    g = [x.to(torch.bfloat16) for x in mk()]
    wd = [0.01 if len(s) == 2 else 0.0 for s in shapes]
    state = []
    for variant in range(2):
        rs = np.random.default_rng(9)
        master = [torch.from_numpy(rs.standard_normal(s).astype(np.float32)).to(DEV) for s in shapes]
        m = [torch.zeros_like(x) for x in master]; v = [torch.zeros_like(x) for x in master]
        w = [x.to(torch.bfloat16) for x in master]
        w[3] = None
        sq = torch.tensor([4.0], device=DEV)
        for step in (1, 2):
            if variant == 0:
                for i in range(len(shapes)):
                    B.mlm_adamw_step(B.MLM_BF16, g[i], master[i], m[i], v[i], w[i], sq, 1.0, LR, B1, B2, EPS, F(wd[i]), step)
            else:
                B.mlm_adamw_step_multi(B.MLM_BF16, g, master, m, v, w, wd, sq, 1.0, LR, B1, B2, EPS, step)
        torch.cuda.synchronize()
        state.append((master, m, v, w))
    for a, b in zip(state[0], state[1]):
        for x, y in zip(a, b):
            assert (x is None and y is None) or torch.equal(x, y)


def test_argument_checks():
    t = torch.zeros(16, device=DEV)
    with pytest.raises(B.MlmError):
        B.mlm_adamw_step(B.MLM_F32, t[:6], t, t, t, None, None, 0.0, 1e-3, 0.9, 0.999, 1e-8, 0.0, 1)    # count % 4
    with pytest.raises(B.MlmError):
        B.mlm_adamw_step(B.MLM_F32, t, t, t, t, None, None, 1.0, 1e-3, 0.9, 0.999, 1e-8, 0.0, 1)        # clip without a norm
    with pytest.raises(B.MlmError):
        B.mlm_adamw_step(B.MLM_F32, t, t, t, t, None, None, 0.0, 1e-3, 0.9, 0.999, 1e-8, 0.0, 0)        # step is 1-based


def test_training_iterations_reduce_the_loss():
    """forward + backward + optimizer step, all shards, a few iterations on fixed synthetic data: every parameter
    moves, the state stays finite and the loss goes down (a property check of the whole iteration; the arithmetic of
    each part is held against the oracle elsewhere)."""
    cfg = synth.small_config(dtype="bf16", b=2, s=64, H=128, h=2, F=512, V=512, p=2)
    L = LayerShards(cfg, [0, 1], DEV)
    L.load_host_inputs(synth.make_inputs(cfg, nonzero_bias=True, random_ln=True))
    before = {n: w.clone() for n, w, _ in L.parameters()}
    losses = []
    for it in range(1, 7):
        L.step()
        losses.append(float(L.act["loss"][0].item()))
        L.optimizer_step(it, lr=2e-3)
    torch.cuda.synchronize()
    assert all(np.isfinite(losses)) and losses[-1] < losses[0] - 0.05, losses
    for n, w, _ in L.parameters():
        assert torch.isfinite(w.float()).all() and not torch.equal(w, before[n]), n
