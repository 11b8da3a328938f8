"""GPU parity: the HIP path (through the C-ABI binding) against the fp64 oracle, element by element."""
import numpy as np
import pytest
import torch

from helpers import TOL, check, relerr, spec_of
from oracle import layer_oracle as O
from paper_1909_08053_amd import binding as B
from paper_1909_08053_amd import synth
from paper_1909_08053_amd.pipeline import LayerShards

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _up(a, dt):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(DEV).to(dt).contiguous()


def _dn(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


# ------------------------------------------------------------------ GEMM building block
GEMM_SHAPES = [(256, 256, 256), (512, 384, 192), (264, 136, 72), (1000, 520, 328), (128, 1152, 3072 // 4),
               (8, 8, 8), (1032, 952, 640), (72, 7648, 136),
               # K an odd multiple of 32 (the last pair of k-slices overlaps the one before it): shortest, short, long
               (264, 200, 96), (520, 264, 160), (136, 520, 7648), (296, 392, 2016)]


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
@pytest.mark.parametrize("layout", [(0, 0), (0, 1), (1, 0)])
@pytest.mark.parametrize("shape", GEMM_SHAPES)
def test_gemm_layouts_and_ragged_tiles(dtype, layout, shape):
    M, N, K = shape
    ta, tb = layout
    rng = np.random.default_rng(M * 7 + N * 3 + K + ta * 2 + tb)
    A = rng.standard_normal((M, K)).astype(np.float32)
    Bm = (rng.standard_normal((K, N)) * 0.05).astype(np.float32)
    bias = rng.standard_normal(N).astype(np.float32)
    if dtype == "bf16":
        A, Bm, bias = synth.round_to_bf16(A), synth.round_to_bf16(Bm), synth.round_to_bf16(bias)
    dt = torch.bfloat16 if dtype == "bf16" else torch.float32
    code = B.MLM_BF16 if dtype == "bf16" else B.MLM_F32
    dA = _up(A.T if ta else A, dt)
    dB = _up(Bm.T if tb else Bm, dt)
    C = torch.full((M + 1, N), 7.0, device=DEV, dtype=dt)   # one canary row after the output
    use_bias = (M + N) % 16 == 0
    B.mlm_gemm(code, ta, tb, M, N, K, dA, dB, C, _up(bias, dt) if use_bias else None)
    torch.cuda.synchronize()
    ref = A.astype(np.float64) @ Bm.astype(np.float64) + (bias.astype(np.float64) if use_bias else 0.0)
    got = _dn(C)
    assert np.all(got[M] == 7.0), "write past the end of C"
    assert relerr(got[:M], ref) <= (TOL[dtype] if dtype == "fp32" else 1e-2)


# ------------------------------------------------------------------ replicated row kernels
@pytest.mark.parametrize("dtype,H", [("fp32", 256), ("bf16", 256), ("bf16", 3072), ("bf16", 1920), ("fp32", 136),
                                     ("bf16", 2560), ("bf16", 4096), ("fp32", 2048), ("bf16", 8)])   # incl. the widest / narrowest rows supported
def test_layernorm_combine_colsum(dtype, H):
    T = 2 * 37                     # ragged against the 4-rows-per-block / 32-rows-per-block groupings
    cfg_dims = B.make_dims(2, 37, H, 1, 4 * H, 8, 1, 0, B.MLM_BF16 if dtype == "bf16" else B.MLM_F32)
    dt = torch.bfloat16 if dtype == "bf16" else torch.float32
    rng = np.random.default_rng(H)
    rnd = (lambda a: synth.round_to_bf16(a)) if dtype == "bf16" else (lambda a: a.astype(np.float32))
    x = rnd(rng.standard_normal((T, H)).astype(np.float32) * 2 + 0.5)
    g = rnd((1 + 0.2 * rng.standard_normal(H)).astype(np.float32))
    be = rnd((0.1 * rng.standard_normal(H)).astype(np.float32))
    dy = rnd(rng.standard_normal((T, H)).astype(np.float32))
    res = rnd(rng.standard_normal((T, H)).astype(np.float32))
    tol = TOL[dtype]
    y = torch.empty(T, H, device=DEV, dtype=dt); mean = torch.empty(T, device=DEV); rstd = torch.empty(T, device=DEV)
    B.mlm_layernorm_fwd(cfg_dims, _up(x, dt), _up(g, dt), _up(be, dt), y, mean, rstd)
    yr, mur, rsr = O.layernorm_fwd(x, g.astype(np.float64), be.astype(np.float64), 1e-5)
    errs = []
    check("ln.y", _dn(y), yr, tol, errs); check("ln.mean", _dn(mean), mur, 1e-5 + 0 * tol, errs)
    check("ln.rstd", _dn(rstd), rsr, 1e-5, errs)
    ws = torch.empty(B.mlm_workspace_bytes(cfg_dims, B.WS_LAYERNORM_BWD), device=DEV, dtype=torch.uint8)
    dx = torch.empty(T, H, device=DEV, dtype=dt); dg = torch.empty(H, device=DEV, dtype=dt); db = torch.empty(H, device=DEV, dtype=dt)
    B.mlm_layernorm_bwd(cfg_dims, _up(dy, dt), _up(x, dt), _up(g, dt), mean, rstd, _up(res, dt), dx, dg, db, ws)
    dxr, dgr, dbr = O.layernorm_bwd(dy.astype(np.float64), x.astype(np.float64), g.astype(np.float64), mur, rsr)
    check("ln.dx", _dn(dx), dxr + res, tol, errs); check("ln.dgamma", _dn(dg), dgr, tol, errs)
    check("ln.dbeta", _dn(db), dbr, tol, errs)
    # combine: sum of partials + bias + residual
    parts = [rnd(rng.standard_normal((T, H)).astype(np.float32)) for _ in range(3)]
    out = torch.empty(T, H, device=DEV, dtype=dt)
    B.mlm_combine(cfg_dims, [_up(p_, dt) for p_ in parts], _up(be, dt), _up(res, dt), out)
    check("combine", _dn(out), sum(p_.astype(np.float64) for p_ in parts) + be + res, tol, errs)
    B.mlm_combine(cfg_dims, [_up(parts[0], dt)], None, None, out)
    assert np.array_equal(_dn(out), parts[0].astype(np.float64))
    # column sums
    ws2 = torch.empty(B.mlm_workspace_bytes(cfg_dims, B.WS_COLSUM), device=DEV, dtype=torch.uint8)
    cs = torch.empty(H, device=DEV, dtype=dt)
    B.mlm_colsum(cfg_dims, _up(dy, dt), cs, ws2)
    check("colsum", _dn(cs), dy.astype(np.float64).sum(0), tol, errs)
    # fused forms: bit-identical to combine followed by the layer norm (same arithmetic on the same rounded sums);
    # the fused column sum of dx adds in another order, so it is compared with the oracle's sum instead
    dparts = [_up(p_, dt) for p_ in parts]
    xo = torch.empty(T, H, device=DEV, dtype=dt); y2 = torch.empty_like(y); m2 = torch.empty_like(mean); r2 = torch.empty_like(rstd)
    B.mlm_combine_layernorm_fwd(cfg_dims, dparts, _up(be, dt), _up(res, dt), xo, _up(g, dt), _up(be, dt), y2, m2, r2)
    B.mlm_layernorm_fwd(cfg_dims, out.copy_(xo), _up(g, dt), _up(be, dt), y, mean, rstd)
    B.mlm_combine(cfg_dims, dparts, _up(be, dt), _up(res, dt), out)
    assert torch.equal(out, xo) and torch.equal(y, y2) and torch.equal(mean, m2) and torch.equal(rstd, r2)
    check("fused.y", _dn(y2), O.layernorm_fwd(_dn(xo), g.astype(np.float64), be.astype(np.float64), 1e-5)[0], tol, errs)
    dyo = torch.empty(T, H, device=DEV, dtype=dt); dx2 = torch.empty_like(dx); dg2 = torch.empty_like(dg); db2 = torch.empty_like(db)
    dcs = torch.empty(H, device=DEV, dtype=dt)
    B.mlm_combine_layernorm_bwd(cfg_dims, dparts, xo, _up(g, dt), m2, r2, _up(res, dt), dyo, dx2, dg2, db2, dcs, ws)
    B.mlm_combine(cfg_dims, dparts, None, None, out)
    B.mlm_layernorm_bwd(cfg_dims, out, xo, _up(g, dt), m2, r2, _up(res, dt), dx, dg, db, ws)
    assert torch.equal(out, dyo) and torch.equal(dx, dx2) and torch.equal(dg, dg2) and torch.equal(db, db2)
    check("fused.dx_colsum", _dn(dcs), _dn(dx2).sum(0), tol, errs)
    dx3 = torch.empty_like(dx)
    B.mlm_combine_layernorm_bwd(cfg_dims, dparts, xo, _up(g, dt), m2, r2, _up(res, dt), None, dx3, dg2, db2, None, ws)
    assert torch.equal(dx3, dx) and torch.equal(dg, dg2) and torch.equal(db, db2)


# ------------------------------------------------------------------ whole layer, all shards, every tensor
def run_layer_parity(cfg, nonzero_bias=True, random_ln=True, store_logits=True, scale_w=1.0, shards=None, fused=True,
                     store_combined=True):
    inp = synth.make_inputs(cfg, nonzero_bias=nonzero_bias, random_ln=random_ln)
    if scale_w != 1.0:
        for k in ("Wq", "Wk", "Wv", "Wo", "A", "B", "E"):
            inp[k] = inp[k] * np.float32(scale_w)
            if cfg.dtype == "bf16":
                inp[k] = synth.round_to_bf16(inp[k])
    spec = spec_of(cfg)
    ref = O.sharded_reference(inp, spec, cfg.p)
    shards = list(range(cfg.p)) if shards is None else shards
    assert shards == list(range(cfg.p)), "full-layer parity needs every shard"
    L = LayerShards(cfg, shards, DEV, store_logits=store_logits, fused=fused, store_combined=store_combined)
    L.load_host_inputs(inp)
    L.forward()
    fwd = L.fetch()
    L.backward()
    out = L.fetch()
    tol = TOL[cfg.dtype]
    errs = []
    # forward, replicated
    for k in ("U", "X1", "U2", "X2", "Hf", "ce", "mu1", "rstd1", "mu2", "rstd2"):
        check(k, fwd[k], ref[k], tol, errs)
    check("M+logS", fwd["M"] + np.log(fwd["S"]), ref["M"] + np.log(ref["S"]), tol, errs)
    assert abs(fwd["loss"] - ref["loss"]) <= tol * abs(ref["loss"]), (fwd["loss"], ref["loss"])
    assert fwd["wsum"] == float(np.asarray(inp["w"]).sum())
    tgt = inp["tgt"].reshape(-1)
    for i, r in enumerate(shards):
        g, rs = fwd["shards"][r], ref["shards"][r]
        for k in ("qkv", "ctx", "lse", "attn_partial", "g", "y", "mlp_partial"):
            check(f"shard{r}.{k}", g[k], rs[k], tol, errs)
        if store_logits:
            check(f"shard{r}.logits", g["logits"], rs["logits"], tol, errs)
        check(f"shard{r}.m+log s", fwd["m"][i] + np.log(fwd["s"][i]), rs["m"] + np.log(rs["s"]), tol, errs)
        check(f"shard{r}.t", fwd["t"][i], rs["t"], tol, errs)
        # integer work: the target-in-shard test is exact -> t is exactly 0 outside the shard's range
        assert np.array_equal(fwd["t"][i] == 0.0, ~rs["tgt_inside"] | (rs["t"] == 0.0))
        assert np.all(fwd["t"][i][~rs["tgt_inside"]] == 0.0)
    # backward, replicated
    for k in ("dHf", "dX2", "dU2", "dX1", "dU", "dX", "dgf", "dbf", "dg2", "db2", "dg1", "db1", "dc", "dbo"):
        if k in ("dgf", "dbf") and not cfg.final_ln:
            continue
        if k not in out:      # combined gradients are not stored in the benchmark's fused configuration
            assert k in ("dHf", "dU2", "dU") and fused and not store_combined
            continue
        check(k, out[k], ref[k], tol, errs)
    for r in shards:
        g, rs = out["shards"][r], ref["shards"][r]
        for k in ("dE", "dhf_partial", "dA", "da", "dB", "du2_partial", "dWqkv", "dbqkv", "dWo", "du_partial"):
            check(f"shard{r}.{k}", g[k], rs[k], tol, errs)
        if store_logits:
            check(f"shard{r}.dlogits", g["logits"], rs["dlogits"], tol, errs)
    return errs


def test_tiny_config_fp32_full_layer():
    errs = run_layer_parity(synth.CONFIGS["tiny"], nonzero_bias=False, random_ln=False)
    print("worst:", sorted(errs, key=lambda e: -e[1])[:5])


@pytest.mark.parametrize("variant", ["bias_ln", "bert", "no_final_ln_erf", "recompute_logits", "p4_d32"])
def test_small_fp32_variants(variant):
    kw = dict(b=2, s=80, H=128, h=4, F=512, V=256, p=2, dtype="fp32")
    store = True
    if variant == "bert":
        kw.update(causal=False, masked_lm=True)
    elif variant == "no_final_ln_erf":
        kw.update(final_ln=False, gelu_tanh=False)
    elif variant == "recompute_logits":
        store = False
    elif variant == "p4_d32":
        kw.update(p=4, s=72)
    run_layer_parity(synth.small_config(**kw), store_logits=store, scale_w=4.0)


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_unfused_entry_points_whole_layer(dtype):
    """The same layer through the separate combine / layer-norm / column-sum calls."""
    cfg = synth.small_config(dtype=dtype, b=2, s=96, H=128, h=2, F=512, V=512, p=2)
    run_layer_parity(cfg, fused=False, scale_w=3.0)


# ------------------------------------------------------------------ bf16 (MFMA) path: small layers spanning several tiles
BF16_CASES = {
    # name: (config overrides, store_logits, weight scale)
    "d64_causal": (dict(b=2, s=200, H=128, h=2, F=512, V=640, p=2), True, 3.0),
    "d96_causal": (dict(b=2, s=328, H=192, h=2, F=768, V=1088, p=2), True, 3.0),
    "d128_causal_p1": (dict(b=1, s=264, H=256, h=2, F=1024, V=520, p=1), True, 3.0),
    "d192_causal": (dict(b=2, s=200, H=384, h=2, F=1536, V=640, p=2), True, 3.0),
    # sequences shorter than one 64-key tile (the second wave group of the attention kernels gets no tile at all) and
    # of exactly one query block
    "d64_short_seq": (dict(b=3, s=40, H=128, h=2, F=512, V=256, p=2), True, 3.0),
    "d96_one_block_bert": (dict(b=2, s=128, H=192, h=2, F=768, V=512, p=1, causal=False, masked_lm=True), True, 3.0),
    "d192_bert": (dict(b=2, s=136, H=768, h=4, F=1536, V=512, p=2, causal=False, masked_lm=True), True, 3.0),
    "d64_bert": (dict(b=3, s=176, H=256, h=4, F=1024, V=960, p=4, causal=False, masked_lm=True), True, 3.0),
    "d96_bert_recompute": (dict(b=2, s=136, H=384, h=4, F=1536, V=512, p=2, causal=False, masked_lm=True), False, 3.0),
    "d64_noln_erf": (dict(b=2, s=128, H=128, h=2, F=512, V=256, p=1, final_ln=False, gelu_tanh=False), True, 3.0),
    # few tiles and a deep reduction: every GEMM's tail round is split along k, so the fix-up kernel runs each
    # epilogue (plain/bias store, bias+GeLU, GeLU', cross-entropy partials; dlogits in the recompute variant)
    "d128_ksplit": (dict(b=2, s=136, H=1024, h=8, F=4096, V=3080 * 2, p=2), True, 1.0),
    "d128_ksplit_recompute": (dict(b=2, s=136, H=1024, h=8, F=4096, V=3080 * 2, p=2), False, 1.0),
}


@pytest.mark.parametrize("case", sorted(BF16_CASES))
def test_small_bf16_layers(case):
    kw, store, scale = BF16_CASES[case]
    cfg = synth.small_config(name=case, dtype="bf16", **kw)
    errs = run_layer_parity(cfg, store_logits=store, scale_w=scale)
    print(case, "worst:", sorted(errs, key=lambda e: -e[1])[:4])


def test_attention_integer_work_bf16():
    """Causal row 0 sees only key 0: its context equals V[0] bit-exactly; padded keys get exactly zero weight,
    so changing them cannot change any output bit."""
    cfg = synth.small_config(dtype="bf16", b=2, s=160, H=128, h=2, F=512, V=256, p=1, causal=False, masked_lm=True)
    inp = synth.make_inputs(cfg, nonzero_bias=True)
    outs = []
    for trial in range(2):
        L = LayerShards(cfg, [0], DEV)
        x = dict(inp)
        if trial == 1:     # scramble X at padded key positions of batch 0 only beyond its key length
            X = inp["X"].copy()
            kl = int(inp["key_len"][0])
            X[0, kl:, :] = synth.round_to_bf16(np.random.default_rng(5).standard_normal(X[0, kl:, :].shape).astype(np.float32))
            x["X"] = X
        L.load_host_inputs(x)
        L.forward()
        outs.append(L.fetch())
    kl = int(inp["key_len"][0])
    ctx0 = outs[0]["shards"][0]["ctx"].reshape(cfg.b, cfg.s, -1)
    ctx1 = outs[1]["shards"][0]["ctx"].reshape(cfg.b, cfg.s, -1)
    assert np.array_equal(ctx0[0, :kl], ctx1[0, :kl]) and np.array_equal(ctx0[1], ctx1[1])
    cfg2 = synth.small_config(dtype="bf16", b=1, s=96, H=128, h=2, F=512, V=256, p=1)
    inp2 = synth.make_inputs(cfg2)
    L = LayerShards(cfg2, [0], DEV)
    L.load_host_inputs(inp2)
    L.forward()
    o = L.fetch()["shards"][0]
    v_row0 = o["qkv"][0, 2 * cfg2.H:]
    assert np.array_equal(o["ctx"][0], v_row0)


# ------------------------------------------------------------------ the benchmark workloads at full size
@pytest.mark.parametrize("name", ["gpt2_8p3b", "bert_3p9b", "gpt2_2p5b", "gpt2_1p2b"])
def test_full_size_configs_all_shards(name):
    """Every shard of the paper-shaped layers (Table 1 / Table 4 sizes), run sequentially on the one GPU through the
    same calls and launch configuration that bench.py times, combined in-device and compared tensor by tensor with
    the fp64 oracle of the sharded method (whose combined results equal the unsharded layer)."""
    cfg = synth.CONFIGS[name]
    errs = run_layer_parity(cfg, nonzero_bias=False, random_ln=False, store_combined=False)
    worst = sorted(errs, key=lambda e: -e[1])[:6]
    print(name, "worst max-norm relative errors:", worst)


@pytest.mark.parametrize("name", ["gpt2_8p3b_h16", "gpt2_8p3b_h24", "gpt2_1p2b_p8", "gpt2_4p2b"])
def test_full_size_sweep_configs_all_shards(name):
    """The shape-sweep workloads (head size 192 and 128 at the 8.3B shape; the 1.2B shape split 8 ways), all shards,
    same launch configuration as the sweep runner, against the fp64 oracle."""
    cfg = synth.SWEEP_CONFIGS[name]
    errs = run_layer_parity(cfg, nonzero_bias=False, random_ln=False, store_combined=False)
    print(name, "worst max-norm relative errors:", sorted(errs, key=lambda e: -e[1])[:6])


def test_full_size_step_is_bit_reproducible():
    """Nothing in the path uses atomics or an order that depends on timing: two steps over the same inputs at the
    benchmark's size and launch configuration give bit-identical results (a race between the asynchronous tile
    copies and the epilogue's staging memory would show here as run-to-run differences)."""
    cfg = synth.CONFIGS["gpt2_8p3b"]
    L = LayerShards(cfg, [0], DEV, store_logits=True)
    L.load_random(seed=cfg.seed)
    snaps = []
    for _ in range(3):
        L.step()
        torch.cuda.synchronize()
        s = L.sh[0]
        snaps.append({k: v.clone() for k, v in s.items() if v is not None and k != "logits"}
                     | {k: L.act[k].clone() for k in ("dX", "dU", "dX1", "dU2", "dX2", "dHf", "loss", "dg1", "db1")})
    for other in snaps[1:]:
        for k, v in snaps[0].items():
            assert torch.equal(v.view(torch.uint8), other[k].view(torch.uint8)), f"{k} differs between identical steps"


def test_activation_recomputation_matches_stored_activations():
    """Checkpointed variant: after the forward everything the layer saved is poisoned, the layer's forward calls are
    re-run from the layer input, and the backward then gives bit-identical gradients to the stored-activation path
    (which the tests above hold against the oracle)."""
    cfg = synth.small_config(dtype="bf16", b=2, s=200, H=256, h=4, F=1024, V=1024, p=2)
    inp = synth.make_inputs(cfg, nonzero_bias=True, random_ln=True)
    grads = []
    for recompute in (False, True):
        L = LayerShards(cfg, [0, 1], DEV)
        L.load_host_inputs(inp)
        L.forward()
        if recompute:
            L.drop_layer_activations()
            L.recompute_layer()
        L.backward()
        torch.cuda.synchronize()
        g = {k: L.act[k].clone() for k in ("dX", "dX1", "dX2", "dg1", "db1", "dg2", "db2", "dbo", "dc")}
        for r in (0, 1):
            for k in ("dWqkv", "dbqkv", "dWo", "dA", "da", "dB", "dE"):
                g[f"{r}.{k}"] = L.sh[r][k].clone()
        grads.append(g)
    for k, v in grads[0].items():
        assert torch.isfinite(v.float()).all(), k
        assert torch.equal(v, grads[1][k]), f"{k}: recomputed activations give a different gradient"


def _all_grads(L):
    g = {k: L.act[k].clone() for k in ("dX", "dX1", "dX2", "dg1", "db1", "dg2", "db2", "dgf", "dbf", "dbo", "dc")}
    for r in L.shards:
        for k in ("dWqkv", "dbqkv", "dWo", "dA", "da", "dB", "dE"):
            g[f"{r}.{k}"] = L.sh[r][k].clone()
    return g


@pytest.mark.parametrize("variant", ["fused_bf16", "fused_fp32", "unfused_bf16", "dropout_bf16", "eight_shards", "short_buffer"])
def test_deferred_sums_equal_the_sums_finished_inside_each_call(variant):
    """Between mlm_deferred_sums_begin and mlm_deferred_sums_flush the bias and layer-norm-weight gradients are summed
    by one launch at the end of the backward pass instead of one per call: every gradient must come out bit-identical.
    eight_shards records more reductions than a list holds (19 > 16) and short_buffer gives the list room for the first
    layer norm only, so both also cover the calls that finish on the spot while a list is open."""
    dtype = "fp32" if variant.endswith("fp32") else "bf16"
    p = 8 if variant == "eight_shards" else 2
    cfg = synth.small_config(dtype=dtype, b=2, s=200, H=512, h=8, F=1024, V=1024, p=p)
    inp = synth.make_inputs(cfg, nonzero_bias=True, random_ln=True)
    kw = {}
    if variant == "unfused_bf16":
        kw["fused"] = False
    if variant == "dropout_bf16":
        kw["dropout"] = dict(p_attn=0.1, p_hidden=0.1, base_seed=9, offsets={"attn": 1, "hidden1": 2, "hidden2": 3, "embed": 4})
    grads = []
    for deferred in (False, True):
        L = LayerShards(cfg, list(range(p)), DEV, deferred_sums=deferred, **kw)
        L.load_host_inputs(inp)
        if deferred and variant == "short_buffer":
            one_ln = ((cfg.T + 31) // 32) * 3 * cfg.H * 4
            L.defer_ws = torch.empty(one_ln + 256, device=DEV, dtype=torch.uint8)
        for k in ("dg1", "db1", "dg2", "db2", "dgf", "dbf", "dbo", "dc"):
            L.act[k].fill_(float("nan"))
        L.step()
        torch.cuda.synchronize()
        grads.append(_all_grads(L))
    for k, v in grads[0].items():
        assert torch.isfinite(v.float()).all(), k
        assert torch.equal(v.view(torch.uint8), grads[1][k].view(torch.uint8)), f"{k}: deferred sum differs"


def test_deferred_sums_leave_the_outputs_unwritten_until_the_flush():
    cfg = synth.small_config(dtype="bf16", b=2, s=136, H=256, h=4, F=1024, V=1024, p=2)
    d = B.make_dims(cfg.b, cfg.s, cfg.H, cfg.h, cfg.F, cfg.V, cfg.p, 0, B.MLM_BF16)
    g = torch.Generator(device="cpu").manual_seed(3)
    dy = torch.randn(cfg.T, cfg.H, generator=g).to(DEV, torch.bfloat16)
    ws = torch.empty(B.mlm_workspace_bytes(d, B.WS_COLSUM), device=DEV, dtype=torch.uint8)
    want = torch.empty(cfg.H, device=DEV, dtype=torch.bfloat16)
    B.mlm_colsum(d, dy, want, ws)
    got = torch.full((cfg.H,), float("nan"), device=DEV, dtype=torch.bfloat16)
    got2 = torch.full((cfg.H,), float("nan"), device=DEV, dtype=torch.bfloat16)
    buf = torch.empty(B.mlm_deferred_sums_bytes(d), device=DEV, dtype=torch.uint8)
    B.mlm_deferred_sums_begin(buf)
    try:
        with pytest.raises(B.MlmError) as ei:
            B.mlm_deferred_sums_begin(buf)              # one list per host thread
        assert ei.value.code == -7
        B.mlm_colsum(d, dy, got, ws)
        ws.zero_()                                      # the call's own workspace is free again
        B.mlm_colsum(d, dy * 2, got2, ws)
        torch.cuda.synchronize()
        assert torch.isnan(got.float()).all() and torch.isnan(got2.float()).all()
    finally:
        B.mlm_deferred_sums_flush()
    torch.cuda.synchronize()
    assert torch.equal(got, want)
    assert torch.isfinite(got2.float()).all() and not torch.equal(got2, want)
    with pytest.raises(B.MlmError) as ei:
        B.mlm_deferred_sums_flush()
    assert ei.value.code == -7


@pytest.mark.parametrize("dtype,shape", [("fp32", "ragged"), ("bf16", "ragged"), ("bf16", "aligned"), ("bf16", "aligned_bert")])
def test_grouped_weight_gradients_equal_the_separate_calls(dtype, shape):
    """Deferring the four weight gradients of a layer shard to one mlm_layer_shard_wgrads call (one grouped GEMM launch
    where the cost model picks it) changes no input gradient at all and the weight gradients only through the k-split
    summation order of the separate GEMMs (none when neither form splits)."""
    if shape == "ragged":        # T = 528 is no multiple of 64: the GEMMs run one by one (register-staged kernel)
        cfg = synth.small_config(dtype=dtype, b=2, s=264, H=256, h=2, F=1024, V=528, p=2)
    elif shape == "aligned":     # T = 512, 24 tiles in all: the cost model picks the single grouped launch
        cfg = synth.small_config(dtype=dtype, b=2, s=256, H=512, h=4, F=2048, V=512, p=2)
    else:
        cfg = synth.small_config(dtype=dtype, b=4, s=128, H=512, h=8, F=2048, V=512, p=2, causal=False, masked_lm=True)
    inp = synth.make_inputs(cfg, nonzero_bias=True, random_ln=True)
    res = []
    for grouped in (False, True):
        L = LayerShards(cfg, [0, 1], DEV, grouped_wgrads=grouped)
        L.load_host_inputs(inp)
        L.step()
        torch.cuda.synchronize()
        res.append((L, {k: L.act[k].clone() for k in ("dX", "dX1", "dX2", "dg1", "db1", "dbo", "dc")}))
    for k, v in res[0][1].items():
        assert torch.equal(v, res[1][1][k]), k
    ref = O.sharded_reference(inp, spec_of(cfg), cfg.p)
    for r in (0, 1):
        for k in ("dbqkv", "da", "du_partial", "du2_partial"):
            assert torch.equal(res[0][0].sh[r][k], res[1][0].sh[r][k]), (r, k)
        for k in ("dWqkv", "dWo", "dA", "dB"):
            assert relerr(_dn(res[1][0].sh[r][k]), ref["shards"][r][k]) <= TOL[dtype], (r, k)
            assert relerr(_dn(res[1][0].sh[r][k]), _dn(res[0][0].sh[r][k])) <= TOL[dtype] * 0.5, (r, k)


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_post_ln_arrangement_all_shards(dtype):
    """The original BERT arrangement (layer norm after each residual add; Section 5.3 of the paper compares it with
    the pre-LN one): same entry points in another order, against the oracle's post-LN definition."""
    cfg = synth.small_config(dtype=dtype, b=3, s=136, H=256, h=4, F=1024, V=512, p=2, causal=False, masked_lm=True)
    inp = synth.make_inputs(cfg, nonzero_bias=True, random_ln=True)
    for k in ("Wq", "Wk", "Wv", "Wo", "A", "B", "E"):
        inp[k] = inp[k] * np.float32(3.0)
        if dtype == "bf16":
            inp[k] = synth.round_to_bf16(inp[k])
    spec = spec_of(cfg)
    c = O.forward_post_ln(inp, spec)
    g = O.backward_post_ln(inp, c, spec)
    L = LayerShards(cfg, [0, 1], DEV, post_ln=True)
    L.load_host_inputs(inp)
    L.step()
    out = L.fetch()
    tol = TOL[dtype]
    errs = []
    assert abs(out["loss"] - c["loss"]) <= tol * abs(c["loss"])
    for k, ref in (("X1", c["S1"]), ("U2", c["X1"]), ("X2", c["S2"]), ("Hf", c["X2"]), ("ce", c["ce"]),
                   ("dX2", g["dS2"]), ("dX1", g["dS1"]), ("dX", g["dX"]), ("dg1", g["dg1"]), ("db1", g["db1"]),
                   ("dg2", g["dg2"]), ("db2", g["db2"]), ("dbo", g["dbo"]), ("dc", g["dc"])):
        check(k, out[k], ref, tol, errs)
    Hl, Fl, Vl = cfg.H // 2, cfg.F // 2, cfg.V // 2
    for r in (0, 1):
        cs, fs, vs = slice(r * Hl, (r + 1) * Hl), slice(r * Fl, (r + 1) * Fl), slice(r * Vl, (r + 1) * Vl)
        sh = out["shards"][r]
        check(f"{r}.dWqkv", sh["dWqkv"], np.concatenate([g["dWq"][:, cs], g["dWk"][:, cs], g["dWv"][:, cs]], axis=1), tol, errs)
        check(f"{r}.dWo", sh["dWo"], g["dWo"][cs, :], tol, errs)
        check(f"{r}.dA", sh["dA"], g["dA"][:, fs], tol, errs)
        check(f"{r}.dB", sh["dB"], g["dB"][fs, :], tol, errs)
        check(f"{r}.dE", sh["dE"], g["dE"][:, vs], tol, errs)
    print("worst:", sorted(errs, key=lambda e: -e[1])[:4])


def test_step_is_capturable_in_a_hip_graph_and_replays_bit_identically():
    """The library allocates nothing, creates no stream and never synchronises, so a whole forward + backward step can
    be captured into a HIP graph on the caller's stream.  Replays (with eager steps and synchronisations in between)
    must reproduce the eager result bit for bit, also after the inputs changed in place."""
    cfg = synth.small_config(dtype="bf16", b=2, s=256, H=512, h=4, F=2048, V=1024, p=2)
    L = LayerShards(cfg, [0, 1], DEV, dropout=dict(p_attn=0.1, p_hidden=0.1, base_seed=5,
                                                   offsets={"attn": 1, "hidden1": 2, "hidden2": 3, "embed": 4}), embed=True)
    L.load_random(seed=1)
    names = ("dX", "dX1", "dg1", "dbo", "dc", "dpos", "loss")
    snap = lambda: {k: L.act[k].clone() for k in names} | {f"{r}.{k}": L.sh[r][k].clone() for r in (0, 1)
                                                          for k in ("dWqkv", "dWo", "dA", "dB", "dE")}
    L.step()                                   # warm-up outside the capture (first-use function attributes)
    torch.cuda.synchronize()
    eager = snap()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            L.step()
    torch.cuda.current_stream().wait_stream(side)
    for it in range(3):
        for v in list(L.act.values()):
            if v.dtype == L.dt:
                v.fill_(float("nan"))           # poison everything the step writes
        graph.replay()
        torch.cuda.synchronize()
        got = snap()
        for k, v in eager.items():
            assert torch.equal(v.view(torch.uint8), got[k].view(torch.uint8)), (it, k)
        L.step()                                # eager work between replays
        torch.cuda.synchronize()
    # new token ids in place: the replay follows the data
    L.rep["ids"].copy_(torch.randint(0, cfg.V, (cfg.T,), device=DEV, dtype=torch.int32))
    L.step()
    torch.cuda.synchronize()
    eager2 = snap()
    graph.replay()
    torch.cuda.synchronize()
    got = snap()
    for k, v in eager2.items():
        assert torch.equal(v.view(torch.uint8), got[k].view(torch.uint8)), ("new ids", k)
    assert not torch.equal(eager["loss"], eager2["loss"])


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_degenerate_key_length_one(dtype):
    """A sequence whose only valid key is key 0 (key_len = 1): every query's probability row is exactly (1, 0, 0, ...),
    so its context equals V[0] bit for bit, and the whole layer still matches the oracle."""
    cfg = synth.small_config(dtype=dtype, b=2, s=136, H=128, h=2, F=512, V=256, p=1, causal=False, masked_lm=True)
    inp = synth.make_inputs(cfg, nonzero_bias=True, random_ln=True)
    inp["key_len"] = np.array([1, cfg.s], np.int32)
    inp["w"] = np.zeros((cfg.b, cfg.s), np.float32)
    inp["w"][0, 0] = 1.0
    inp["w"][1, ::7] = 1.0
    ref = O.sharded_reference(inp, spec_of(cfg), 1)
    L = LayerShards(cfg, [0], DEV)
    L.load_host_inputs(inp)
    L.step()
    out = L.fetch()
    sh = out["shards"][0]
    ctx = sh["ctx"].reshape(cfg.b, cfg.s, cfg.H)
    v0 = sh["qkv"].reshape(cfg.b, cfg.s, 3 * cfg.H)[0, 0, 2 * cfg.H:]
    assert np.array_equal(ctx[0], np.broadcast_to(v0, (cfg.s, cfg.H)))
    tol = TOL[dtype]
    errs = []
    assert abs(out["loss"] - ref["loss"]) <= tol * abs(ref["loss"])
    for k in ("X2", "dX", "dX1", "dg1", "dbo"):
        check(k, out[k], ref[k], tol, errs)
    for k in ("lse", "dWqkv", "dbqkv", "dWo", "dE"):
        check(k, sh[k], ref["shards"][0][k], tol, errs)


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_key_lengths_outside_the_contract_are_clamped(dtype):
    """key_len lives in device memory, so the kernels clamp it to [1, s] themselves: 0 and negative lengths behave as 1,
    lengths above s as s (the tile index arithmetic of the streamed kernels then never leaves the buffer)."""
    cfg = synth.small_config(dtype=dtype, b=4, s=200, H=128, h=2, F=512, V=256, p=1, causal=False, masked_lm=True)
    inp = synth.make_inputs(cfg, nonzero_bias=True, random_ln=True)
    inp["w"] = np.zeros((cfg.b, cfg.s), np.float32)
    inp["w"][:, ::5] = 1.0
    given = np.array([0, -3, cfg.s + 1, 10 * cfg.s], np.int32)
    inp["key_len"] = np.clip(given, 1, cfg.s).astype(np.int32)
    ref = O.sharded_reference(inp, spec_of(cfg), 1)
    inp["key_len"] = given
    L = LayerShards(cfg, [0], DEV)
    L.load_host_inputs(inp)
    L.step()
    out = L.fetch()
    tol = TOL[dtype]
    errs = []
    assert abs(out["loss"] - ref["loss"]) <= tol * abs(ref["loss"])
    for k in ("X2", "dX", "dX1"):
        check(k, out[k], ref[k], tol, errs)
    for k in ("ctx", "lse", "dWqkv", "dbqkv", "dWo"):
        check(k, out["shards"][0][k], ref["shards"][0][k], tol, errs)


# ------------------------------------------------------------------ loss merge over shards, called directly
@pytest.mark.parametrize("T,n_shards,weighted,misalign", [(74, 3, True, 0), (74, 1, False, 0), (8200, 3, True, 0),
                                                          (8200, 1, False, 0), (16388, 2, True, 0), (1024, 3, True, 1),
                                                          (4, 1, True, 0), (1, 2, False, 0)])
def test_loss_merge_over_shards_ragged_multi_pass_and_unaligned(T, n_shards, weighted, misalign):
    """mlm_vocab_ce_merge on per-shard (max, sum-exp, target-logit) triples built from the definition of the call's
    inputs, against the plain cross entropy of the full logits: token counts that are not a multiple of 4, that need
    more than one pass of the single block (> 8192), one shard (identity merge) and several, and buffers that are only
    4-byte aligned (the kernel must then leave its 16-byte path)."""
    p, Vl = 3, 8
    V = p * Vl
    dims = B.make_dims(1, T, 24, 3, 96, V, p, 0, B.MLM_F32)
    rng = np.random.default_rng(T + 7 * n_shards)
    Vn = n_shards * Vl                                     # the merge sees the first n_shards shards only
    L = (4.0 * rng.standard_normal((T, Vn))).astype(np.float32).astype(np.float64)
    L[0, :Vl] = -60.0                                      # a shard whose maximum is far below the row's maximum
    tgt = rng.integers(0, Vn, T)
    w = (rng.random(T) < 0.3).astype(np.float64) if weighted else np.ones(T)
    w[0] = 1.0
    m = np.stack([L[:, r * Vl:(r + 1) * Vl].max(1) for r in range(n_shards)])
    s = np.stack([np.exp(L[:, r * Vl:(r + 1) * Vl] - m[r][:, None]).sum(1) for r in range(n_shards)])
    t = np.stack([np.where((tgt >= r * Vl) & (tgt < (r + 1) * Vl), L[np.arange(T), tgt], 0.0) for r in range(n_shards)])
    loss_r, ce_r, mx_r, se_r = O.cross_entropy_fwd(L, tgt, w)

    def dev(a):                                            # optionally a view that starts 4 bytes into its buffer
        flat = torch.zeros(a.size + 4, device=DEV, dtype=torch.float32)
        v = flat[misalign:misalign + a.size]
        v.copy_(torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).reshape(-1))
        return v
    md, sd, td = dev(m), dev(s), dev(t)
    wd = dev(w) if weighted else None
    ce, M, S = dev(np.zeros(T)), dev(np.zeros(T)), dev(np.zeros(T))
    loss = torch.zeros(2, device=DEV, dtype=torch.float32)
    B.mlm_vocab_ce_merge(dims, md, sd, td, n_shards, wd, ce, M, S, loss)
    errs = []
    check("merge.ce", _dn(ce), ce_r, 1e-5, errs)
    check("merge.M", _dn(M), mx_r, 1e-6, errs)
    check("merge.S", _dn(S), se_r, 1e-5, errs)
    assert abs(float(loss[0]) - loss_r) <= 1e-5 * abs(loss_r)
    assert float(loss[1]) == w.sum()                       # the weight count is integer work: exact
