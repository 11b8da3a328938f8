"""GPU parity of the dropout (two random streams) and input-embedding entry points against the oracle: keep decisions
and the sort are integer work (bit-exact), everything else within the storage type's tolerance."""
import numpy as np
import pytest
import torch

from helpers import TOL, check, relerr, spec_of
from oracle import layer_oracle as O
from oracle import rng_embed_oracle as R
from paper_1909_08053_amd import binding as B
from paper_1909_08053_amd import synth
from paper_1909_08053_amd.pipeline import LayerShards

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
OFFSETS = {"attn": 0x0000000500000011, "hidden1": 12, "hidden2": 0xFFFFFFFF00000003, "embed": 14}
BASE_SEED = 0x1234567FFFFFFFFE          # + 1 + r carries into the upper key word for r >= 1


def _up(a, dt):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(DEV).to(dt).contiguous()


def _dn(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def _tdt(dtype):
    return (torch.bfloat16, B.MLM_BF16) if dtype == "bf16" else (torch.float32, B.MLM_F32)


# ------------------------------------------------------------------ the generator itself, through the combine kernel
@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("p_drop", [0.1, 0.5, 0.999])
def test_residual_dropout_mask_is_bit_exact(dtype, p_drop):
    dt, code = _tdt(dtype)
    b, s, H = 3, 37, 264                       # ragged against the 256-thread blocks
    T = b * s
    dims = B.make_dims(b, s, H, 1, 4 * H, 8, 1, 0, code)
    seed, off = B.mlm_rng_stream_seed(BASE_SEED, B.STREAM_MODEL_PARALLEL, 3), OFFSETS["hidden2"]
    assert seed == R.stream_seed(BASE_SEED, R.STREAM_MODEL_PARALLEL, 3)
    ones = torch.ones(T, H, device=DEV, dtype=dt)
    out = torch.empty_like(ones)
    B.mlm_combine_dropout(dims, [ones], None, 1, B.make_dropout(p_drop, seed, off), None, out)
    got = _dn(out)
    keep = R.keep_mask(seed, off, (T, H), p_drop)
    assert np.array_equal(got != 0.0, keep), "keep decisions differ from the oracle's generator"
    scale = 1.0 / (1.0 - float(np.float32(p_drop)))
    assert relerr(got[keep], np.full(int(keep.sum()), scale)) <= TOL[dtype]
    # with bias rows, residual and several partials: residual + dropout(sum + bias[t mod rows])
    rng = np.random.default_rng(7)
    rnd = synth.round_to_bf16 if dtype == "bf16" else (lambda a: a.astype(np.float32))
    parts = [rnd(rng.standard_normal((T, H)).astype(np.float32)) for _ in range(3)]
    pos = rnd(rng.standard_normal((s, H)).astype(np.float32))
    res = rnd(rng.standard_normal((T, H)).astype(np.float32))
    B.mlm_combine_dropout(dims, [_up(q, dt) for q in parts], _up(pos, dt), s, B.make_dropout(p_drop, seed, off),
                          _up(res, dt), out)
    z = sum(q.astype(np.float64) for q in parts) + np.tile(pos.astype(np.float64), (b, 1))
    assert relerr(_dn(out), res + np.where(keep, z, 0.0) * scale) <= TOL[dtype]
    # p = 0 and drop = NULL are the plain combine
    o2 = torch.empty_like(out)
    B.mlm_combine_dropout(dims, [_up(parts[0], dt)], None, 1, B.make_dropout(0.0, seed, off), None, out)
    B.mlm_combine_dropout(dims, [_up(parts[0], dt)], None, 1, None, None, o2)
    assert torch.equal(out, o2) and np.array_equal(_dn(out), parts[0].astype(np.float64))


def test_dropout_argument_validation():
    dims = B.make_dims(2, 30, 64, 2, 256, 64, 1, 0, B.MLM_F32)        # s = 30: not a multiple of 4
    x = torch.zeros(60, 64, device=DEV)
    with pytest.raises(B.MlmError) as ei:
        B.mlm_combine_dropout(dims, [x], None, 1, B.make_dropout(1.0, 1, 1), None, x)
    assert ei.value.code == -2
    with pytest.raises(B.MlmError) as ei:
        B.mlm_combine_dropout(dims, [x], None, 1, B.make_dropout(-0.1, 1, 1), None, x)
    assert ei.value.code == -2
    L = LayerShards(synth.small_config(b=2, s=30, H=64, h=2, F=256, V=64, p=1), [0], DEV,
                    dropout=dict(p_attn=0.1, p_hidden=0.1, base_seed=1, offsets=OFFSETS))
    L.load_random()
    with pytest.raises(B.MlmError) as ei:
        L.forward()
    assert ei.value.code == -5                                       # attention dropout needs s % 4 == 0


# ------------------------------------------------------------------ whole layer with dropout, every tensor
def run_dropout_layer(cfg, p_attn, p_hidden, scale_w=3.0, embed=False):
    inp = synth.make_inputs(cfg, nonzero_bias=True, random_ln=True)
    for k in ("Wq", "Wk", "Wv", "Wo", "A", "B", "E"):
        inp[k] = inp[k] * np.float32(scale_w)
        if cfg.dtype == "bf16":
            inp[k] = synth.round_to_bf16(inp[k])
    spec = spec_of(cfg)
    inp["drop"] = R.layer_dropout_masks(cfg.b, cfg.s, cfg.H, cfg.h, cfg.p, BASE_SEED, OFFSETS, p_attn, p_hidden)
    keep0 = None
    if embed:
        rng = np.random.default_rng(cfg.seed + 100)
        inp["ids"] = rng.integers(0, cfg.V, size=(cfg.b, cfg.s)).astype(np.int32)
        inp["ids"][0, : min(5, cfg.s)] = inp["ids"][0, 0]            # repeated ids: runs in the backward pass
        pos = (rng.standard_normal((cfg.s, cfg.H)) * 0.5).astype(np.float32)
        inp["pos"] = synth.round_to_bf16(pos) if cfg.dtype == "bf16" else pos
        keep0 = R.keep_mask(R.stream_seed(BASE_SEED, R.STREAM_REPLICATED, 0), OFFSETS["embed"], (cfg.T, cfg.H), p_hidden)
        p32 = float(np.float32(p_hidden))
        x0 = R.embedding_fwd(inp["E"], inp["ids"], inp["pos"], keep0, p32)
        # the layer's input as the GPU holds it: rounded to the storage type
        inp["X"] = (synth.round_to_bf16(x0.astype(np.float32)) if cfg.dtype == "bf16" else x0.astype(np.float32)
                    ).reshape(cfg.b, cfg.s, cfg.H)
    ref = O.sharded_reference(inp, spec, cfg.p)
    L = LayerShards(cfg, list(range(cfg.p)), DEV, store_combined=True, embed=embed,
                    dropout=dict(p_attn=p_attn, p_hidden=p_hidden, base_seed=BASE_SEED, offsets=OFFSETS))
    L.load_host_inputs(inp)
    L.step()
    out = L.fetch()
    tol = TOL[cfg.dtype]
    errs = []
    if embed:
        check("X0", _dn(L.rep["X"]), x0, tol, errs)
    for k in ("U", "X1", "U2", "X2", "Hf", "ce"):
        check(k, out[k], ref[k], tol, errs)
    assert abs(out["loss"] - ref["loss"]) <= tol * abs(ref["loss"])
    for k in ("dHf", "dX2", "dZ2", "dU2", "dX1", "dZ1", "dU", "dX", "dgf", "dbf", "dg2", "db2", "dg1", "db1", "dc", "dbo"):
        if k in ("dgf", "dbf", "dHf") and not cfg.final_ln:
            continue
        check(k, out[k], ref[k], tol, errs)
    hl, pitch = cfg.h // cfg.p, 4 * ((cfg.s + 127) // 128)
    for r in range(cfg.p):
        g, rs = out["shards"][r], ref["shards"][r]
        # keep bits of every allowed (query, key) pair equal the oracle's mask of worker r: integer work, exact
        words = L.sh[r]["keep_bits"].cpu().numpy().view(np.uint32).reshape(cfg.b, hl, cfg.s, pitch)
        j = np.arange(cfg.s)
        bits = ((words[..., j // 32] >> (j % 32).astype(np.uint32)) & 1).astype(bool)
        want = inp["drop"]["keep_attn"][:, r * hl:(r + 1) * hl]
        for bi in range(cfg.b):
            ok = O.allowed_mask(cfg.s, cfg.causal, int(inp["key_len"][bi]))
            assert np.array_equal(bits[bi][:, ok], want[bi][:, ok]), f"shard {r}: attention keep bits"
        for k in ("qkv", "ctx", "lse", "attn_partial", "g", "y", "mlp_partial"):
            check(f"shard{r}.{k}", g[k], rs[k], tol, errs)
        grads = ("dhf_partial", "dA", "da", "dB", "du2_partial", "dWqkv", "dbqkv", "dWo", "du_partial")
        for k in grads + (() if embed else ("dE",)):
            check(f"shard{r}.{k}", g[k], rs[k], tol, errs)
    if embed:
        dE_emb, dpos = R.embedding_bwd(ref["dX"], inp["ids"], cfg.V, cfg.s, keep0, float(np.float32(p_hidden)))
        check("dpos", out["dpos"], dpos, tol, errs)
        Vl = cfg.V // cfg.p
        for r in range(cfg.p):
            # tied weights: gradient of the output embedding plus the scattered rows of the input embedding
            check(f"shard{r}.dE(tied)", out["shards"][r]["dE"], ref["shards"][r]["dE"] + dE_emb[:, r * Vl:(r + 1) * Vl],
                  tol, errs)
    return errs


@pytest.mark.parametrize("variant", ["gpt", "bert", "no_final_ln", "p4", "embed"])
def test_small_fp32_dropout_layers(variant):
    kw = dict(b=2, s=80, H=128, h=4, F=512, V=256, p=2, dtype="fp32")
    if variant == "bert":
        kw.update(causal=False, masked_lm=True)
    elif variant == "no_final_ln":
        kw.update(final_ln=False)
    elif variant == "p4":
        kw.update(p=4, s=72)
    errs = run_dropout_layer(synth.small_config(**kw), 0.25, 0.125, embed=variant == "embed")
    print(variant, "worst:", sorted(errs, key=lambda e: -e[1])[:4])


BF16_DROP_CASES = {
    "d64_causal": dict(b=2, s=200, H=128, h=2, F=512, V=640, p=2),
    "d96_causal": dict(b=2, s=328, H=192, h=2, F=768, V=1088, p=2),
    "d128_causal_p1": dict(b=1, s=264, H=256, h=2, F=1024, V=520, p=1),
    "d192_causal": dict(b=2, s=200, H=384, h=2, F=1536, V=640, p=2),
    "d64_short_seq": dict(b=3, s=40, H=128, h=2, F=512, V=256, p=2),
    "d96_bert": dict(b=2, s=136, H=384, h=4, F=1536, V=512, p=2, causal=False, masked_lm=True),
    "d64_bert_p4": dict(b=3, s=176, H=256, h=4, F=1024, V=960, p=4, causal=False, masked_lm=True),
    "d96_embed": dict(b=2, s=328, H=192, h=2, F=768, V=1088, p=2),
}


@pytest.mark.parametrize("case", sorted(BF16_DROP_CASES))
def test_small_bf16_dropout_layers(case):
    cfg = synth.small_config(name=case, dtype="bf16", **BF16_DROP_CASES[case])
    errs = run_dropout_layer(cfg, 0.1, 0.1, embed=case.endswith("embed"))
    print(case, "worst:", sorted(errs, key=lambda e: -e[1])[:4])


def test_full_size_8p3b_shape_dropout_and_embedding_all_shards():
    """The 8.3B-shaped layer (s = 1024, H = 3072, 32 heads of 96, vocabulary 51,200, 8 shards: the launch
    configuration of the benchmark, batch 2 of 8 to bound the oracle's s x s mask and probability tensors) with
    dropout 0.1 at every site (Section 4.2) and the input embedding, all shards, against the oracle."""
    cfg = synth.with_batch(synth.CONFIGS["gpt2_8p3b"], 2)
    errs = run_dropout_layer(cfg, 0.1, 0.1, scale_w=1.0, embed=True)
    print("worst max-norm relative errors:", sorted(errs, key=lambda e: -e[1])[:6])


# ------------------------------------------------------------------ input embedding on its own
@pytest.mark.parametrize("dtype,H,V,p", [("fp32", 80, 96, 2), ("bf16", 288, 1024, 4), ("bf16", 3072, 512, 1)])
def test_embedding_entry_points(dtype, H, V, p):
    dt, code = _tdt(dtype)
    b, s = 3, 45
    T = b * s
    rng = np.random.default_rng(H + V)
    rnd = synth.round_to_bf16 if dtype == "bf16" else (lambda a: a.astype(np.float32))
    E = rnd(rng.standard_normal((H, V)).astype(np.float32))
    ids = rng.integers(0, V, size=(b, s)).astype(np.int32)
    ids[1, :20] = ids[0, 3]                                      # a long run of one id
    dx0 = rnd(rng.standard_normal((T, H)).astype(np.float32))
    dE0 = rnd(rng.standard_normal((H, V)).astype(np.float32))    # what the output embedding's backward left
    parts_ref = R.embedding_sharded(E, ids, p)
    Vl = V // p
    flat = ids.reshape(-1)
    d_ids = torch.from_numpy(flat).to(DEV)
    drop = B.make_dropout(0.25, 99, 5)
    keep = R.keep_mask(99, 5, (T, H), 0.25)
    dz_ref = np.where(keep, dx0.astype(np.float64), 0.0) / 0.75
    dE_ref, dpos_ref = R.embedding_bwd(dx0, ids, V, s, keep, 0.25)
    dz = torch.empty(T, H, device=DEV, dtype=dt); dpos = torch.empty(s, H, device=DEV, dtype=dt)
    dims0 = B.make_dims(b, s, H, p, 4 * H, V, p, 0, code)    # heads play no part here; h = p keeps the dims valid
    B.mlm_embed_bwd_replicated(dims0, _up(dx0, dt), drop, dz, dpos)
    assert np.array_equal(_dn(dz) != 0, keep & (dx0 != 0))
    assert relerr(_dn(dz), dz_ref) <= TOL[dtype] and relerr(_dn(dpos), dpos_ref) <= TOL[dtype]
    for r in range(p):
        dims = B.make_dims(b, s, H, p, 4 * H, V, p, r, code)
        perm = torch.empty(T, device=DEV, dtype=torch.int32)
        part = torch.full((T + 1, H), 7.0, device=DEV, dtype=dt)
        B.mlm_embed_shard_fwd(dims, d_ids, _up(E[:, r * Vl:(r + 1) * Vl], dt), perm, part)
        # integer work: the order is the stable sort by local id, ids outside the shard last
        key = np.where((flat >= r * Vl) & (flat < (r + 1) * Vl), flat - r * Vl, Vl)
        assert np.array_equal(perm.cpu().numpy(), np.argsort(key, kind="stable"))
        got = _dn(part)
        assert np.all(got[T] == 7.0)
        assert np.array_equal(got[:T], parts_ref[r])             # a lookup copies values: exact
        dE = _up(dE0[:, r * Vl:(r + 1) * Vl], dt)
        B.mlm_embed_shard_bwd(dims, d_ids, perm, dz, dE)
        want = dE0[:, r * Vl:(r + 1) * Vl].astype(np.float64) + R.embedding_bwd(_dn(dz), ids, V, s)[0][:, r * Vl:(r + 1) * Vl]
        assert relerr(_dn(dE), want) <= TOL[dtype]
        untouched = np.setdiff1d(np.arange(Vl), key[key < Vl])
        assert np.array_equal(_dn(dE)[:, untouched], dE0[:, r * Vl:(r + 1) * Vl][:, untouched].astype(np.float64))


def test_dropout_recompute_and_determinism_bf16():
    """Same seeds, same masks: the recomputed forward (activation checkpointing) regenerates identical dropout, so
    gradients from poisoned + recomputed activations are bit-identical to the stored-activation path."""
    cfg = synth.small_config(dtype="bf16", b=2, s=200, H=256, h=4, F=1024, V=1024, p=2)
    inp = synth.make_inputs(cfg, nonzero_bias=True, random_ln=True)
    grads = []
    for recompute in (False, True):
        L = LayerShards(cfg, [0, 1], DEV, dropout=dict(p_attn=0.1, p_hidden=0.1, base_seed=3, offsets=OFFSETS))
        L.load_host_inputs(inp)
        L.forward()
        if recompute:
            L.drop_layer_activations()
            for r in (0, 1):
                L.sh[r]["keep_bits"].fill_(-1)
            L.recompute_layer()
        L.backward()
        torch.cuda.synchronize()
        g = {k: L.act[k].clone() for k in ("dX", "dX1", "dX2", "dg1", "dbo", "dc")}
        for r in (0, 1):
            for k in ("dWqkv", "dWo", "dA", "dB", "dE"):
                g[f"{r}.{k}"] = L.sh[r][k].clone()
        grads.append(g)
    for k, v in grads[0].items():
        assert torch.isfinite(v.float()).all(), k
        assert torch.equal(v, grads[1][k]), k


# ------------------------------------------------------------------ loss on the masked rows only (BERT-shaped loss)
def _run_loss_rows(cfg, scale_w, dropout=None):
    inp = synth.make_inputs(cfg, nonzero_bias=True, random_ln=True)
    for k in ("Wq", "Wk", "Wv", "Wo", "A", "B", "E"):
        inp[k] = inp[k] * np.float32(scale_w)
        if cfg.dtype == "bf16":
            inp[k] = synth.round_to_bf16(inp[k])
    if dropout:
        inp["drop"] = R.layer_dropout_masks(cfg.b, cfg.s, cfg.H, cfg.h, cfg.p, BASE_SEED, OFFSETS, *dropout)
    ref = O.sharded_reference(inp, spec_of(cfg), cfg.p)
    L = LayerShards(cfg, list(range(cfg.p)), DEV, store_combined=True, loss_rows=True,
                    dropout=dict(p_attn=dropout[0], p_hidden=dropout[1], base_seed=BASE_SEED, offsets=OFFSETS) if dropout else None)
    L.load_host_inputs(inp)
    L.step()
    out = L.fetch()
    tol = TOL[cfg.dtype]
    rows = np.flatnonzero(inp["w"].reshape(-1) > 0)
    assert np.array_equal(L.rep["row_idx"].cpu().numpy(), rows) and L.n_rows == rows.size     # integer work
    errs = []
    assert abs(out["loss"] - ref["loss"]) <= tol * abs(ref["loss"])
    assert out["wsum"] == float(rows.size)
    check("ce(rows)", out["ce"][:rows.size], ref["ce"][rows], tol, errs)
    check("Hf_c", out["Hf_c"][:rows.size], ref["Hf"][rows], tol, errs)
    assert np.all(out["Hf_c"][rows.size:] == 0.0)
    got_dhf = out["dHf"]
    assert np.all(got_dhf[np.setdiff1d(np.arange(cfg.T), rows)] == 0.0)         # rows without loss: exactly zero
    check("dHf", got_dhf, ref["dHf"], tol, errs)
    for k in ("dX2", "dX1", "dX", "dgf", "dbf", "dg2", "db1", "dc", "dbo"):
        if k in ("dgf", "dbf") and not cfg.final_ln:
            continue
        check(k, out[k], ref[k], tol, errs)
    for r in range(cfg.p):
        g, rs = out["shards"][r], ref["shards"][r]
        check(f"shard{r}.logits->dlogits", g["logits"][:rows.size], rs["dlogits"][rows], tol, errs)
        for k in ("dE", "dA", "dB", "dWqkv", "dWo"):
            check(f"shard{r}.{k}", g[k], rs[k], tol, errs)
    return errs


@pytest.mark.parametrize("variant", ["fp32", "fp32_no_final_ln", "bf16", "bf16_dropout"])
def test_loss_rows_gather_matches_full_loss(variant):
    kw = dict(b=3, s=136, H=128, h=2, F=512, V=640, p=2, causal=False, masked_lm=True)
    if variant.startswith("fp32"):
        cfg = synth.small_config(dtype="fp32", final_ln=variant == "fp32", **kw)
    else:
        cfg = synth.small_config(dtype="bf16", **kw)
    errs = _run_loss_rows(cfg, 3.0, dropout=(0.1, 0.1) if variant.endswith("dropout") else None)
    print(variant, "worst:", sorted(errs, key=lambda e: -e[1])[:4])


def test_full_size_bert_shape_loss_rows_all_shards():
    """The BERT-shaped workload (3.9B shape, 4 shards, masked-LM loss on ~15 % of the valid positions) with the logits
    computed for the loss rows only, all shards, against the oracle of the full layer."""
    errs = _run_loss_rows(synth.CONFIGS["bert_3p9b"], 1.0)
    print("worst max-norm relative errors:", sorted(errs, key=lambda e: -e[1])[:6])
