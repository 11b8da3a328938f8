#!/usr/bin/env python3
"""Benchmark of the layer-shard hot path on one MI355X.

One "step" = forward + backward of ONE GPU's share (shard 0 of p) of a model-parallel transformer layer plus the
vocabulary-parallel loss: the replicated layer norms / combines / bias-gradient sums and every shard-0 call
(QKV GEMM, attention, projection, MLP GEMMs, logits GEMM fused with the cross-entropy partials, and all their
gradients).  Workload: the 8.3B-shape 1/8 shard (b=8, s=1024, H=3072, 4 local heads of 96, FFN 1536 local, vocab 6400
local), bf16 storage with fp32 accumulation, synthetic inputs resident in HBM before the timed region.

Prints ONE JSON line: whole-job throughput in model TFLOP/s (FLOP convention: GEMM = 2MKN, backward = 2x forward,
causal attention counted at its algorithmic half, recomputation not counted), a `roofline` object for the dominant
kernel (the logits GEMM fused with the cross-entropy partials) and a `cpu_baseline` object (the fp64 oracle timed on
the host cores on a bounded sample).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "layer-shard fwd+bwd TFLOP/s (bf16) and % MFMA peak, 8.3B-shape 1/8 shard"
PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA (published)
PEAK_HBM_GBS = 8000.0
# The matrix pipe alone on this chip, measured: back-to-back v_mfma_f32_16x16x32_bf16 (the shape the GEMM loop uses) on
# normally distributed operands that change every instruction, no memory traffic (csrc/tools/microbench.hip;
# profiles/mfma_lds_microbench.txt; 2.03-2.05 PFLOP/s on three boxes).  The 32 x 32 x 16 shape reaches 1.72-1.79 on the
# same operands, both reach 2.44-2.46 on loop-constant operands: the difference is clock lost to switching power.
MEASURED_MFMA_TFLOPS = 2040.0


def shard_flops(cfg, causal_algorithmic=True):
    """Model FLOPs of one shard's fwd+bwd (same convention as the docstring)."""
    T, H, d, p = cfg.T, cfg.H, cfg.H // cfg.h, cfg.p
    hl, Fl, Vl = cfg.h // p, cfg.F // p, cfg.V // p
    Hl = hl * d
    gemm = lambda M, K, N: 2.0 * M * K * N
    att = 2.0 * (2.0 * cfg.b * hl * cfg.s * cfg.s * d)
    if cfg.causal and causal_algorithmic:
        att *= 0.5
    fwd = gemm(T, H, 3 * Hl) + gemm(T, Hl, H) + gemm(T, H, Fl) + gemm(T, Fl, H) + gemm(T, H, Vl) + att
    return 3.0 * fwd, gemm(T, H, Vl)


def cpu_baseline(cfg, sample_b=None):
    """Time the fp64 oracle (as it stands) on the host cores: the UNSHARDED layer + loss of the same model shape at the
    full batch (all p shards' work; about 20 s on the box's 16 cores)."""
    import numpy as np
    from oracle import layer_oracle as O
    from paper_1909_08053_amd import synth
    try:
        from threadpoolctl import threadpool_info
        threads = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    sample_b = cfg.b if sample_b is None else sample_b
    small = synth.with_batch(cfg, sample_b)
    inp = synth.make_inputs(small)
    spec = O.Spec(b=small.b, s=small.s, H=small.H, h=small.h, F=small.F, V=small.V, causal=small.causal,
                  final_ln=small.final_ln, gelu_tanh=small.gelu_tanh, ln_eps=small.ln_eps)
    t0 = time.perf_counter()
    c = O.forward(inp, spec)
    g = O.backward(inp, c, spec)
    dt = time.perf_counter() - t0
    flops = O.model_flops(spec, p=1)["fwd_bwd"]
    assert np.isfinite(c["loss"]) and np.all(np.isfinite(g["dX"]))
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": int(threads), "kind": "oracle",
            "sample": f"unsharded {cfg.name} layer+loss fwd+bwd in fp64, batch {sample_b} of {cfg.b} (nothing extrapolated) "
                      f"({flops / 1e12:.3f} model TFLOP in {dt:.1f} s)", "seconds": dt}


# Work of every call of one benchmark step, for the per-call table: ("flop", model flops) for the calls that hold the
# MFMA kernels, ("byte", algorithmic bytes: every tensor read or written once) for the bandwidth-bound row kernels.
def call_work(cfg):
    T, H, d, p = cfg.T, cfg.H, cfg.H // cfg.h, cfg.p
    hl, Fl, Vl = cfg.h // p, cfg.F // p, cfg.V // p
    Hl = hl * d
    gemm = lambda M, K, N: 2.0 * M * K * N
    att = 2.0 * (2.0 * cfg.b * hl * cfg.s * cfg.s * d) * (0.5 if cfg.causal else 1.0)
    TH = T * H * 2.0
    return [
        ("mlm_layernorm_fwd", "F1 layer norm 1", "byte", 2 * TH),
        ("mlm_attn_shard_fwd", "F2-F4 QKV GEMM + attention + projection GEMM", "flop",
         gemm(T, H, 3 * Hl) + att + gemm(T, Hl, H)),
        ("mlm_combine_layernorm_fwd", "F5+F6 reduction + bias + residual + layer norm 2", "byte", 4 * TH),
        ("mlm_mlp_shard_fwd", "F7-F8 FC1 GEMM + bias + GeLU, FC2 GEMM", "flop", gemm(T, H, Fl) + gemm(T, Fl, H)),
        ("mlm_combine_layernorm_fwd", "F9+F10 reduction + bias + residual + final layer norm", "byte", 4 * TH),
        ("mlm_vocab_ce_shard_fwd", "F11 logits GEMM + cross-entropy partials (+ tail fix-up, tile merge)", "flop",
         gemm(T, H, Vl)),
        ("mlm_vocab_ce_merge", "F12 loss merge", "byte", 7 * T * 4.0),
        ("mlm_vocab_ce_shard_bwd", "B1 dlogits + dE GEMM + dHf GEMM", "flop", 2 * gemm(T, H, Vl)),
        ("mlm_combine_layernorm_bwd", "B2 reduction + final layer norm backward (column sums deferred)", "byte", 3 * TH),
        ("mlm_mlp_shard_bwd_input", "B3-B5 dG GEMM + GeLU', da, dU2 GEMM", "flop", gemm(T, H, Fl) + gemm(T, Fl, H)),
        ("mlm_combine_layernorm_bwd", "B6 reduction + layer norm 2 backward + residual (column sums deferred)", "byte", 4 * TH),
        ("mlm_attn_shard_bwd_input", "B7-B9 dC GEMM, attention backward, dbqkv, dU GEMM", "flop",
         gemm(T, H, Hl) + 2 * att + gemm(T, 3 * Hl, H)),
        ("mlm_layer_shard_wgrads", "B3,B5,B7,B9 weight gradients dB, dA, dWqkv, dWo", "flop",
         gemm(T, H, Fl) + gemm(T, Fl, H) + gemm(T, H, 3 * Hl) + gemm(T, Hl, H)),
        ("mlm_combine_layernorm_bwd", "B10 reduction + layer norm 1 backward + residual (column sums deferred)", "byte", 4 * TH),
        ("mlm_deferred_sums_flush", "B2,B4,B6,B9,B10 all column sums (dgamma, dbeta, dc, da, dbo, dbqkv) in one launch",
         "byte", 4.0 * (-(-T // 32) * 8 * H + -(-T // 64) * (Fl + 3 * Hl))),
    ]


def per_call_table(L, P, cfg, steps):
    """Event brackets around every library call of `steps` extra steps (outside the timed region): median duration of
    each call position, its algorithmic rate, and the sums over the MFMA calls and over the row-kernel calls."""
    import torch
    work = call_work(cfg)
    names = sorted(set(w[0] for w in work))
    orig = {n: getattr(P.B, n) for n in names}
    rec = []

    def wrap(name):
        def f(*a, **k):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            orig[name](*a, **k)
            e1.record()
            rec.append((name, e0, e1))
        return f

    for n in names:
        setattr(P.B, n, wrap(n))
    per_pos = [[] for _ in work]
    try:
        for _ in range(steps):
            rec.clear()
            L.step()
            torch.cuda.synchronize()
            if [r[0] for r in rec] != [w[0] for w in work]:
                return None                      # another call sequence (other options than the benchmark's): no table
            for i, (_, e0, e1) in enumerate(rec):
                per_pos[i].append(e0.elapsed_time(e1))
    finally:
        for n in names:
            setattr(P.B, n, orig[n])
    calls, mf_ms, mf_fl, row_ms, row_by = [], 0.0, 0.0, 0.0, 0.0
    for (name, what, kind, w), v in zip(work, per_pos):
        ms = sorted(v)[len(v) // 2]
        if kind == "flop":
            calls.append({"call": name, "what": what, "ms": round(ms, 4), "TFLOP/s": round(w / ms / 1e9, 1)})
            mf_ms += ms
            mf_fl += w
        else:
            calls.append({"call": name, "what": what, "ms": round(ms, 4), "GB/s": round(w / ms / 1e6, 1)})
            if name != "mlm_vocab_ce_merge":
                row_ms += ms
                row_by += w
    return {"calls": calls,
            "mfma_calls": {"ms": round(mf_ms, 4), "TFLOP/s": round(mf_fl / mf_ms / 1e9, 1),
                           "frac_of_bf16_mfma_peak": round(mf_fl / mf_ms / 1e9 / PEAK_BF16_TFLOPS, 4),
                           "note": "sum over the seven calls that hold the GEMM and attention kernels; their brackets "
                                   "also hold the small kernels those calls launch (dlogits, column partial sums, fix-ups)"},
            "row_calls": {"ms": round(row_ms, 4), "GB/s": round(row_by / row_ms / 1e6, 1),
                          "frac_of_hbm_peak": round(row_by / row_ms / 1e6 / PEAK_HBM_GBS, 4),
                          "note": "layer-norm forward / backward calls and the one launch that finishes their column "
                                  "sums (bytes of that launch: the fp32 block partials it reads)"}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="gpt2_8p3b")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-call-table", action="store_true", help="skip the per-call event table (10 extra untimed steps)")
    ap.add_argument("--breakdown", action="store_true", help="print per-call timings to stderr")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="after the timed region, run three plain [T,H] copies (mlm_combine with one partial) so that a "
                         "rocprofv3 --pmc run has a kernel of known traffic to scale FETCH_SIZE / WRITE_SIZE with")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (no collectives are part of it); use --gpus 1")

    import torch
    from paper_1909_08053_amd import binding as B
    from paper_1909_08053_amd import synth
    from paper_1909_08053_amd.pipeline import LayerShards
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    B.lib()   # fail loudly if the HIP library is missing
    cfg = synth.CONFIGS[args.config]
    dev = "cuda:0"
    L = LayerShards(cfg, [0], dev, store_logits=True)
    L.load_random(seed=cfg.seed)
    torch.cuda.synchronize()

    # The dominant kernel (logits GEMM fused with the cross-entropy partials) is timed live, inside the timed steps,
    # with events recorded on the launch stream around the one call that enqueues it.  That bracket holds three
    # launches: the GEMM, the fix-up of its split last round and the few-microsecond merge of the per-tile partials.
    from paper_1909_08053_amd import pipeline as P
    ce_events = []
    real_ce_fwd = B.mlm_vocab_ce_shard_fwd

    def timed_ce_fwd(*a_, **k_):
        e0_, e1_ = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0_.record()
        real_ce_fwd(*a_, **k_)
        e1_.record()
        ce_events.append((e0_, e1_))

    for _ in range(args.warmup):
        L.step()
    torch.cuda.synchronize()
    P.B.mlm_vocab_ce_shard_fwd = timed_ce_fwd
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for _ in range(args.steps):
        L.step()
    ev1.record()
    torch.cuda.synchronize()
    P.B.mlm_vocab_ce_shard_fwd = real_ce_fwd
    ms_per_step = ev0.elapsed_time(ev1) / args.steps
    loss = float(L.act["loss"][0].item())
    flops, logits_flops = shard_flops(cfg)
    dense_flops, _ = shard_flops(cfg, causal_algorithmic=False)
    value = flops / (ms_per_step * 1e-3) / 1e12
    k_ms = sum(x.elapsed_time(y) for x, y in ce_events) / len(ce_events)
    # step periods from the events already in the stream (start of the timed call in consecutive steps): spread only
    periods = sorted(ce_events[i][0].elapsed_time(ce_events[i + 1][0]) for i in range(len(ce_events) - 1))
    step_ms = ({"median": periods[len(periods) // 2], "min": periods[0], "max": periods[-1]} if periods else None)
    achieved = logits_flops / (k_ms * 1e-3) / 1e12
    traffic, traffic_src = None, None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        try:
            traffic = json.load(open(tpath)).get(args.config, {}).get("logits_ce_fwd_bytes")
            traffic_src = ("profiles/traffic.json: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of the GEMM kernel of this "
                           "call, scaled by a copy of known size (not re-measured in this run)")
        except Exception:
            traffic = None
    roofline = {"bound": "mfma", "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": achieved / PEAK_BF16_TFLOPS, "traffic": traffic, "traffic_source": traffic_src,
                "kernel": "gemm_bf16_v2_kernel<true,false,EPI_CE,8> (logits GEMM + cross-entropy partials), timed as "
                          "the whole mlm_vocab_ce_shard_fwd call: + gemm_v2_fixup_kernel<EPI_CE> + ce_tile_merge_kernel",
                "kernel_ms": k_ms, "launches_in_bracket": 3, "flops_per_launch": logits_flops}

    table = None if args.no_call_table else per_call_table(L, P, cfg, 10)
    if args.breakdown:
        breakdown(L, B, cfg)
    if args.copy_calibration:
        d0 = L.dims[0]
        for _ in range(3):
            B.mlm_combine(d0, [L.rep["X"]], None, None, L.act["U"])
        torch.cuda.synchronize()

    out = {"metric": METRIC, "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": f"{cfg.name} shard 0 of {cfg.p}: b={cfg.b} s={cfg.s} H={cfg.H} local heads="
                                  f"{cfg.h // cfg.p} d={cfg.H // cfg.h} F_local={cfg.F // cfg.p} V_local={cfg.V // cfg.p}, "
                                  f"causal={cfg.causal}, fwd+bwd layer shard + vocab-parallel CE",
                      "model_tflop_per_step": flops / 1e12, "dense_equivalent_tflop_per_step": dense_flops / 1e12,
                      "frac_of_bf16_mfma_peak": value / PEAK_BF16_TFLOPS,
                      "frac_of_measured_mfma_peak": value / MEASURED_MFMA_TFLOPS,
                      "measured_mfma_peak_tflops": MEASURED_MFMA_TFLOPS, "loss": loss},
           "roofline": roofline, "step_ms": step_ms}
    if table is not None:
        out.update(table)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg)
    print(json.dumps(out))


def breakdown(L, B, cfg):
    """Per-call event timings of one step (stderr); diagnostic only."""
    import torch
    names, evs = [], []

    def mark(name):
        ev = torch.cuda.Event(enable_timing=True)
        ev.record()
        names.append(name)
        evs.append(ev)

    orig = {}
    calls = ["mlm_layernorm_fwd", "mlm_layernorm_bwd", "mlm_combine", "mlm_colsum", "mlm_combine_layernorm_fwd",
             "mlm_combine_layernorm_bwd", "mlm_attn_shard_fwd",
             "mlm_attn_shard_bwd", "mlm_mlp_shard_fwd", "mlm_mlp_shard_bwd", "mlm_vocab_ce_shard_fwd",
             "mlm_vocab_ce_merge", "mlm_vocab_ce_shard_bwd"]
    for c in calls:
        orig[c] = getattr(B, c)

        def wrap(*a, _c=c, **k):
            r = orig[_c](*a, **k)
            mark(_c)
            return r
        setattr(B, c, wrap)
    try:
        tot = {}
        for _ in range(5):
            names.clear(); evs.clear()
            mark("start")
            L.step()
            torch.cuda.synchronize()
            for i in range(1, len(evs)):
                tot.setdefault((i, names[i]), []).append(evs[i - 1].elapsed_time(evs[i]))
        total = 0.0
        for (i, n), v in sorted(tot.items()):
            ms = sorted(v)[len(v) // 2]
            total += ms
            print(f"  {i:2d} {n:28s} {ms * 1e3:9.1f} us", file=sys.stderr)
        print(f"  sum {total * 1e3:.1f} us", file=sys.stderr)
    finally:
        for c in calls:
            setattr(B, c, orig[c])


if __name__ == "__main__":
    main()
