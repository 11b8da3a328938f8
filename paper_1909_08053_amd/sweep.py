#!/usr/bin/env python3
"""Single-GPU shape sweeps of the layer-shard path (one shard, forward + backward, bf16).

    python -m paper_1909_08053_amd.sweep [--sweep heads|strong_1p2b|all] [--steps K] [--warmup W]

"table1" follows Table 1 (1.2B / 2.5B / 4.2B / 8.3B on 1 / 2 / 4 / 8 GPUs); "heads" follows the paper's Table 7 (8.3B configuration, 8-way model parallel, 16 / 24 / 32 heads: head size
192 / 128 / 96); "strong_1p2b" follows Table 8 (1.2B configuration split 1 / 2 / 4 / 8 ways at batch 8).  Both are
run here as the per-GPU COMPUTE of one shard (shard 0) with synthetic inputs; the all-reduces the paper's numbers
include are not part of this build, so the printed ratios are an upper bound on what those tables measure.
Prints one line per configuration and a short ratio summary.
"""
from __future__ import annotations

import argparse
import sys


def shard_flops(cfg):
    """Model FLOPs of one shard's forward + backward (GEMM = 2MKN, backward = 2 x forward, causal attention at its
    algorithmic half)."""
    T, H, d, p = cfg.T, cfg.H, cfg.H // cfg.h, cfg.p
    hl, Fl, Vl = cfg.h // p, cfg.F // p, cfg.V // p
    Hl = hl * d
    gemm = lambda M, K, N: 2.0 * M * K * N
    att = 2.0 * (2.0 * cfg.b * hl * cfg.s * cfg.s * d) * (0.5 if cfg.causal else 1.0)
    return 3.0 * (gemm(T, H, 3 * Hl) + gemm(T, Hl, H) + gemm(T, H, Fl) + gemm(T, Fl, H) + gemm(T, H, Vl) + att)


def time_config(cfg, steps, warmup, dev="cuda:0", recompute=False):
    import torch
    from .pipeline import LayerShards
    L = LayerShards(cfg, [0], dev, store_logits=True)
    L.load_random(seed=cfg.seed)
    for _ in range(warmup):
        L.step(recompute)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        L.step(recompute)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    del L
    torch.cuda.empty_cache()
    return ms


def optimizer_timing(steps, warmup, dev="cuda:0"):
    """Global-norm clip + AdamW over one worker's parameters of the 8.3B-shape 1/8 shard (layer shard + vocabulary
    shard + replicated vectors): bandwidth-bound, 2 + 28 bytes per bf16 parameter (norm pass, then update)."""
    import torch
    from . import synth
    from .pipeline import LayerShards
    cfg = synth.CONFIGS["gpt2_8p3b"]
    L = LayerShards(cfg, [0], dev)
    L.load_random(seed=cfg.seed)
    L.step()
    for i in range(warmup):
        L.optimizer_step(i + 1, lr=1e-4)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(steps):
        L.optimizer_step(warmup + i + 1, lr=1e-4)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    nparam = sum(w.numel() for _, w, _ in L.parameters())
    nbytes = nparam * 30.0
    print(f"# optimizer step, gpt2_8p3b shard 0 of 8: {nparam / 1e6:.2f} M parameters in {len(L.parameters())} tensors")
    print(f"{ms * 1e3:9.1f} us/step  {nbytes / 1e6:8.1f} MB algorithmic  {nbytes / (ms * 1e-3) / 1e12:6.2f} TB/s "
          f"({nbytes / (ms * 1e-3) / 8e12 * 100:.1f} % of the 8 TB/s HBM peak)")


def dropout_embed_timing(steps, warmup, dev="cuda:0"):
    """Cost of the training-time extras on the 8.3B-shape 1/8 shard: dropout 0.1 at every site (attention
    probabilities from the worker's own stream, hidden sites from the replicated stream) and the vocabulary-parallel
    input embedding in front of the layer, against the dropout-free step the benchmark times."""
    import torch
    from . import binding as B
    from . import synth
    from .pipeline import LayerShards
    cfg = synth.CONFIGS["gpt2_8p3b"]
    drop = dict(p_attn=0.1, p_hidden=0.1, base_seed=1234, offsets={"attn": 1, "hidden1": 2, "hidden2": 3, "embed": 4})
    print(f"# {cfg.name} shard 0 of {cfg.p}, forward + backward, bf16")
    base = None
    for label, kw in (("dropout-free (benchmark step)", {}), ("dropout 0.1, all sites", dict(dropout=drop)),
                      ("dropout 0.1 + input embedding", dict(dropout=drop, embed=True))):
        L = LayerShards(cfg, [0], dev, store_logits=True, **kw)
        L.load_random(seed=cfg.seed)
        for _ in range(warmup):
            L.step()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            L.step()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / steps
        base = base or ms
        print(f"{label:34s} {ms * 1e3:9.1f} us/step  ({ms / base:.3f} x)", flush=True)
        if kw.get("embed"):
            # the embedding calls on their own (event-timed, one at a time)
            d0, rep, s0, a = L.dims[0], L.rep, L.sh[0], L.act
            calls = {
                "mlm_embed_shard_fwd (rank sort + column gather)":
                    lambda: B.mlm_embed_shard_fwd(d0, rep["ids"], L.w[0]["E"], s0["perm"], s0["embed_partial"]),
                "mlm_combine_dropout (+ position embedding)":
                    lambda: B.mlm_combine_dropout(d0, [s0["embed_partial"]], rep["pos"], cfg.s, L.drop["embed"], None, rep["X"]),
                "mlm_embed_bwd_replicated":
                    lambda: B.mlm_embed_bwd_replicated(d0, a["dX"], L.drop["embed"], a["dZ0"], a["dpos"]),
                "mlm_embed_shard_bwd (run sums into dE columns)":
                    lambda: B.mlm_embed_shard_bwd(d0, rep["ids"], s0["perm"], a["dZ0"], s0["dE"]),
            }
            for name, fn in calls.items():
                for _ in range(3):
                    fn()
                torch.cuda.synchronize()
                e0.record()
                for _ in range(steps):
                    fn()
                e1.record()
                torch.cuda.synchronize()
                print(f"    {name:48s} {e0.elapsed_time(e1) / steps * 1e3:8.1f} us", flush=True)
        del L
        torch.cuda.empty_cache()


def stack_timing(steps, warmup, n_layers=4, dev="cuda:0"):
    """One worker's training iteration at the 8.3B shape, 1/8 shard, on a stack of `n_layers` layers: embedding,
    layers, loss, backward, global-norm clip + AdamW.  Four variants: stored activations or checkpointing after every
    layer (the paper's setting), without and with dropout 0.1 on every site."""
    import torch
    from . import synth
    from .stack import ModelShards
    cfg = synth.CONFIGS["gpt2_8p3b"]
    per_layer = shard_flops(cfg)
    T, H, Vl = cfg.T, cfg.H, cfg.V // cfg.p
    logits = 3.0 * 2.0 * T * H * Vl
    layer = per_layer - logits
    model_flops = n_layers * layer + logits
    print(f"# {cfg.name} shard 0 of {cfg.p}, {n_layers} layers + embedding + loss + optimizer, bf16; "
          f"{model_flops / 1e12:.3f} model TFLOP per iteration (recomputation not counted)")
    drop = dict(p_attn=0.1, p_hidden=0.1, base_seed=99, step=1)
    for label, kw in (("stored activations, no dropout", dict(checkpoint=False)),
                      ("checkpoint every layer, no dropout", dict(checkpoint=True)),
                      ("stored activations, dropout 0.1", dict(checkpoint=False, dropout=drop)),
                      ("checkpoint every layer, dropout 0.1", dict(checkpoint=True, dropout=drop))):
        M = ModelShards(cfg, n_layers, [0], dev, **kw)
        M.load_random(seed=cfg.seed)
        for i in range(warmup):
            M.step()
            M.optimizer_step(i + 1, lr=1e-4)
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        t_fb = t_opt = 0.0
        for i in range(steps):
            ev[0].record()
            M.step()
            ev[1].record()
            M.optimizer_step(warmup + i + 1, lr=1e-4)
            ev[2].record()
            torch.cuda.synchronize()
            t_fb += ev[0].elapsed_time(ev[1])
            t_opt += ev[1].elapsed_time(ev[2])
        t_fb /= steps
        t_opt /= steps
        mem = torch.cuda.max_memory_allocated() / 2 ** 30
        print(f"{label:38s} fwd+bwd {t_fb * 1e3:9.1f} us  optimizer {t_opt * 1e3:7.1f} us  "
              f"{model_flops / ((t_fb + t_opt) * 1e-3) / 1e12:7.1f} model TFLOP/s  peak memory {mem:5.2f} GiB", flush=True)
        del M
        torch.cuda.empty_cache()
        torch.cuda.reset_peak_memory_stats()


def bert_loss_rows_timing(steps, warmup, dev="cuda:0"):
    """The BERT-shaped shard (3.9B shape, shard 0 of 4, masked-LM loss on ~15 % of the valid positions): logits for
    every row versus logits for the loss rows only."""
    import torch
    from . import synth
    from .pipeline import LayerShards
    cfg = synth.CONFIGS["bert_3p9b"]
    print(f"# {cfg.name} shard 0 of {cfg.p}, forward + backward, bf16")
    base = None
    for label, kw in (("logits for all rows", {}), ("logits for the loss rows only", dict(loss_rows=True))):
        L = LayerShards(cfg, [0], dev, store_logits=True, **kw)
        L.load_random(seed=cfg.seed)
        for _ in range(warmup):
            L.step()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            L.step()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / steps
        base = base or ms
        extra = f"  ({L.n_rows} of {cfg.T} rows)" if kw else ""
        print(f"{label:32s} {ms * 1e3:9.1f} us/step  ({ms / base:.3f} x){extra}", flush=True)
        del L
        torch.cuda.empty_cache()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--sweep", default="all", choices=["heads", "strong_1p2b", "table1", "optimizer", "dropout", "stack", "bert_rows", "all"])
    ap.add_argument("--recompute", action="store_true",
                    help="checkpointed variant: re-run the layer's forward before its backward (activation recomputation)")
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    args = ap.parse_args()
    import torch
    from . import binding as B
    from . import synth
    if not torch.cuda.is_available():
        sys.exit("sweep: no GPU visible")
    B.lib()
    names = ["heads", "strong_1p2b", "table1"] if args.sweep == "all" else [args.sweep]
    if args.sweep == "optimizer":
        optimizer_timing(args.steps, args.warmup)
        return
    if args.sweep == "bert_rows":
        bert_loss_rows_timing(args.steps, args.warmup)
        return
    if args.sweep == "stack":
        stack_timing(args.steps, args.warmup)
        return
    if args.sweep == "dropout":
        dropout_embed_timing(args.steps, args.warmup)
        return
    for sw in names:
        print(f"# sweep {sw}" + (" (activation recomputation: layer forward run twice)" if args.recompute else ""))
        rows = []
        for cfg in synth.SWEEPS[sw]:
            ms = time_config(cfg, args.steps, args.warmup, recompute=args.recompute)
            fl = shard_flops(cfg)
            rows.append((cfg, ms, fl))
            print(f"{cfg.name:16s} p={cfg.p} heads={cfg.h:2d} d={cfg.H // cfg.h:3d} local_heads={cfg.h // cfg.p:2d}  "
                  f"{ms * 1e3:9.1f} us/step  {fl / 1e12:6.3f} model TFLOP  {fl / (ms * 1e-3) / 1e12:7.1f} TFLOP/s", flush=True)
        if sw == "heads":
            ref = rows[0][1]
            print("  step time relative to 16 heads: " + ", ".join(f"{c.h} heads {ms / ref:.3f}" for c, ms, _ in rows))
        elif sw == "table1":
            ref = rows[0][2] / rows[0][1]
            print("  per-GPU model throughput relative to the 1-GPU row: " +
                  ", ".join(f"p={c.p} {(fl / ms) / ref:.3f}" for c, ms, fl in rows))
        else:
            ref = rows[0][1]
            print("  compute-only speed-up of one shard over p = 1: " +
                  ", ".join(f"p={c.p} {ref / ms:.2f}x" for c, ms, _ in rows))


if __name__ == "__main__":
    main()
