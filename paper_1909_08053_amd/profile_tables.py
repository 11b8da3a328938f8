"""Turns the raw output of profile_run.sh (rocprofv3 CSVs, benchmark JSON, sweep logs) into the text summaries under
profiles/ and profiles/traffic.json.  No GPU needed:

    python -m paper_1909_08053_amd.profile_tables <raw output directory of profile_run.sh> [core|sweeps|all]

Every summary starts with the command that produced its raw data.  The summaries hold measured figures and ratios
derived from them only, no interpretation.
"""
from __future__ import annotations

import collections
import csv
import glob
import json
import os
import re
import statistics as st
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PROF = os.path.join(ROOT, "profiles")
PRE = "cd /tmp && export TMPDIR=/tmp && cd <repo> && "


def _short(n):
    return n.replace("mlm::", "").replace("void ", "")


def _find(raw, sub, pattern):
    hits = sorted(glob.glob(os.path.join(raw, sub, "**", pattern), recursive=True))
    if not hits:
        raise FileNotFoundError(f"{pattern} under {raw}/{sub}")
    return hits[0]


def _write(name, lines):
    path = os.path.join(PROF, name)
    with open(path, "w") as f:
        f.write("\n".join(lines).rstrip() + "\n")
    print("wrote", os.path.relpath(path, ROOT))


# ---------------------------------------------------------------------------------------------- kernel trace
def step_roles(cfg_dims):
    """(label, substring of the kernel name, kind, algorithmic work) of every launch of one benchmark step, in launch
    order.  kind: F = flops (rate in TFLOP/s), B = bytes (GB/s), - = finishing launch (no rate)."""
    T, H, Hl, Fl, Vl = cfg_dims
    TH = T * H * 2
    GF = lambda m, k, n: 2.0 * m * k * n
    att = 2.0 * 2.0 * 8 * 4 * 1024 * 1024 * 96 * 0.5       # causal-algorithmic forward flops at the benchmark shape
    return [
        ("F1  layer norm 1", "ln_fwd", "B", 2 * TH),
        ("F2  QKV GEMM + bias 8192x3072x1152", "gemm_bf16_v2_kernel", "F", GF(T, H, 3 * Hl)),
        ("F3  attention forward (causal, 32 x 1024 x 96)", "attn_fwd", "F", att),
        ("F4  projection GEMM 8192x384x3072 -> partial", "gemm_bf16_v2_kernel", "F", GF(T, Hl, H)),
        ("F5+F6  reduction + bias + residual + layer norm 2", "ln_fwd", "B", 4 * TH),
        ("F7  FC1 GEMM + bias + GeLU 8192x3072x1536", "gemm_bf16_v2_kernel", "F", GF(T, H, Fl)),
        ("F8  FC2 GEMM 8192x1536x3072 -> partial", "gemm_bf16_v2_kernel", "F", GF(T, Fl, H)),
        ("F9+F10  reduction + bias + residual + final layer norm", "ln_fwd", "B", 4 * TH),
        ("F11 logits GEMM + CE partials + logits store 8192x3072x6400", "gemm_bf16_v2_kernel", "F", GF(T, H, Vl)),
        ("F11 fix-up of the split last round", "fixup", "-", 0),
        ("F11 merge of the per-tile (m, s, t)", "ce_tile_merge", "-", 0),
        ("F12 loss merge over shards", "ce_merge", "-", 0),
        ("B1  dlogits in place", "dlogits", "B", 2 * T * Vl * 2),
        ("B1  dE = Hf^T dL 3072x8192x6400", "gemm_bf16_v2_kernel", "F", GF(T, H, Vl)),
        ("B1  fix-up", "fixup", "-", 0),
        ("B1  dHf partial = dL E^T 8192x6400x3072", "gemm_bf16_v2_kernel", "F", GF(T, H, Vl)),
        ("B1  fix-up of dHf's split half round", "fixup", "-", 0),
        ("B2  reduction + final layer norm backward", "ln_bwd", "B", 3 * TH),
        ("B3+B4  dG = (dX2 B^T) o GeLU' 8192x3072x1536", "gemm_bf16_v2_kernel", "F", GF(T, H, Fl)),
        ("B4  da partial sums", "colsum_partial", "B", T * Fl * 2),
        ("B5  dU2 partial = dG A^T 8192x1536x3072", "gemm_bf16_v2_kernel", "F", GF(T, Fl, H)),
        ("B6  reduction + layer norm 2 backward + residual", "ln_bwd", "B", 4 * TH),
        ("B7  dC = dX1 Wo^T 8192x3072x384", "gemm_bf16_v2_kernel", "F", GF(T, H, Hl)),
        ("B7  fix-up", "fixup", "-", 0),
        ("B8  attention backward dQ (+ delta)", "attn_bwd_dq", "Q", 0),
        ("B8  attention backward dK, dV", "attn_bwd_dkv", "K", 2 * att),
        ("B9  dbqkv partial sums", "colsum_partial", "B", T * 3 * Hl * 2),
        ("B9  dU partial = dQKV Wqkv^T 8192x1152x3072", "gemm_bf16_v2_kernel", "F", GF(T, H, 3 * Hl)),
        ("B3,B5,B7,B9  dB, dA, dWqkv, dWo in one grouped launch", "group_kernel", "F",
         GF(T, H, Fl) * 2 + GF(T, H, 3 * Hl) + GF(T, Hl, H)),
        ("B10 reduction + layer norm 1 backward + residual", "ln_bwd", "B", 4 * TH),
        ("B2,B4,B6,B9,B10  all deferred column sums (dgamma, dbeta, dc, da, dbo, dbqkv)", "reduce_cols_batch", "-", 0),
    ]


def position_table(trace_csv, steps):
    rows = list(csv.DictReader(open(trace_csv)))
    rows.sort(key=lambda r: int(r["Start_Timestamp"]))
    rows = [r for r in rows if "at::native" not in r["Kernel_Name"] and "rocclr" not in r["Kernel_Name"]]
    roles = step_roles((8192, 3072, 384, 1536, 6400))
    n = len(roles)
    names = [r["Kernel_Name"] for r in rows]
    # a step starts at the plain (not fused) layer-norm forward: template argument FUSED = false
    starts = [i for i, nm in enumerate(names) if "ln_fwd" in nm and "Li6ELb0E" in nm and i + n <= len(rows)]
    starts = starts[-steps:]
    dur = [[] for _ in range(n)]
    for s0 in starts:
        for k in range(n):
            r = rows[s0 + k]
            if roles[k][1] not in r["Kernel_Name"]:
                raise RuntimeError(f"launch {k} of a step is {r['Kernel_Name'][:60]}, expected {roles[k][1]}")
            dur[k].append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
    out = [f"{'step of the path (kernel position inside one benchmark step)':74s} {'avg us':>8s} {'min us':>8s}   rate"]
    tot = 0.0
    sums = collections.Counter()
    for k in range(n):
        a, mn = st.mean(dur[k]), min(dur[k])
        tot += a
        label, _, kind, w = roles[k]
        rate = ""
        if kind == "K":
            both = a + st.mean(dur[k - 1])
            rate = f"{w / both / 1e6:7.0f} TFLOP/s (dQ + dK/dV, {w / 1e9:.1f} GF)"
            sums["mfma"] += a
        elif kind in ("F", "Q"):
            rate = f"{w / a / 1e6:7.0f} TFLOP/s" if kind == "F" else ""
            sums["mfma"] += a
        elif kind == "B":
            rate = f"{w / a / 1e3:7.0f} GB/s"
            sums["row"] += a
        else:
            sums["finish"] += a
        out.append(f"{label:74s} {a:8.1f} {mn:8.1f}   {rate}")
    out.append(f"{'sum of kernel durations':74s} {tot:8.1f}")
    wall = [(int(rows[s + n - 1]["End_Timestamp"]) - int(rows[s]["Start_Timestamp"])) / 1e3 for s in starts]
    out.append(f"{'first kernel start to last kernel end, per step':74s} {st.mean(wall):8.1f} {min(wall):8.1f}")
    flops = 1.681479696384e12
    out.append("")
    out.append(f"GEMM + attention kernels: {sums['mfma']:.1f} us per step = {flops / sums['mfma'] / 1e6:.0f} model TFLOP/s over their "
               f"own time = {flops / sums['mfma'] / 1e6 / 2500 * 100:.1f} % of the 2.5 PFLOP/s bf16 dense peak")
    out.append(f"bandwidth-bound row kernels: {sums['row']:.1f} us; launches that only finish a reduction (fix-ups, column "
               f"sums, loss merges): {sums['finish']:.1f} us")
    return out, len(starts)


def kernels(raw):
    bench = json.loads(open(os.path.join(raw, "bench.json")).read().strip().splitlines()[-1])
    stats = list(csv.DictReader(open(_find(raw, "trace", "*kernel_stats.csv"))))
    cmd = "rocprofv3 --kernel-trace --stats -d gpurun_out/prof/trace -o bench --output-format csv -- python3 bench.py --no-call-table"
    L = ["rocprofv3 kernel summary of the default benchmark run (8.3B-shape 1/8 shard, bf16, one MI355X)",
         "command: " + PRE + cmd,
         f"(bench.py defaults: --gpus 1 --steps {bench['steps']} --warmup {bench['warmup']}; produced by "
         "paper_1909_08053_amd/profile_run.sh + profile_tables.py)", "",
         f"{'kernel':100s} {'calls':>6s} {'avg us':>9s} {'min us':>9s} {'max us':>9s} {'% time':>7s}"]
    for r in stats:
        n = _short(r["Name"])
        if "at::native" in n or "rocclr" in n:
            continue
        L.append(f"{n[:100]:100s} {r['Calls']:>6s} {float(r['AverageNs']) / 1e3:9.1f} {float(r['MinNs']) / 1e3:9.1f} "
                 f"{float(r['MaxNs']) / 1e3:9.1f} {float(r['Percentage']):7.2f}")
    us = lambda key: next((float(r["AverageNs"]) / 1e3 for r in stats if key in r["Name"]), 0.0)
    ce_us, fx_us, tm_us = us("gemm_bf16_v2_kernel<true, false, 3"), us("gemm_v2_fixup_kernel<3>"), us("ce_tile_merge_kernel")
    gf = 2.0 * 8192 * 3072 * 6400
    tf = gf / ce_us / 1e6
    rl = bench["roofline"]
    L += ["",
          "dominant kernel: gemm_bf16_v2_kernel<true,false,EPI_CE,8> (logits GEMM 8192x3072x6400 fused with the cross-entropy "
          "partials + logits store)",
          f"  rocprofv3 average duration {ce_us:.1f} us  ->  {gf / 1e9:.2f} GFLOP / {ce_us:.1f} us = {tf:.1f} TFLOP/s = "
          f"{tf / 25:.1f} % of the 2.5 PFLOP/s bf16 dense peak",
          f"  the same call also launches the tail fix-up of this GEMM (gemm_v2_fixup_kernel<3>, {fx_us:.1f} us) and the per-tile "
          f"partial merge (ce_tile_merge_kernel, {tm_us:.1f} us): {ce_us + fx_us + tm_us:.1f} us for the three",
          f"  bench.py live (hip events on the launch stream around mlm_vocab_ce_shard_fwd inside the timed steps = those three "
          f"launches): {rl['kernel_ms'] * 1e3:.1f} us, {rl['achieved']:.1f} TFLOP/s, frac {rl['frac']:.3f}",
          f"whole path (untraced run of the same command): {bench['ms_per_step'] * 1e3:.1f} us per step, "
          f"{bench['value']:.1f} model TFLOP/s = {bench['value'] / 25:.1f} % of the bf16 dense peak, "
          f"{bench['value'] / bench['config']['measured_mfma_peak_tflops'] * 100:.1f} % of the matrix pipe's measured rate on "
          f"normally distributed operands ({bench['config']['measured_mfma_peak_tflops']:.0f} TFLOP/s)"]
    tab, nsteps = position_table(_find(raw, "trace", "*kernel_trace.csv"), bench["steps"])
    L += ["",
          "The same trace by position inside the step (kernel names repeat across roles, the launch order does not): average and "
          f"minimum over the {nsteps} timed steps,",
          "with the algorithmic rate of each launch (GEMM 2MKN; attention causal-algorithmic; row kernels: bytes each tensor is "
          "read or written once; bf16 = 2 bytes).",
          "Peaks: 2500 TFLOP/s bf16 MFMA, 8000 GB/s HBM.", ""] + tab
    if "calls" in bench:
        L += ["", "bench.py's own per-call table of the same untraced run (hip-event brackets around every library call, 10 "
                  "extra steps; a bracket adds the launch gaps around its kernels):"]
        for c in bench["calls"]:
            rate = f"{c['TFLOP/s']:8.1f} TFLOP/s" if "TFLOP/s" in c else f"{c['GB/s']:8.1f} GB/s"
            L.append(f"  {c['call']:28s} {c['ms'] * 1e3:8.1f} us {rate}   {c['what']}")
        m, r = bench["mfma_calls"], bench["row_calls"]
        L.append(f"  calls holding the MFMA kernels: {m['ms'] * 1e3:.1f} us, {m['TFLOP/s']:.1f} TFLOP/s; layer-norm calls: "
                 f"{r['ms'] * 1e3:.1f} us, {r['GB/s']:.0f} GB/s")
    _write("bench_gpt2_8p3b_shard_kernel_stats.txt", L)


# ---------------------------------------------------------------------------------------------- HBM traffic
def _pmc(path, ctr):
    d = collections.defaultdict(list)
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] == ctr:
            d[_short(r["Kernel_Name"])].append(float(r["Counter_Value"]))
    return d


def traffic(raw):
    f = _pmc(_find(raw, "fetch", "*counter_collection.csv"), "FETCH_SIZE")
    w = _pmc(_find(raw, "write", "*counter_collection.csv"), "WRITE_SIZE")
    avg = lambda v: sum(v) / len(v)
    comb = next(k for k in f if "combine_kernel" in k)
    cek = next(k for k in f if "gemm_bf16_v2_kernel<true, false, 3" in k)
    copy_bytes = 8192 * 3072 * 2
    # every combine_kernel dispatch of these runs is a plain copy (bench.py --copy-calibration)
    fr, fw = copy_bytes / (avg(f[comb]) * 1024), copy_bytes / (avg(w[comb]) * 1024)
    ce_f, ce_w = avg(f[cek]) * 1024 * fr, avg(w[cek]) * 1024 * fw
    alg = (8192 * 3072 + 3072 * 6400 + 8192 * 6400) * 2
    args = "--steps 3 --warmup 1 --no-cpu-baseline --no-call-table --copy-calibration"
    L = ["HBM-side traffic of the dominant kernel from rocprofv3 PMC counters (FETCH_SIZE and WRITE_SIZE, KiB per dispatch, one "
         "counter per run)",
         f"commands: {PRE}rocprofv3 --pmc FETCH_SIZE -d gpurun_out/prof/fetch -o bench --output-format csv -- python3 bench.py {args}",
         f"          the same with --pmc WRITE_SIZE -d gpurun_out/prof/write      (paper_1909_08053_amd/profile_run.sh + profile_tables.py)",
         "",
         f"calibration: combine_kernel (three launches after the timed steps, one partial, no bias, no residual) is a plain copy of "
         f"[8192,3072] bf16 = {copy_bytes / 1e6:.2f} MB in, same out",
         f"  FETCH_SIZE reads {avg(f[comb]):.0f} KiB  -> scale {fr:.3f};  WRITE_SIZE reads {avg(w[comb]):.0f} KiB -> scale {fw:.3f}",
         f"logits GEMM + CE partials (gemm_bf16_v2_kernel<true,false,EPI_CE,8>): FETCH_SIZE {avg(f[cek]):.0f} KiB, WRITE_SIZE "
         f"{avg(w[cek]):.0f} KiB per dispatch",
         f"  scaled: {ce_f / 1e6:.1f} MB read + {ce_w / 1e6:.1f} MB written = {(ce_f + ce_w) / 1e6:.1f} MB per launch",
         f"  algorithmic (each operand once, logits once): {alg / 1e6:.1f} MB  ->  ratio {(ce_f + ce_w) / alg:.2f}"]
    fxk = [k for k in f if "gemm_v2_fixup_kernel<3>" in k]
    if fxk:
        L.append(f"  its tail fix-up kernel (gemm_v2_fixup_kernel<EPI_CE>, sums the fp32 partial tiles of the split last round): "
                 f"{avg(f[fxk[0]]) * 1024 * fr / 1e6:.1f} MB read + {avg(w[fxk[0]]) * 1024 * fw / 1e6:.1f} MB written")
    panel = 256 * 3072 * 2 / 1e6
    L += ["",
          "Lower bound of the reads for this tiling: FETCH_SIZE counts every read that leaves an XCD's L2.  The chip has 8 XCDs "
          "with private 4-MB L2s and 32 CUs each,",
          f"one 256 x 256 tile per CU.  The 32 tiles resident on an XCD touch at least 2 sqrt(32) = 11.3 operand panels of "
          f"256 x 3072 bf16 = {panel:.2f} MB per round (a 4 x 8 patch touches 12),",
          f"and one round's panels (12 x {panel:.2f} = {12 * panel:.1f} MB) exceed the L2, so nothing survives to the next round: "
          f"800 tiles / 256 = 3.125 rounds x 8 XCDs x 12 panels x {panel:.2f} MB = {3.125 * 8 * 12 * panel:.0f} MB",
          f"of reads against {(8192 * 3072 + 3072 * 6400) * 2 / 1e6:.0f} MB of operands; the re-reads are served by the 256-MB "
          "memory-side cache.  The writes are the logits (104.9 MB) plus the fp32 partial tiles of the split last round."]
    _write("logits_ce_gemm_hbm_traffic.txt", L)
    with open(os.path.join(PROF, "traffic.json"), "w") as fjs:
        json.dump({"gpt2_8p3b": {"logits_ce_fwd_bytes": ce_f + ce_w, "fetch_bytes": ce_f, "write_bytes": ce_w,
                                 "fetch_scale": fr, "write_scale": fw,
                                 "source": "paper_1909_08053_amd/profile_tables.py from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE"}},
                  fjs, indent=1)
    print("wrote profiles/traffic.json")


def sq_counters(raw):
    disp = {}
    for r in csv.DictReader(open(_find(raw, "sq", "*counter_collection.csv"))):
        d = disp.setdefault(int(r["Dispatch_Id"]), {"name": r["Kernel_Name"]})
        d[r["Counter_Name"]] = d.get(r["Counter_Name"], 0.0) + float(r["Counter_Value"])
    agg = collections.OrderedDict()
    for i in sorted(disp):
        d = disp[i]
        n = _short(d["name"])
        if not ("gemm_bf16_v2" in n or "attn_" in n):
            continue
        a = agg.setdefault(n, collections.Counter())
        a["n"] += 1
        for k, v in d.items():
            if k != "name":
                a[k] += v
    L = ["SQ counters of the MFMA kernels in the benchmark step (one MI355X; sums over the dispatches of 3 timed steps + 1 warm-up).",
         f"command: {PRE}rocprofv3 --pmc SQ_LDS_BANK_CONFLICT SQ_LDS_IDX_ACTIVE SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CYCLES -d "
         "gpurun_out/prof/sq -o bench --output-format csv -- python3 bench.py --steps 3 --warmup 1 --no-cpu-baseline --no-call-table",
         "(SQ_VALU_MFMA_BUSY_CYCLES is summed over the four SIMDs of a CU and SQ_BUSY_CYCLES counted per CU group, so the last "
         "column is a relative measure across kernels, not a fraction)", "",
         f"{'kernel':78s} {'dispatches':>10s} {'LDS conflict / LDS active':>26s} {'MFMA busy / SQ busy':>20s}"]
    for n, a in sorted(agg.items()):
        L.append(f"{n[:78]:78s} {a['n']:10d} {a['SQ_LDS_BANK_CONFLICT'] / max(a['SQ_LDS_IDX_ACTIVE'], 1):26.3f} "
                 f"{a['SQ_VALU_MFMA_BUSY_CYCLES'] / max(a['SQ_BUSY_CYCLES'], 1):20.2f}")
    _write("mfma_kernels_sq_counters.txt", L)


def microbench(raw):
    mb = open(os.path.join(raw, "microbench.txt")).read().rstrip().splitlines()
    L = ["On-box ceilings (MI355X, gfx950): matrix pipe on constant and on normally distributed operands, with the GEMM main "
         "loop's LDS fragment reads and HBM -> LDS copies added one at a time; LDS and HBM bandwidth.",
         "command: hipcc --offload-arch=gfx950 -O3 -Xclang -target-feature -Xclang -packed-fp32-ops "
         "paper_1909_08053_amd/csrc/tools/microbench.hip -o gpurun_out/prof/mlm_microbench && gpurun_out/prof/mlm_microbench",
         "(256 workgroups = one per CU, 2 x 10^4 k-slices of 32 per launch, mean and best of 5 launches; peak of the data sheet: "
         "2500 TFLOP/s)", ""] + mb
    _write("mfma_lds_microbench.txt", L)


# ---------------------------------------------------------------------------------------------- sweeps
def _raw_lines(path):
    return [l.rstrip() for l in open(path).read().splitlines() if l.strip() and "amdgpu.ids" not in l]


def sweeps(raw):
    L = ["Single-GPU shape sweeps of the layer-shard path (one shard: forward + backward, bf16, synthetic inputs, one MI355X).",
         "commands: python -m paper_1909_08053_amd.sweep          (defaults: --sweep all --steps 20 --warmup 3)",
         "          python -m paper_1909_08053_amd.sweep --sweep table1 --recompute",
         "(one box of the pool, back to back; the same build varies by about +-3 % from box to box)", ""]
    L += _raw_lines(os.path.join(raw, "sweeps.txt")) + [""] + _raw_lines(os.path.join(raw, "sweeps_recompute.txt"))
    _write("shape_sweeps_heads_and_strong_scaling.txt", L)
    _write("bert_3p9b_shard_loss_rows.txt",
           ["BERT-shaped shard (3.9B shape, shard 0 of 4: b=8 s=512 H=2560 10 local heads of 64, FFN 2560 local, vocabulary 7648 "
            "local;", "key padding, masked-LM loss on 15 % of the valid positions), forward + backward, bf16, one MI355X.",
            "command: python -m paper_1909_08053_amd.sweep --sweep bert_rows      (defaults: --steps 20 --warmup 3; hip-event timing)",
            "(0.981 model TFLOP per step with logits for all rows)", ""] + _raw_lines(os.path.join(raw, "bert_rows.txt")))
    _write("training_step_4_layers_gpt2_8p3b_shard.txt",
           ["One worker's training iteration on a 4-layer stack at the 8.3B shape, shard 0 of 8 (one MI355X, bf16): input embedding,",
            "4 layers, final layer norm, vocabulary-parallel loss, backward, global-norm clip + AdamW over all 55 parameter tensors.",
            "command: python -m paper_1909_08053_amd.sweep --sweep stack --steps 10      (hip-event timing; warm-up 3)", ""]
           + _raw_lines(os.path.join(raw, "stack.txt")))
    _write("dropout_embedding_gpt2_8p3b_shard.txt",
           ["Cost of dropout (two random streams) and of the vocabulary-parallel input embedding on the 8.3B-shape 1/8 shard (one "
            "MI355X, bf16).",
            "command: python -m paper_1909_08053_amd.sweep --sweep dropout      (defaults: --steps 20 --warmup 3; hip-event timing)", ""]
           + _raw_lines(os.path.join(raw, "dropout.txt")))
    _write("optimizer_step_gpt2_8p3b_shard.txt",
           ["Optimizer step of one model-parallel worker (global gradient-norm clip + AdamW, fp32 master weights), one MI355X.",
            "command: python -m paper_1909_08053_amd.sweep --sweep optimizer      (defaults: --steps 20 --warmup 3; hip-event timing)", ""]
           + _raw_lines(os.path.join(raw, "optimizer.txt")))
    # A/B of the two schedule-level GEMM choices
    cols = ["default", "bn256", "nogroup", "neither"]
    table = collections.OrderedDict()
    for c in cols:
        for l in _raw_lines(os.path.join(raw, f"ab_{c}.txt")):
            m = re.match(r"^(\S.*?)\s+([0-9.]+) us/step", l)
            if m:
                key = re.sub(r"\s+p=.*$", "", m.group(1)).strip()
                if key.startswith("logits for"):
                    key = "bert_3p9b, " + key
                table.setdefault(key, {})[c] = float(m.group(2))
    L = ["Effect of the two schedule-level GEMM choices on every benchmark shape (one shard, forward + backward, bf16, one MI355X,",
         "one box, back to back): the grouped launch of a layer shard's weight gradients and the 256 x 192 tile, each switched off",
         "by its environment override against the default (cost model decides per GEMM).",
         "commands: python -m paper_1909_08053_amd.sweep --sweep table1 --steps 10 ; python -m paper_1909_08053_amd.sweep --sweep "
         "bert_rows --steps 10", "          run four times: as is, with MLM_GEMM_BN=256, with MLM_GEMM_GROUP=0, with both", "",
         f"{'us per step':36s} {'default':>10s} {'BN=256 only':>12s} {'no grouping':>12s} {'neither':>10s}"]
    for k, v in table.items():
        L.append(f"{k[:36]:36s} " + " ".join(f"{v.get(c, float('nan')):>{w}.1f}" for c, w in zip(cols, (10, 12, 12, 10))))
    _write("gemm_grouping_and_narrow_tile_ab.txt", L)


def main():
    raw = sys.argv[1] if len(sys.argv) > 1 else os.path.join(ROOT, "gpurun_out", "prof")
    part = sys.argv[2] if len(sys.argv) > 2 else "all"
    os.makedirs(PROF, exist_ok=True)
    if part in ("all", "core"):
        microbench(raw)
        kernels(raw)
        traffic(raw)
        sq_counters(raw)
    if part in ("all", "sweeps"):
        sweeps(raw)


if __name__ == "__main__":
    main()
