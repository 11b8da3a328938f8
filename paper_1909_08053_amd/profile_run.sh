#!/bin/bash
# Produces the raw measurements behind profiles/*.txt on a one-GPU MI355X machine.  Run from the repository root with the
# library built (python -m paper_1909_08053_amd.build); raw output goes to the directory $O below and
#   python -m paper_1909_08053_amd.profile_tables $O
# turns it into the text summaries under profiles/ (that step needs no GPU).
# Every GPU step has its own time limit and the script stops at the first failure.
set -o pipefail
cd /tmp && export TMPDIR=/tmp && cd "${GRAFT_REPO_ROOT:-$OLDPWD}" || exit 1
O=gpurun_out/prof
rm -rf $O && mkdir -p $O
PARTS="${1:-all}"          # all | core | sweeps
step() { echo "== $1"; }

if [ "$PARTS" = all ] || [ "$PARTS" = core ]; then
  step "ceilings microbenchmark"
  hipcc --offload-arch=gfx950 -O3 -Xclang -target-feature -Xclang -packed-fp32-ops \
        paper_1909_08053_amd/csrc/tools/microbench.hip -o $O/mlm_microbench 2> /dev/null || exit 1
  timeout -k 10 300 $O/mlm_microbench > $O/microbench.txt 2>&1 || exit 1
  step "benchmark line"
  timeout -k 10 400 python3 bench.py > $O/bench.json 2> $O/bench.err || exit 1
  step "kernel trace of the default benchmark run"
  timeout -k 10 400 rocprofv3 --kernel-trace --stats -d $O/trace -o bench --output-format csv -- \
        python3 bench.py --no-call-table > $O/trace.log 2>&1 || exit 1
  step "FETCH_SIZE"
  timeout -s KILL 150 rocprofv3 --pmc FETCH_SIZE -d $O/fetch -o bench --output-format csv -- \
        python3 bench.py --steps 3 --warmup 1 --no-cpu-baseline --no-call-table --copy-calibration > $O/fetch.log 2>&1 || exit 1
  step "WRITE_SIZE"
  timeout -s KILL 150 rocprofv3 --pmc WRITE_SIZE -d $O/write -o bench --output-format csv -- \
        python3 bench.py --steps 3 --warmup 1 --no-cpu-baseline --no-call-table --copy-calibration > $O/write.log 2>&1 || exit 1
  step "SQ counters of the MFMA kernels"
  timeout -s KILL 150 rocprofv3 --pmc SQ_LDS_BANK_CONFLICT SQ_LDS_IDX_ACTIVE SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CYCLES \
        -d $O/sq -o bench --output-format csv -- \
        python3 bench.py --steps 3 --warmup 1 --no-cpu-baseline --no-call-table > $O/sq.log 2>&1 || exit 1
fi

if [ "$PARTS" = all ] || [ "$PARTS" = sweeps ]; then
  step "shape sweeps (heads, strong scaling, Table 1 rows)"
  timeout -k 10 600 python3 -u -m paper_1909_08053_amd.sweep > $O/sweeps.txt 2>&1 || exit 1
  timeout -k 10 400 python3 -u -m paper_1909_08053_amd.sweep --sweep table1 --recompute > $O/sweeps_recompute.txt 2>&1 || exit 1
  step "BERT-shaped shard, 4-layer training step, dropout + embedding, optimizer"
  timeout -k 10 200 python3 -u -m paper_1909_08053_amd.sweep --sweep bert_rows > $O/bert_rows.txt 2>&1 || exit 1
  timeout -k 10 300 python3 -u -m paper_1909_08053_amd.sweep --sweep stack --steps 10 > $O/stack.txt 2>&1 || exit 1
  timeout -k 10 300 python3 -u -m paper_1909_08053_amd.sweep --sweep dropout > $O/dropout.txt 2>&1 || exit 1
  timeout -k 10 200 python3 -u -m paper_1909_08053_amd.sweep --sweep optimizer > $O/optimizer.txt 2>&1 || exit 1
  step "A/B of the grouped weight-gradient launch and the 256 x 192 tile (environment overrides)"
  for v in default bn256 nogroup neither; do
    unset MLM_GEMM_BN MLM_GEMM_GROUP
    case $v in bn256) export MLM_GEMM_BN=256 ;; nogroup) export MLM_GEMM_GROUP=0 ;; neither) export MLM_GEMM_BN=256 MLM_GEMM_GROUP=0 ;; esac
    timeout -k 10 300 python3 -u -m paper_1909_08053_amd.sweep --sweep table1 --steps 10 > $O/ab_${v}.txt 2>&1 || exit 1
    timeout -k 10 200 python3 -u -m paper_1909_08053_amd.sweep --sweep bert_rows --steps 10 >> $O/ab_${v}.txt 2>&1 || exit 1
  done
  unset MLM_GEMM_BN MLM_GEMM_GROUP
fi
echo "profile_run: done"
