#!/bin/bash
# Profiles `bench.py` for one workload with rocprofv3 and writes raw output plus text summaries under
# $OUT (default: prof_<tag> under the output folder of the repository): a kernel trace with statistics, the HBM traffic counters
# (FETCH_SIZE, WRITE_SIZE: one counter per run) and two passes of SQ counters (instruction mix, matrix-core
# busy cycles, wait cycles).  The program follows `--` directly in every rocprofv3 command.
#
# usage: paper_2603_14303_amd/profile.sh <tag> [bench.py arguments, e.g. --workload stack32k --tau 0.979]
set -u
tag=$1; shift
R=$(cd "$(dirname "$0")/.." && pwd)
OUT=${OUT:-$R/gpurun_out/prof_$tag}
rm -rf "$OUT"; mkdir -p "$OUT"
cd /tmp && export TMPDIR=/tmp
SQ_A="SQ_WAVES SQ_BUSY_CYCLES SQ_WAVE_CYCLES SQ_INSTS_VALU SQ_INSTS_MFMA SQ_VALU_MFMA_BUSY_CYCLES SQ_INSTS_VALU_MFMA_MOPS_BF16 SQ_INSTS_VMEM"
SQ_B="SQ_ACTIVE_INST_ANY SQ_ACTIVE_INST_VALU SQ_ACTIVE_INST_LDS SQ_ACTIVE_INST_VMEM SQ_WAIT_ANY SQ_WAIT_INST_ANY SQ_WAIT_INST_LDS SQ_INSTS_LDS"
echo "== kernel trace ($tag)"
timeout -k 10 600 rocprofv3 --kernel-trace --stats --output-format csv -d "$OUT/trace" -o run -- \
    python3 "$R/bench.py" --no-cpu-baseline --steps 10 --warmup 3 "$@" > "$OUT/bench_traced.json" 2> "$OUT/trace.err" \
    || { echo "trace failed"; tail -5 "$OUT/trace.err"; exit 1; }
i=0
for ctrs in "FETCH_SIZE" "WRITE_SIZE" "$SQ_A" "$SQ_B"; do
    i=$((i + 1))
    echo "== pmc pass $i: $ctrs"
    timeout -s KILL 300 rocprofv3 --pmc $ctrs -d "$OUT/pmc$i" -o run -- \
        python3 "$R/bench.py" --no-cpu-baseline --eager --steps 2 --warmup 1 "$@" > "$OUT/bench_pmc$i.json" 2> "$OUT/pmc$i.err" \
        || { echo "pmc pass $i failed"; tail -5 "$OUT/pmc$i.err"; exit 1; }
done
echo "== the same command without the profiler"
timeout -k 10 600 python3 "$R/bench.py" --no-cpu-baseline "$@" > "$OUT/bench_plain.json" 2> "$OUT/plain.err" || { echo "plain run failed"; exit 1; }
cd "$R" && python3 -m paper_2603_14303_amd.profile_summary "$tag" "$OUT" "$@"
rc=$?
find "$OUT" -name "*.db" -delete      # the raw counter databases are large; the summaries hold what is used
find "$OUT" -name "*kernel_trace.csv" -delete
[ $rc -eq 0 ] || exit 1
echo "summaries in $OUT"
