#!/bin/bash
# Hardware-counter passes over bench.py with rocprofv3 (one pass per counter set: the profiler
# does not split a set over several runs).  Usage, from the repository root on a GPU machine:
#   bash paper_2206_15014_amd/profile_counters.sh <output dir>
#   python3 paper_2206_15014_amd/summarize_counters.py <output dir>
# Writes <output dir>/<workload>.<set>_counter_collection.csv for each layer of the benchmark
# workload on its own, the skinny single-layer workload, and a plain 256 MiB copy (which
# calibrates FETCH_SIZE / WRITE_SIZE against a known number of bytes).
set -u
export TMPDIR=/tmp
OUT=${1:-counters_out}
mkdir -p "$OUT"
run() {  # name, counters, bench args...
  local name=$1 counters=$2; shift 2
  timeout -s KILL 120 rocprofv3 --pmc $counters --output-format csv -d "$OUT" -o "$name" -- python3 -u bench.py "$@" \
      > "$OUT/$name.log" 2>&1 || { echo "pass $name failed"; tail -5 "$OUT/$name.log"; return 1; }
  echo "pass $name done"
}
B="--steps 20 --warmup 2 --no-cpu-baseline --launch eager --compress per_layer"
SQ="SQ_WAVES SQ_BUSY_CYCLES SQ_WAVE_CYCLES SQ_VALU_MFMA_BUSY_CYCLES SQ_INSTS_VALU_MFMA_MOPS_I8 SQ_WAIT_INST_ANY SQ_LDS_BANK_CONFLICT SQ_LDS_IDX_ACTIVE"
TCC="TCC_REQ_sum TCC_HIT_sum TCC_MISS_sum TCC_EA0_RDREQ_sum"
for L in qkv attn_out ffn_up ffn_down; do
  run ${L}.fetch "FETCH_SIZE" --only $L $B || exit 1
  run ${L}.write "WRITE_SIZE" --only $L $B || exit 1
  run ${L}.sq "$SQ" --only $L $B || exit 1
  run ${L}.tcc "$TCC" --only $L $B || exit 1
done
run single.fetch "FETCH_SIZE" --workload single $B || exit 1
run single.write "WRITE_SIZE" --workload single $B || exit 1
run single.sq "$SQ" --workload single $B || exit 1
run copy.fetch "FETCH_SIZE" --workload copy --steps 5 || exit 1
run copy.write "WRITE_SIZE" --workload copy --steps 5 || exit 1
run copy.tcc "$TCC" --workload copy --steps 5 || exit 1
