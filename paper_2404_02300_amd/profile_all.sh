#!/bin/bash
# Measurement pass on the GPU machine, run from the repository root:
#   bash paper_2404_02300_amd/profile_all.sh [workload ...]
# For every workload: bench.py on its own, then under rocprofv3 for a kernel trace, the two HBM traffic
# counters (each a run of its own) and, where matrix cores matter, MfmaUtil.  Raw output goes to
# gpurun_out/; `python -m paper_2404_02300_amd.profile_summary` turns it into profiles/*.txt and
# profiles/traffic.json afterwards (see the end of this file for the calls).
set -o pipefail
R=$PWD
O=$R/gpurun_out
W="${@:-dense products sparse_bf16 fullgraph sampling gather}"
args_of() {
  case $1 in
    fullgraph|sampling|gather) echo "--workload $1 --steps 6 --warmup 2 --no-cpu-baseline" ;;
    *) echo "--workload $1 --also none --steps 10 --warmup 2 --reps 1 --no-cpu-baseline --serial" ;;
  esac
}
for w in $W; do
  echo "== bench $w"; timeout -k 10 400 python3 -u bench.py --workload $w --also none --no-cpu-baseline > $O/bench_$w.json 2> $O/bench_$w.err; rc=$?
  tail -1 $O/bench_$w.err; [ $rc -eq 0 ] || exit $rc
done
cd /tmp && export TMPDIR=/tmp
for w in $W; do
  a=$(args_of $w)
  echo "== trace $w"; rm -rf $O/prof_$w
  timeout -k 10 300 rocprofv3 --kernel-trace --stats --output-format csv -d $O/prof_$w -o trace -- python3 $R/bench.py $a > $O/prof_$w.log 2>&1; rc=$?
  tail -1 $O/prof_$w.log; [ $rc -eq 0 ] || exit $rc
  for c in FETCH_SIZE WRITE_SIZE; do
    echo "== pmc $c $w"; rm -rf $O/pmc_${c}_$w
    timeout -s KILL 240 rocprofv3 --pmc $c --output-format csv -d $O/pmc_${c}_$w -o pmc -- python3 $R/bench.py $a --calibrate-copy > $O/pmc_${c}_$w.log 2>&1; rc=$?
    tail -1 $O/pmc_${c}_$w.log; [ $rc -eq 0 ] || exit $rc
  done
  case $w in dense|fullgraph|sparse_bf16|products)
    echo "== pmc MfmaUtil $w"; rm -rf $O/pmc_MfmaUtil_$w
    timeout -s KILL 240 rocprofv3 --pmc MfmaUtil --output-format csv -d $O/pmc_MfmaUtil_$w -o pmc -- python3 $R/bench.py $a > $O/pmc_MfmaUtil_$w.log 2>&1; rc=$?
    tail -1 $O/pmc_MfmaUtil_$w.log; [ $rc -eq 0 ] || exit $rc ;;
  esac
done
# afterwards, in the repository root (CPU only), for each workload w:
#   python -m paper_2404_02300_amd.profile_summary w --trace gpurun_out/prof_w --fetch gpurun_out/pmc_FETCH_SIZE_w \
#          --write gpurun_out/pmc_WRITE_SIZE_w [--mfma gpurun_out/pmc_MfmaUtil_w] --bench gpurun_out/bench_w.json \
#          --command "<the bench.py arguments printed by args_of above>"
