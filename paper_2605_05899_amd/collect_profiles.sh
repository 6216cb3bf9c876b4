#!/bin/bash
# Runs on a GPU machine from the repository root: the rocprofv3 passes behind the summaries kept under profiles/.
# Every rocprofv3 line runs committed files only (bench.py and the built library). Raw output goes to the directory
# named by PROF_OUT (default prof_raw under the repository root);
# `python -m paper_2605_05899_amd.profile_summary regen <that directory>` turns it into profiles/.
# Counters are collected in runs of their own (one counter block per run, no tracing alongside).
set -o pipefail
R=${GRAFT_REPO_ROOT:-$(pwd)}
cd /tmp && export TMPDIR=/tmp
O=${PROF_OUT:-$R/prof_raw}; case $O in /*) ;; *) O=$R/$O;; esac; rm -rf $O; mkdir -p $O
for W in ${WORKLOADS:-C4 C5 C3}; do
  B="python3 $R/bench.py --config $W --no-cpu-baseline --no-also"
  timeout -s KILL 300 rocprofv3 --kernel-trace --stats -d $O/${W}_trace -o t --output-format csv -- $B --steps 50 --warmup 10 > $O/${W}_trace.log 2>&1 || exit 1
  echo $W trace done
  timeout -s KILL 200 rocprofv3 --pmc FETCH_SIZE -d $O/${W}_fetch -o p --output-format csv -- $B --steps 5 --warmup 2 --calib-copy > $O/${W}_fetch.log 2>&1 || exit 2
  timeout -s KILL 200 rocprofv3 --pmc WRITE_SIZE -d $O/${W}_write -o p --output-format csv -- $B --steps 5 --warmup 2 --calib-copy > $O/${W}_write.log 2>&1 || exit 3
  echo $W traffic done
  timeout -s KILL 200 rocprofv3 --pmc SQ_BUSY_CYCLES SQ_WAVE_CYCLES SQ_VALU_MFMA_BUSY_CYCLES SQ_INSTS_VALU_MFMA_MOPS_BF16 SQ_LDS_BANK_CONFLICT SQ_ACTIVE_INST_LDS SQ_WAIT_INST_ANY SQ_WAIT_INST_LDS -d $O/${W}_sq -o p --output-format csv -- $B --steps 5 --warmup 2 > $O/${W}_sq.log 2>&1 || exit 4
  timeout -s KILL 200 rocprofv3 --pmc TCC_HIT_sum TCC_MISS_sum TCC_REQ_sum GRBM_GUI_ACTIVE -d $O/${W}_tcc -o p --output-format csv -- $B --steps 5 --warmup 2 > $O/${W}_tcc.log 2>&1 || exit 5
  echo $W counters done
done
B="python3 $R/bench.py --config P2 --no-cpu-baseline"
timeout -s KILL 200 rocprofv3 --kernel-trace --stats -d $O/P2_trace -o t --output-format csv -- $B --steps 200 --warmup 10 > $O/P2_trace.log 2>&1 || exit 6
echo P2 trace done
B="python3 $R/bench.py --config P3 --no-cpu-baseline"
timeout -s KILL 200 rocprofv3 --kernel-trace --stats -d $O/P3_trace -o t --output-format csv -- $B --steps 200 --warmup 10 > $O/P3_trace.log 2>&1 || exit 8
echo P3 trace done
B="python3 $R/bench.py --config PF"
timeout -s KILL 200 rocprofv3 --kernel-trace --stats -d $O/PF_trace -o t --output-format csv -- $B --steps 200 --warmup 10 > $O/PF_trace.log 2>&1 || exit 7
echo PF trace done
# keep what comes back small: the CSVs the summariser reads
find $O -type f ! -name '*.csv' ! -name '*.log' -delete
