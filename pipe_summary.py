"""Turns one rocprofv3 counter run of bench.py into per-kernel pipe utilisation figures.

Counters (one pass, 8 SQ counters): SQ_VALU_MFMA_BUSY_CYCLES SQ_ACTIVE_INST_VALU SQ_INSTS_VALU
SQ_BUSY_CYCLES SQ_WAVE_CYCLES SQ_WAIT_INST_ANY SQ_INSTS_LDS SQ_LDS_BANK_CONFLICT.

usage: python pipe_summary.py <dir of the counter run> <workload name> <file with a bench line>
The bench line comes from a run WITHOUT counters (under --pmc the profiler serialises the launches
and the event times grow by 100 us); it may be the line of another workload, whose `other_workloads`
entry is then used.  Prints the text kept as profiles/pipe_utilisation.txt: per kernel the average
duration that bench.py measured with events, and
  mfma   = SQ_VALU_MFMA_BUSY_CYCLES / (1024 SIMDs x duration x 2.4 GHz): matrix-core busy cycles (the
           counter adds up the SIMDs: 16 cycles per 16x16x32 bf16 product) against the peak clock;
  valu   = 4 x SQ_ACTIVE_INST_VALU / (1024 x duration x 2.4 GHz): vector-ALU issue cycles likewise
           (the counter is in units of 4 cycles, one wave64 instruction);
  waves  = 4 x SQ_WAVE_CYCLES / (1024 x duration x 2.4 GHz): average resident wavefronts per SIMD;
  wait   = SQ_WAIT_INST_ANY / SQ_WAVE_CYCLES: share of wavefront time spent waiting on any instruction;
  clock  = SQ_BUSY_CYCLES / 32 shader engines / duration: the clock the counters imply.
"""
from __future__ import annotations

import collections
import csv
import glob
import json
import re
import sys

from traffic_summary import NAMES

MORE = {"k_gemm": "gemm", "k_token_ln": "block_ln", "k_mlp_fused64": "block_mlp_fused", "k_mlp_stream": "block_mlp_fused",
        "k_attn_gen": "mfma_attention", "k_pool_wide": "mfma_pool_qk", "k_route_qk": "mfma_route_rows"}
SIMDS, PEAK_HZ, ENGINES = 1024, 2.4e9, 32


def main():
    directory, workload, line_file = sys.argv[1:4]
    line = json.loads(open(line_file).read().strip().splitlines()[-1])
    if line["config"]["workload"].startswith(workload):
        durations = {k: v["avg_us"] for k, v in line["kernels"].items()}
    else:
        durations = dict(line["other_workloads"][workload]["kernels_avg_us"])
    acc = collections.defaultdict(lambda: collections.defaultdict(list))
    for path in glob.glob(directory + "/**/*counter_collection.csv", recursive=True):
        for row in csv.DictReader(open(path)):
            m = re.search(r"(k_[a-z0-9_]+)", row["Kernel_Name"])
            if not m:
                continue
            name = NAMES.get(m.group(1)) or MORE.get(m.group(1))
            if re.search(r"k_qkv<\d+, \d+, 1, \d+>", row["Kernel_Name"]):
                name = "mfma_wo"
            if name:
                acc[name][row["Counter_Name"]].append(float(row["Counter_Value"]))
    print(f"# workload: {workload}")
    print("# columns: 'pipes' workload kernel avg_us mfma valu waves wait clock_GHz")
    for name, avg_us in durations.items():
        c = {k: sum(v) / len(v) for k, v in acc.get(name, {}).items()}
        if not c:
            continue
        cycles = avg_us * 1e-6 * PEAK_HZ * SIMDS
        print(f"pipes {workload} {name} {avg_us:.2f} {c['SQ_VALU_MFMA_BUSY_CYCLES'] / cycles:.3f} "
              f"{4 * c['SQ_ACTIVE_INST_VALU'] / cycles:.3f} {4 * c['SQ_WAVE_CYCLES'] / cycles:.2f} "
              f"{c['SQ_WAIT_INST_ANY'] / c['SQ_WAVE_CYCLES']:.2f} "
              f"{c['SQ_BUSY_CYCLES'] / ENGINES / (avg_us * 1e-6) / 1e9:.2f}")


if __name__ == "__main__":
    main()
