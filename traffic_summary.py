"""Turns two rocprofv3 counter runs (FETCH_SIZE, then WRITE_SIZE) of bench.py --calibrate
into HBM bytes per kernel launch, scaled by what the same counters read for the plain
copy kernel of known size (bra_util_copy, 64 MiB read + 64 MiB written per launch).

usage: python traffic_summary.py <dir FETCH run> <dir WRITE run> <workload name>
Prints the text kept as profiles/hbm_traffic.txt.
"""
from __future__ import annotations

import collections
import csv
import glob
import re
import sys

COPY_BYTES = 64 << 20
NAMES = {"k_fused": "mfma_fused_k1", "k_pool": "mfma_pool_qk", "k_route": "mfma_route_rows",
         "k_route_p": "mfma_route_rows", "k_route_u": "mfma_route_rows", "k_route_w": "mfma_route_rows",
         "k_attn_map": "mfma_attn_small", "k_attn_map4": "mfma_attn_small",
         "k_qkv": "mfma_qkv", "k_attn_big": "mfma_attention", "k_attn_q32": "mfma_attention", "k_attn_small": "mfma_attn_small",
         "k_small": "mfma_attn_small", "k_lce_add": "mfma_lce_add", "k_prep_weights": "mfma_prep",
         "k_token_ln": "block_ln", "k_mlp_fused64": "block_mlp_fused", "k_mlp_stream": "block_mlp_fused",
         "k_util_copy": "copy"}


def averages(directory, counter):
    acc = collections.defaultdict(list)
    for path in glob.glob(directory + "/**/*counter_collection.csv", recursive=True):
        for row in csv.DictReader(open(path)):
            if row["Counter_Name"] != counter:
                continue
            m = re.search(r"(k_[a-z0-9_]+)", row["Kernel_Name"])
            if m and m.group(1) in NAMES:
                name = NAMES[m.group(1)]
                if re.search(r"k_qkv<\d+, \d+, 1, \d+>", row["Kernel_Name"]):   # the same kernel with Wo as its only matrix
                    name = "mfma_wo"
                if m.group(1) == "k_token_ln":                               # position encoding (0) or residual (1) + LayerNorm
                    name = "block_pos_ln" if "k_token_ln<0" in row["Kernel_Name"] else "block_add_ln"
                acc[name].append(float(row["Counter_Value"]))
    return {k: sum(v) / len(v) for k, v in acc.items()}


def main():
    fetch_dir, write_dir, workload = sys.argv[1:4]
    fetch, write = averages(fetch_dir, "FETCH_SIZE"), averages(write_dir, "WRITE_SIZE")
    # counters are in KiB per dispatch; scale so that the copy kernel reads its known size
    f_scale = COPY_BYTES / (fetch["copy"] * 1024.0)
    w_scale = COPY_BYTES / (write["copy"] * 1024.0)
    print(f"# copy kernel: FETCH_SIZE {fetch['copy']:.0f} KiB, WRITE_SIZE {write['copy']:.0f} KiB per launch "
          f"for {COPY_BYTES} B each way -> scale factors {f_scale:.4f} (fetch), {w_scale:.4f} (write)")
    print("# columns: 'traffic' workload kernel bytes_per_launch (fetch_bytes write_bytes)")
    for k in sorted(set(fetch) | set(write)):
        if k == "copy":
            continue
        fb = fetch.get(k, 0.0) * 1024.0 * f_scale
        wb = write.get(k, 0.0) * 1024.0 * w_scale
        print(f"traffic {workload} {k} {fb + wb:.0f} {fb:.0f} {wb:.0f}")


if __name__ == "__main__":
    main()
