"""Turns rocprofv3 counter runs of bench.py into profiles/hbm_traffic.json, the file bench.py reads its
`roofline.traffic` from.

For every workload two runs are expected, each made as

    rocprofv3 --pmc FETCH_SIZE -d <dir>/<workload>_FETCH_SIZE -o p --output-format csv -- \
        python3 bench.py --only --workload <workload> --steps 5 --warmup 2 --no-cpu-baseline --calibrate-copy

(and the same with WRITE_SIZE).  `--calibrate-copy` adds three launches of the library's plain copy kernel
over 1 GiB: what a counter reads for those known bytes fixes its scale (FETCH_SIZE counts in units that differ
from KiB by a constant factor on this chip).  The result is the mean over the decode-attention launches of a
run, scaled, read plus written, in bytes per launch, stored with a hash of the kernel sources: bench.py reports
`traffic: null` once those sources have changed.

    python3 -m paper_2603_12831_amd.hbm_traffic <dir>        # prints a table and rewrites the file
"""
import collections
import csv
import json
import os
import re
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
COPY_BYTES = 1 << 30
WORKLOAD_NAMES = {"cfg2": "cfg2-mha-b64", "cfg3": "cfg3-gqa-b256", "cfg4": "cfg4-hybrid-32ls-224be",
                  "cfg5": "cfg5-long-b32-L32768"}
# (the fused instance, which bench.py also runs on the hybrid batch, is a different kernel: left out)
DECODE = re.compile(r"decode_(mfma_persistent_kernel<false|mfma_grid_kernel|vector_kernel)")


def mean_per_kernel(path):
    acc = collections.defaultdict(list)
    with open(path) as f:
        for r in csv.DictReader(f):
            k = r["Kernel_Name"]
            key = "copy" if "copy_kernel" in k else "decode" if DECODE.search(k) else None
            if key:
                acc[key].append(float(r["Counter_Value"]))
    return {k: sum(v) / len(v) for k, v in acc.items()}, {k: len(v) for k, v in acc.items()}


def main(argv):
    if len(argv) != 2:
        print(__doc__)
        return 2
    sys.path.insert(0, ROOT)
    import bench

    out = {}
    for short, name in WORKLOAD_NAMES.items():
        total, parts = 0.0, {}
        for ctr in ("FETCH_SIZE", "WRITE_SIZE"):
            path = os.path.join(argv[1], "%s_%s" % (short, ctr), "p_counter_collection.csv")
            if not os.path.isfile(path):
                parts = None
                break
            mean, n = mean_per_kernel(path)
            if "copy" not in mean or "decode" not in mean:
                parts = None
                break
            scale = COPY_BYTES / mean["copy"]            # bytes per counter unit
            parts[ctr] = (mean["decode"], mean["copy"], n["decode"], mean["decode"] * scale)
            total += mean["decode"] * scale
        if parts is None:
            print("%s: counter runs missing or incomplete, left out" % short)
            continue
        out[name] = int(round(total))
        print("%-24s FETCH_SIZE %.1f (copy %.1f, %d launches) -> %.1f MB; WRITE_SIZE %.1f (copy %.1f) -> %.1f MB;"
              " total %d B" % (name, parts["FETCH_SIZE"][0], parts["FETCH_SIZE"][1], parts["FETCH_SIZE"][2],
                               parts["FETCH_SIZE"][3] / 1e6, parts["WRITE_SIZE"][0], parts["WRITE_SIZE"][1],
                               parts["WRITE_SIZE"][3] / 1e6, out[name]))
    with open(bench.TRAFFIC_FILE, "w") as f:
        json.dump({"kernel_source_hash": bench.kernel_source_hash(), "bytes_per_launch": out}, f, indent=1)
        f.write("\n")
    print("wrote", bench.TRAFFIC_FILE)
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
