"""Turns two rocprofv3 --pmc runs of bench.py (FETCH_SIZE, then WRITE_SIZE; csv output) into the HBM
traffic per launch of each kernel, scaled by what the same counters read for the plain copy kernel of
known size that `bench.py --calibrate-copy` runs.  Writes the JSON that bench.py reads for `traffic`.

    python -m paper_2601_12917_amd.pmc_summary FETCH_counter_collection.csv WRITE_counter_collection.csv COPY_BYTES out.json [VALU_counter_collection.csv]

The optional fifth argument is a run with SQ_INSTS_VALU among its counters: the vector instructions (wave64) per
launch of each kernel go into the same JSON, from which bench.py derives the instructions per Philox call.
"""
import collections
import csv
import json
import sys

from .build import source_digest


def per_kernel(path, counter):
    agg = collections.defaultdict(list)
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] != counter:
            continue
        name = r["Kernel_Name"].replace("zgr::(anonymous namespace)::", "").replace("void ", "").split("(")[0]
        agg[name].append(float(r["Counter_Value"]))
    return {k: (sum(v) / len(v), len(v)) for k, v in agg.items()}


def main(argv):
    fetch_csv, write_csv, copy_bytes, out = argv[1], argv[2], float(argv[3]), argv[4]
    f = per_kernel(fetch_csv, "FETCH_SIZE")
    w = per_kernel(write_csv, "WRITE_SIZE")
    # counters are in KiB; the copy kernel reads and writes copy_bytes
    f_scale = copy_bytes / (f["copy_kernel"][0] * 1024.0)
    w_scale = copy_bytes / (w["copy_kernel"][0] * 1024.0)
    kernels = {}
    for k in f:
        if k in w:
            kernels[k] = {"launches": f[k][1], "fetch_bytes": f[k][0] * 1024.0 * f_scale, "write_bytes": w[k][0] * 1024.0 * w_scale}
    if len(argv) > 5:
        for k, (val, _) in per_kernel(argv[5], "SQ_INSTS_VALU").items():
            if k in kernels:
                kernels[k]["valu_insts"] = val
    json.dump({"source_digest": source_digest(), "fetch_scale": f_scale, "write_scale": w_scale, "copy_bytes": copy_bytes,
               "kernels": kernels}, open(out, "w"), indent=1)
    for k, v in sorted(kernels.items(), key=lambda kv: -kv[1]["fetch_bytes"] * kv[1]["launches"]):
        print(f"{k:60s} launches {v['launches']:5d}  fetch {v['fetch_bytes'] / 1e6:10.1f} MB  write {v['write_bytes'] / 1e6:10.1f} MB")
    print("scale factors: fetch", f_scale, "write", w_scale)


if __name__ == "__main__":
    main(sys.argv)
