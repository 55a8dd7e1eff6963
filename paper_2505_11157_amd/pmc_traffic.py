"""HBM bytes per kernel launch from rocprofv3 counter files -> profiles/hbm_traffic.json (read by bench.py).

Counters: FETCH_SIZE and WRITE_SIZE (KiB per dispatch), one `rocprofv3 --pmc` run each, scaled by what the same
counter reads for a device-to-device copy of known size (`bench.py --copy-calibration`: 1 GiB per copy).

    cd /tmp && export TMPDIR=/tmp
    rocprofv3 --pmc FETCH_SIZE --output-format csv -d $OUT/cal_fetch -o t -- python3 $REPO/bench.py --copy-calibration
    rocprofv3 --pmc WRITE_SIZE --output-format csv -d $OUT/cal_write -o t -- python3 $REPO/bench.py --copy-calibration
    rocprofv3 --pmc FETCH_SIZE --output-format csv -d $OUT/fetch3 -o t -- python3 $REPO/bench.py --config 3 \
        --steps 2 --warmup 1 --no-cpu-baseline --no-workloads          (and WRITE_SIZE -> $OUT/write3; same per workload)
    python3 -m paper_2505_11157_amd.pmc_traffic --cal $OUT/cal_fetch $OUT/cal_write \
        --cfg 3 $OUT/fetch3 $OUT/write3 [--cfg 4 ...] --out profiles/hbm_traffic.json

Kernel names are mapped from the C++ names in the counter files to the names the library's launch trace reports
(which is what bench.py keys its `roofline.traffic` lookup by).
"""
import argparse
import collections
import csv
import glob
import json
import os
import re

COPY_BYTES = 1 << 30


def trace_name(cxx):
    """C++ kernel name of a counter file -> name in the library's launch trace."""
    n = cxx.replace("(anonymous namespace)::", "").replace("void ", "").split("(")[0].strip()
    m = re.match(r"(\w+)<(.*)>$", n)
    if not m:
        return n
    base, args = m.group(1), [a.strip() for a in m.group(2).split(",")]
    waves = {"nattn_fwd_tiled": 2, "nattn_bwd_dq_tiled": 1, "nattn_bwd_dkdv_tiled": 0, "nattn_bwd_dkdv2_tiled": 0}
    if base in waves:
        w = args[waves[base]]
        up = len(args) > waves[base] + 1 and args[waves[base] + 1] == "true"
        label = "8 waves" if w == "8" else "1 wave"
        if up and base != "nattn_fwd_tiled":
            label += ", classes"
        return "%s<%s>" % (base, label)
    return base


def per_kernel(directory, counter):
    """Mean counter value per dispatch, by trace name."""
    files = glob.glob(os.path.join(directory, "**", "*counter_collection.csv"), recursive=True)
    if not files:
        raise SystemExit("no *counter_collection.csv under %s" % directory)
    acc = collections.defaultdict(list)
    for f in files:
        for r in csv.DictReader(open(f)):
            if r["Counter_Name"] == counter:
                acc[trace_name(r["Kernel_Name"])].append(float(r["Counter_Value"]))
    return {k: sum(v) / len(v) for k, v in acc.items()}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--cal", nargs=2, metavar=("FETCH_DIR", "WRITE_DIR"), required=True)
    ap.add_argument("--cfg", nargs=3, action="append", metavar=("N", "FETCH_DIR", "WRITE_DIR"), default=[])
    ap.add_argument("--out", default=os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))),
                                                   "profiles", "hbm_traffic.json"))
    args = ap.parse_args()
    copy = lambda d, c: next(v for k, v in per_kernel(d, c).items() if "copyBuffer" in k or "copy" in k.lower())
    cal_f, cal_w = copy(args.cal[0], "FETCH_SIZE"), copy(args.cal[1], "WRITE_SIZE")
    kf, kw = COPY_BYTES / 1024.0 / cal_f, COPY_BYTES / 1024.0 / cal_w
    res = {"calibration": {"copy_bytes": COPY_BYTES, "FETCH_SIZE_KiB": cal_f, "WRITE_SIZE_KiB": cal_w,
                           "fetch_scale": kf, "write_scale": kw},
           "bytes_per_launch": {}, "read_write_MB": {}}
    for n, fd, wd in args.cfg:
        f, w = per_kernel(fd, "FETCH_SIZE"), per_kernel(wd, "WRITE_SIZE")
        keep = [k for k in f if k.startswith(("nattn_", "global_", "prepare_", "disco_", "s2_", "mha_"))]
        res["bytes_per_launch"][n] = {k: (f[k] * kf + w.get(k, 0.0) * kw) * 1024.0 for k in keep}
        res["read_write_MB"][n] = {k: [round(f[k] * kf * 1024.0 / 1e6, 1), round(w.get(k, 0.0) * kw * 1024.0 / 1e6, 1)] for k in keep}
    with open(args.out, "w") as fo:
        json.dump(res, fo, indent=1, sort_keys=True)
        fo.write("\n")
    print(json.dumps(res["read_write_MB"], indent=1))


if __name__ == "__main__":
    main()
