"""Turn two rocprofv3 --pmc runs of bench.py into profiles/traffic.json (HBM bytes per launch).

bench.py's `roofline.traffic` is the HBM traffic of the dominant kernel as the hardware counters
see it.  It cannot be measured inside bench.py (counters need the profiler), so it is measured by
this profiling step and kept in a small tracked file that bench.py reads -- and refuses when the
kernel named in it is no longer the kernel bench.py measures.

Two runs, one counter each (rocprofv3 does not split counters over passes; no tracing options):

    cd /tmp && export TMPDIR=/tmp
    rocprofv3 --pmc FETCH_SIZE --output-format csv -d gpurun_out/pmc_f -o f -- \
        python3 bench.py --workload cfg5 --steps 10 --warmup 2 --no-cpu --no-ttg --no-others --copy-calibration-gib 4
    rocprofv3 --pmc WRITE_SIZE --output-format csv -d gpurun_out/pmc_w -o w -- \
        python3 bench.py --workload cfg5 --steps 10 --warmup 2 --no-cpu --no-ttg --no-others --copy-calibration-gib 4
    python3 pmc_traffic.py --workload cfg5 --fetch gpurun_out/pmc_f --write gpurun_out/pmc_w

--copy-calibration-gib appends plain device copies of known size; the largest copy dispatch gives
the factor between a counter's unit and KiB (FETCH_SIZE has read 2 KiB per count and WRITE_SIZE
1 KiB per count on the machines used so far; the factors found are stored with the result).
"""
import argparse
import collections
import csv
import glob
import json
import os
import re

ROOT = os.path.dirname(os.path.abspath(__file__))
TRAFFIC = os.path.join(ROOT, "profiles", "traffic.json")

# dominant kernels per kind of workload: (name in bench.py's roofline objects, regular expressions that
# pick their dispatches out of the profiler's kernel names)
GAP_KERNELS = {"dense": ["gap_dense_kernel"], "sparse": ["csr_sliced_dot_kernel", "csr_blocked_finish_kernel"]}
CD_KERNELS = {"dense": ["cd_dense_worker_kernel", "merge_workers_kernel"], "sparse": ["cd_csr_plan_kernel", "cd_csr_async_kernel"]}


def per_kernel(path, counter):
    """{short kernel name: [value per dispatch]} from the *_counter_collection.csv under path."""
    files = glob.glob(os.path.join(path, "**", "*counter_collection.csv"), recursive=True)
    if not files:
        raise SystemExit(f"no *_counter_collection.csv under {path}")
    out = collections.defaultdict(list)
    for f in files:
        for r in csv.DictReader(open(f)):
            if r["Counter_Name"] != counter:
                continue
            name = r["Kernel_Name"].replace("duhl::(anonymous namespace)::", "duhl::").replace("void ", "")
            out[re.sub(r"\(.*", "", name)].append(float(r["Counter_Value"]))
    return out


def pick(values, short, exclude=None):
    """Dispatches whose kernel is duhl::<short>..., optionally leaving some template instances out."""
    got = []
    for name, v in values.items():
        if re.match(r"duhl::" + re.escape(short) + r"\b", name) and not (exclude and re.search(exclude, name)):
            got += v
    return got


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", required=True)
    ap.add_argument("--kind", default="dense", choices=["dense", "sparse"])
    ap.add_argument("--fetch", required=True, help="output directory of the FETCH_SIZE run")
    ap.add_argument("--write", required=True, help="output directory of the WRITE_SIZE run")
    ap.add_argument("--calibration-gib", type=float, default=4.0)
    ap.add_argument("--passes-per-round", type=int, default=1)
    args = ap.parse_args()
    fetch, write = per_kernel(args.fetch, "FETCH_SIZE"), per_kernel(args.write, "WRITE_SIZE")
    kib = args.calibration_gib * (1 << 20)
    f_unit = kib / max(max(v) for k, v in fetch.items() if "copyBuffer" in k)      # KiB per count
    w_unit = kib / max(max(v) for k, v in write.items() if "copyBuffer" in k)
    entry = {"calibration": {"copy_GiB": args.calibration_gib, "FETCH_SIZE_KiB_per_count": round(f_unit, 4),
                             "WRITE_SIZE_KiB_per_count": round(w_unit, 4)}}

    def launch_bytes(short, exclude=None):
        f, w = pick(fetch, short, exclude), pick(write, short, exclude)
        if not f or not w:
            raise SystemExit(f"kernel {short} not found in the counter files")
        return (sum(f) / len(f) * f_unit + sum(w) / len(w) * w_unit) * 1024.0, len(f)

    # the gap pass: one launch per kernel named (the instance that also computes the norms is set_data's)
    gap = 0.0
    for short in GAP_KERNELS[args.kind]:
        b, _ = launch_bytes(short, exclude=r"true>$" if short == "gap_dense_kernel" else None)
        gap += b
    entry["gap"] = {"kernels": GAP_KERNELS[args.kind], "bytes_per_launch": gap}
    # a CD pass: its kernels' dispatches per pass, counted against the selections (one per round)
    rounds = len(pick(fetch, "select_fused_kernel"))
    total = 0.0
    for short in CD_KERNELS[args.kind]:
        b, count = launch_bytes(short)
        total += b * count / max(rounds * args.passes_per_round, 1)
    entry["cd_pass"] = {"kernels": CD_KERNELS[args.kind], "bytes_per_pass": total}
    data = {}
    if os.path.exists(TRAFFIC):
        data = json.load(open(TRAFFIC))
    data[args.workload] = entry
    with open(TRAFFIC, "w") as f:
        json.dump(data, f, indent=1, sort_keys=True)
        f.write("\n")
    print(json.dumps({args.workload: entry}, indent=1))


if __name__ == "__main__":
    main()
