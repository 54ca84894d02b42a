"""Turn rocprofv3 CSV output of a bench.py run into the short summaries bench.py and the documentation quote.

    # per-kernel durations (text, to stdout)
    python -m paper_2503_16163_amd.profile_summary stats <dir written by rocprofv3 --kernel-trace --stats>

    # HBM bytes and vector instructions per launch (profiles/traffic.json, profiles/valu.json, text to stdout)
    python -m paper_2503_16163_amd.profile_summary counters --workload M0 \
        --fetch <dir of the --pmc FETCH_SIZE run> --write <dir of the --pmc WRITE_SIZE run> [--valu <dir of the SQ run>]

The counter runs profile `bench.py --calibrate-copy`, whose plain device copy of known size gives the factor
between what FETCH_SIZE / WRITE_SIZE read and bytes.  Every figure is stored with the hash of the sources its
kernel compiles from (paper_2503_16163_amd.build.kernel_source_hash); bench.py quotes a figure only for a kernel
whose sources still have that hash.  Host logic only: nothing here touches the GPU or the method's arithmetic."""
import argparse
import collections
import csv
import glob
import json
import os
import re
import sys

from . import build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
COPY_KERNEL = "__amd_rocclr_copyBuffer"
COPY_KIB = 262144.0   # bench.py --calibrate-copy copies 256 MiB device to device


def short_name(full):
    """'attend_i8_kernel+score' for the instantiation with the scoring pass in front, else the bare kernel name;
    None for kernels that are not this library's."""
    m = re.search(r"specache::\(anonymous namespace\)::(\w+)\s*(<([^>]*)>)?", full)
    if not m:
        return COPY_KERNEL if COPY_KERNEL in full else None
    name, targs = m.group(1), (m.group(3) or "")
    if name == "attend_i8_kernel" and targs.replace(" ", "").endswith("true"):
        return name + "+score"
    return name


def find(dir_, suffix):
    hits = sorted(glob.glob(os.path.join(dir_, "**", "*" + suffix), recursive=True))
    if not hits:
        sys.exit(f"no *{suffix} under {dir_}")
    return hits[0]


def stats(dir_):
    rows = list(csv.DictReader(open(find(dir_, "kernel_stats.csv"))))
    agg = collections.OrderedDict()
    for r in rows:
        n = short_name(r["Name"])
        if n is None or n == COPY_KERNEL:
            continue
        a = agg.setdefault(n, [0, 0.0, 1e30, 0.0])
        a[0] += int(r["Calls"])
        a[1] += float(r["TotalDurationNs"])
        a[2] = min(a[2], float(r["MinNs"]))
        a[3] = max(a[3], float(r["MaxNs"]))
    total = sum(a[1] for a in agg.values()) or 1.0
    print(f"{'kernel':32s} {'calls':>7s} {'avg us':>10s} {'min us':>10s} {'max us':>10s} {'share':>7s}")
    for n, a in sorted(agg.items(), key=lambda kv: -kv[1][1]):
        print(f"{n:32s} {a[0]:7d} {a[1] / a[0] / 1e3:10.2f} {a[2] / 1e3:10.2f} {a[3] / 1e3:10.2f} {100 * a[1] / total:6.1f}%")


def medians(dir_, counter):
    """-> ({kernel: median over its launches}, {kernel: launches}); for the plain copy kernel the largest launch
    (torch issues small copies through the same kernel; the calibration copy is the 256 MiB one)."""
    vals = collections.defaultdict(list)
    for r in csv.DictReader(open(find(dir_, "counter_collection.csv"))):
        if r["Counter_Name"] != counter:
            continue
        n = short_name(r["Kernel_Name"])
        if n is not None:
            vals[n].append(float(r["Counter_Value"]))
    return ({n: (max(v) if n == COPY_KERNEL else sorted(v)[len(v) // 2]) for n, v in vals.items()},
            {n: len(v) for n, v in vals.items()})


def hash_of(short):
    return build.kernel_source_hash(short.split("+")[0])


def update_json(fname, workload, table, extra):
    path = os.path.join(ROOT, "profiles", fname)
    try:
        d = json.load(open(path))
    except (OSError, ValueError):
        d = {}
    hashes = d.get("kernel_source_hash", {}) if isinstance(d.get("kernel_source_hash"), dict) else {}
    # tables without recorded hashes are from before the figures were attributed to sources: dropped
    d = {k: v for k, v in d.items() if not isinstance(v, dict) or k in hashes}
    d[workload] = table
    hashes[workload] = {n: hash_of(n) for n in table}
    d["kernel_source_hash"] = hashes
    d.update(extra)
    with open(path, "w") as f:
        json.dump(d, f, indent=1)
        f.write("\n")
    return path


def counters(a):
    fetch, n_f = medians(a.fetch, "FETCH_SIZE")
    write, _ = medians(a.write, "WRITE_SIZE")
    if COPY_KERNEL not in fetch or COPY_KERNEL not in write:
        sys.exit("the runs hold no plain device copy: profile bench.py with --calibrate-copy")
    ff, wf = COPY_KIB / fetch[COPY_KERNEL], COPY_KIB / write[COPY_KERNEL]
    print(f"calibration: the 256 MiB device copy ({COPY_KERNEL}) reads FETCH_SIZE = {fetch[COPY_KERNEL]:.1f} and WRITE_SIZE = "
          f"{write[COPY_KERNEL]:.1f} for {COPY_KIB:.0f} KiB each way: fetch_factor = {ff:.4f}, write_factor = {wf:.4f}")
    print("counters are KiB per dispatch, median over the launches of the run\n")
    print(f"{'kernel':32s} {'launches':>8s} {'FETCH_SIZE':>12s} {'WRITE_SIZE':>12s} {'HBM MB per launch':>18s}")
    table = {}
    per_step = max(c for n, c in n_f.items() if n != COPY_KERNEL) // 2   # launched at least every other layer-step: not the loading of the prompt
    for n in sorted(fetch):
        if n == COPY_KERNEL or n not in write or hash_of(n) is None:
            continue
        nbytes = int(round((fetch[n] * ff + write[n] * wf) * 1024))
        if n_f[n] >= per_step:
            table[n] = nbytes
        print(f"{n:32s} {n_f[n]:8d} {fetch[n]:12.1f} {write[n]:12.1f} {nbytes / 1e6:18.2f}"
              + ("" if n_f[n] >= per_step else "   (the prompt's load; not stored)"))
    p = update_json("traffic.json", a.workload, table, {
        "unit": "HBM bytes per launch (FETCH_SIZE * fetch_factor + WRITE_SIZE * write_factor, KiB -> bytes)",
        "fetch_factor": round(ff, 4), "write_factor": round(wf, 4),
        "calibration": f"256 MiB device copy issued by bench.py --calibrate-copy ({COPY_KERNEL})"})
    print(f"\nwrote {os.path.relpath(p, ROOT)}")
    if a.valu:
        insts, n_i = medians(a.valu, "SQ_INSTS_VALU")
        waves, _ = medians(a.valu, "SQ_WAVES")
        busy, _ = medians(a.valu, "SQ_BUSY_CYCLES")
        print(f"\n{'kernel':32s} {'launches':>8s} {'SQ_INSTS_VALU':>14s} {'SQ_WAVES':>10s} {'per wave':>9s}")
        vt = {}
        for n in sorted(insts):
            if n == COPY_KERNEL or hash_of(n) is None:
                continue
            if n_i[n] >= max(c for m, c in n_i.items() if m != COPY_KERNEL) // 2:
                vt[n] = int(insts[n])
            w = waves.get(n, 0.0)
            print(f"{n:32s} {n_i[n]:8d} {insts[n]:14.0f} {w:10.0f} {insts[n] / w if w else 0.0:9.1f}")
        p = update_json("valu.json", a.workload, vt, {"unit": "wave64 vector-ALU instructions per launch (SQ_INSTS_VALU)"})
        print(f"\nwrote {os.path.relpath(p, ROOT)}")


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    s = sub.add_parser("stats")
    s.add_argument("dir")
    c = sub.add_parser("counters")
    c.add_argument("--workload", required=True)
    c.add_argument("--fetch", required=True)
    c.add_argument("--write", required=True)
    c.add_argument("--valu")
    a = ap.parse_args()
    if a.cmd == "stats":
        stats(a.dir)
    else:
        counters(a)


if __name__ == "__main__":
    main()
