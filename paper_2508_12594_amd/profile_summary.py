"""Condense rocprofv3 CSV output into the short text summaries kept under profiles/.

    python -m paper_2508_12594_amd.profile_summary kernels <dir>    # after --kernel-trace --stats
    python -m paper_2508_12594_amd.profile_summary counters <dir>   # after --pmc ...

`<dir>` is the rocprofv3 output directory (-d); every *_kernel_stats.csv / *_kernel_trace.csv /
*_counter_collection.csv below it is read.  Only flare kernels and plain copy kernels are listed.
"""
import collections
import csv
import glob
import os
import sys


def _short(name):
    for key in ("encode_mfma_kernel", "decode_mfma_kernel", "bwd_dq_mfma_kernel", "bwd_dkdv_mfma_kernel",
                "encode_merge_kernel", "dz_merge_kernel", "dq_reduce_kernel", "encode_partial_kernel",
                "token_pass_kernel", "dz_partial_kernel", "dq_partial_kernel", "dkdv_kernel",
                "bwd_prep_kernel"):
        if key in name:
            args = name[name.index(key) + len(key):]
            tmpl = args[:args.index(">") + 1] if args.startswith("<") and ">" in args else ""
            return key + tmpl
    if "copy" in name.lower() or "elementwise" in name.lower():
        return "copy/elementwise (torch)"
    return None


def kernels(root):
    rows = collections.defaultdict(list)
    for path in glob.glob(os.path.join(root, "**", "*kernel_trace.csv"), recursive=True):
        for r in csv.DictReader(open(path)):
            name = _short(r["Kernel_Name"])
            if name:
                rows[name].append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) * 1e-3)
    print("%-58s %7s %12s %12s %12s" % ("kernel", "calls", "mean us", "min us", "max us"))
    for name, d in sorted(rows.items(), key=lambda kv: -sum(kv[1])):
        print("%-58s %7d %12.2f %12.2f %12.2f" % (name, len(d), sum(d) / len(d), min(d), max(d)))


def counters(root):
    rows = collections.defaultdict(lambda: collections.defaultdict(list))
    for path in glob.glob(os.path.join(root, "**", "*counter_collection.csv"), recursive=True):
        for r in csv.DictReader(open(path)):
            name = _short(r["Kernel_Name"])
            if name:
                rows[name][r["Counter_Name"]].append(float(r["Counter_Value"]))
    print("%-58s %-28s %9s %16s" % ("kernel", "counter", "dispatches", "mean per dispatch"))
    for name, cs in sorted(rows.items()):
        for c, v in sorted(cs.items()):
            print("%-58s %-28s %9d %16.6g" % (name, c, len(v), sum(v) / len(v)))


if __name__ == "__main__":
    if len(sys.argv) != 3 or sys.argv[1] not in ("kernels", "counters"):
        print(__doc__)
        sys.exit(2)
    (kernels if sys.argv[1] == "kernels" else counters)(sys.argv[2])
