"""Summarise rocprofv3 --pmc passes (CSV output) per kernel as text.

    python -m paper_2110_09195_amd.devtools.pmcsum pass1/x_counter_collection.csv [pass2/...csv ...] > profiles/<name>.txt

Prints, per kernel whose name contains one of the wanted substrings (default: the library's kernels and the copy
probe), the number of dispatches and the mean per dispatch of every counter found in the files.
"""
import collections
import csv
import sys

WANTED = ("subbit_", "bnn_", "pack_", "dense_", "copy_kernel", "project")


def short(name):
    return name.replace("void ", "").replace("(anonymous namespace)::", "").replace("snn::", "").split("(")[0]


def main(paths, out=sys.stdout):
    per = collections.defaultdict(lambda: collections.defaultdict(list))
    for p in paths:
        with open(p) as fh:
            for row in csv.DictReader(fh):
                k = short(row["Kernel_Name"])
                if any(w in k for w in WANTED):
                    per[k][row["Counter_Name"]].append(float(row["Counter_Value"]))
    for k in sorted(per):
        n = max(len(v) for v in per[k].values())
        out.write("%s  (%d dispatches)\n" % (k, n))
        for c in sorted(per[k]):
            v = per[k][c]
            out.write("    %-34s %18.1f\n" % (c, sum(v) / len(v)))


if __name__ == "__main__":
    main(sys.argv[1:])
