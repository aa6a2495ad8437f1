"""Reduce a rocprofv3 counter-collection CSV to one line per (kernel, grid, counter).

    python -m paper_2601_10155_amd.counters <x_counter_collection.csv> [<summary.csv>]

rocprofv3 --pmc writes one row per dispatch and counter; a run of bench.py makes tens of thousands
of them (hundreds of megabytes).  This keeps, for the library's kernels only, the number of
dispatches and the mean / minimum / maximum of each counter: the figures the summaries under
profiles/ quote.  Units are the counters' own (FETCH_SIZE and WRITE_SIZE: see the calibration
against lookat::stream_read_kernel, a plain read of known size, in those summaries).
"""
import collections
import csv
import re
import sys


def summarise(path):
    acc = collections.OrderedDict()
    with open(path, newline="") as f:
        for r in csv.DictReader(f):
            name = r["Kernel_Name"]
            if "lookat" not in name:
                continue
            short = re.sub(r"\(.*", "", name).replace("void ", "")
            key = (short, r["Grid_Size"], r["Workgroup_Size"], r["Counter_Name"])
            v = float(r["Counter_Value"])
            a = acc.setdefault(key, [0, 0.0, v, v])
            a[0] += 1
            a[1] += v
            a[2] = min(a[2], v)
            a[3] = max(a[3], v)
    lines = ["kernel,grid,wg,counter,dispatches,mean,min,max"]
    for (n, g, w, c), (cnt, tot, mn, mx) in acc.items():
        lines.append(f'"{n}",{g},{w},{c},{cnt},{tot / cnt:.6g},{mn:.6g},{mx:.6g}')
    return "\n".join(lines) + "\n"


def main(argv):
    if len(argv) < 2:
        print(__doc__)
        return 2
    text = summarise(argv[1])
    if len(argv) > 2:
        with open(argv[2], "w") as f:
            f.write(text)
    sys.stdout.write(text)
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
