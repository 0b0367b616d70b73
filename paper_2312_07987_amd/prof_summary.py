"""Turns rocprofv3 CSV output into the short text summaries kept under profiles/.

    python -m paper_2312_07987_amd.prof_summary stats  <kernel_stats.csv>            > profiles/x.txt
    python -m paper_2312_07987_amd.prof_summary pmc    <counter_collection.csv> NAME > profiles/y.txt

`stats`: per-kernel calls / average / share from `rocprofv3 --kernel-trace --stats`.
`pmc`:   per-kernel average of counter NAME per dispatch from `rocprofv3 --pmc NAME`.
"""
import collections
import csv
import sys


def stats(path, top=40):
    rows = list(csv.DictReader(open(path)))
    print("%-110s %6s %10s %7s" % ("kernel", "calls", "avg_us", "pct"))
    for r in rows[:top]:
        print("%-110s %6s %10.1f %7.2f" % (r["Name"][:110], r["Calls"], float(r["AverageNs"]) / 1e3, float(r["Percentage"])))


def pmc(path, name):
    tot = collections.defaultdict(float)
    cnt = collections.Counter()
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] != name:
            continue
        tot[r["Kernel_Name"]] += float(r["Counter_Value"])
        cnt[r["Kernel_Name"]] += 1
    print("%-110s %6s %14s" % ("kernel", "calls", name + "/dispatch"))
    for k in sorted(tot, key=lambda k: -tot[k]):
        print("%-110s %6d %14.1f" % (k[:110], cnt[k], tot[k] / cnt[k]))


if __name__ == "__main__":
    if sys.argv[1] == "stats":
        stats(sys.argv[2])
    else:
        pmc(sys.argv[2], sys.argv[3])
