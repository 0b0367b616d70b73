"""Turns rocprofv3 CSV output into the short text summaries kept under profiles/.

    python -m paper_2312_07987_amd.prof_summary stats  <kernel_stats.csv>            > profiles/x.txt
    python -m paper_2312_07987_amd.prof_summary pmc    <counter_collection.csv> NAME > profiles/y.txt

    python -m paper_2312_07987_amd.prof_summary traffic <fetch.csv> <write.csv> <copy_fetch.csv> <copy_write.csv> > profiles/t.json

`stats`:   per-kernel calls / average / share from `rocprofv3 --kernel-trace --stats`.
`pmc`:     per-kernel average of counter NAME per dispatch from `rocprofv3 --pmc NAME`.
`mfma`:    python -m paper_2312_07987_amd.prof_summary mfma <counter_collection.csv>: matrix-core
           utilisation per kernel from one `rocprofv3 --pmc SQ_VALU_MFMA_BUSY_CYCLES GRBM_GUI_ACTIVE` run
           = busy cycles (summed over the chip's 1024 SIMDs) / (active cycles, which rocprofv3 reports
           summed over the 8 XCDs, x 128 SIMDs per XCD).
`traffic_table`: python -m paper_2312_07987_amd.prof_summary traffic_table <traffic.json>: that JSON as a table.
`traffic`: HBM bytes per dispatch of every kernel as JSON, from a `--pmc FETCH_SIZE` and a
           `--pmc WRITE_SIZE` run of the benchmark (counters in KiB), each scaled by what the same
           counter reads for `bench.py --copy-only` (a 256 MiB device copy, 5 launches).
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


def _avg(path, name):
    tot = collections.defaultdict(float)
    cnt = collections.Counter()
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] == name:
            tot[r["Kernel_Name"]] += float(r["Counter_Value"])
            cnt[r["Kernel_Name"]] += 1
    return {k: tot[k] / cnt[k] for k in tot}


def _source_hash():
    """sha256 (first 16 hex digits) of the kernel sources the figures were taken with; bench.py quotes a figure
    only while the sources still hash to this."""
    import hashlib
    import os
    d = os.path.join(os.path.dirname(os.path.abspath(__file__)), "csrc")
    h = hashlib.sha256()
    for n in sorted(os.listdir(d)):
        if n.endswith((".hip", ".h")):
            h.update(open(os.path.join(d, n), "rb").read())
    return h.hexdigest()[:16]


def traffic(fetch, write, copy_fetch, copy_write, copy_bytes=256 << 20):
    import json
    cf = _avg(copy_fetch, "FETCH_SIZE")
    cw = _avg(copy_write, "WRITE_SIZE")
    kf = [k for k in cf if "copyBuffer" in k or "copy" in k.lower()]
    kw = [k for k in cw if "copyBuffer" in k or "copy" in k.lower()]
    sf = copy_bytes / (cf[kf[0]] * 1024.0)   # true bytes per counted KiB-unit, reads
    sw = copy_bytes / (cw[kw[0]] * 1024.0)
    f = _avg(fetch, "FETCH_SIZE")
    w = _avg(write, "WRITE_SIZE")
    out = {"source_sha16": _source_hash(), "fetch_scale": sf, "write_scale": sw, "copy_kernel": kf[0], "kernels": {}}
    for k in sorted(set(f) | set(w)):
        out["kernels"][k] = {"fetch_bytes": f.get(k, 0.0) * 1024.0 * sf, "write_bytes": w.get(k, 0.0) * 1024.0 * sw}
    print(json.dumps(out, indent=1))


def traffic_table(path):
    """The figures of a traffic JSON (see `traffic`) as a table, MiB per launch, largest first."""
    import json
    t = json.load(open(path))
    print("%-110s %10s %12s" % ("kernel", "read MiB", "written MiB"))
    ks = t["kernels"]
    for k in sorted(ks, key=lambda k: -(ks[k]["fetch_bytes"] + ks[k]["write_bytes"])):
        print("%-110s %10.1f %12.1f" % (k[:110], ks[k]["fetch_bytes"] / 2 ** 20, ks[k]["write_bytes"] / 2 ** 20))


def mfma(path, simds=128):
    busy = _avg(path, "SQ_VALU_MFMA_BUSY_CYCLES")
    act = _avg(path, "GRBM_GUI_ACTIVE")
    print("%-110s %14s %12s %8s" % ("kernel", "mfma_busy/disp", "active_clk", "util_%"))
    for k in sorted(busy, key=lambda k: -busy[k]):
        if busy[k] <= 0 or act.get(k, 0) <= 0:
            continue
        print("%-110s %14.0f %12.0f %8.1f" % (k[:110], busy[k], act[k], 100.0 * busy[k] / (act[k] * simds)))


if __name__ == "__main__":
    if sys.argv[1] == "mfma":
        mfma(sys.argv[2])
    elif sys.argv[1] == "stats":
        stats(sys.argv[2])
    elif sys.argv[1] == "traffic":
        traffic(*sys.argv[2:6])
    elif sys.argv[1] == "traffic_table":
        traffic_table(sys.argv[2])
    else:
        pmc(sys.argv[2], sys.argv[3])
