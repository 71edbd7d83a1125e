"""Short summaries of rocprofv3 CSV output for the files under profiles/.

    python -m paper_2603_12617_amd.rocprof_summary trace  <X_kernel_stats.csv>
        per kernel: calls, average and total duration (the table of `--kernel-trace --stats`)
    python -m paper_2603_12617_amd.rocprof_summary pmc    <X_counter_collection.csv>
        per kernel and counter: dispatches and the mean counter value per dispatch
    python -m paper_2603_12617_amd.rocprof_summary traffic --name c4 --kernel dense_window_kernel \
            --fetch F.csv --write W.csv --copy-fetch CF.csv --copy-write CW.csv \
            --json profiles/hbm_traffic.json --commit <hash> --plan "<launch plan>"
        HBM bytes per launch of one kernel: FETCH_SIZE and WRITE_SIZE (KiB per dispatch) scaled by
        what the same counters read for a plain device copy of known size (`bench.py --copy-probe`,
        1 GiB read and written), stored with the commit and launch plan they were measured at.

Nothing here runs a GPU; it only reads what rocprofv3 wrote.
"""
import argparse
import csv
import json
import os
import re
import sys
from collections import OrderedDict

COPY_KIB = float(1 << 20)         # bench.py --copy-probe copies 1 GiB


def short(name):
    """Kernel name without return type, namespaces and argument list."""
    n = re.sub(r"\(anonymous namespace\)::", "", name)
    n = re.sub(r"^void ", "", n)
    n = n.split("(")[0]
    return n.replace("oco::", "")


def trace(path):
    rows = list(csv.DictReader(open(path)))
    out = ["| kernel | calls | average ms | total ms | % |", "|---|---|---|---|---|"]
    for r in rows:
        out.append("| `%s` | %s | %.4f | %.3f | %s |" % (short(r["Name"]), r["Calls"], float(r["AverageNs"]) / 1e6,
                                                        float(r["TotalDurationNs"]) / 1e6, r["Percentage"]))
    return "\n".join(out)


def pmc_means(path):
    """{(kernel, counter): (dispatches, mean value)} in order of first appearance."""
    acc = OrderedDict()
    for r in csv.DictReader(open(path)):
        k = (short(r["Kernel_Name"]), r["Counter_Name"])
        s = acc.setdefault(k, [0, 0.0])
        s[0] += 1
        s[1] += float(r["Counter_Value"])
    return OrderedDict((k, (n, t / n)) for k, (n, t) in acc.items())


def pmc(path):
    out = ["| kernel | counter | dispatches | mean per dispatch |", "|---|---|---|---|"]
    for (k, c), (n, m) in pmc_means(path).items():
        out.append("| `%s` | %s | %d | %.1f |" % (k, c, n, m))
    return "\n".join(out)


def _one(path, counter, kernel):
    hits = [(k, v) for (k, c), v in pmc_means(path).items() if c == counter and kernel in k]
    if not hits:
        raise SystemExit("no dispatch of a kernel matching %r with %s in %s" % (kernel, counter, path))
    n = sum(v[0] for _, v in hits)
    return n, sum(v[0] * v[1] for _, v in hits) / n


def traffic(a):
    _, cf = _one(a.copy_fetch, "FETCH_SIZE", "copyBuffer")
    _, cw = _one(a.copy_write, "WRITE_SIZE", "copyBuffer")
    kf, kw = COPY_KIB / cf, COPY_KIB / cw
    nf, f = _one(a.fetch, "FETCH_SIZE", a.kernel)
    nw, w = _one(a.write, "WRITE_SIZE", a.kernel)
    entry = {"kernel": a.kernel, "read_bytes_per_launch": f * kf * 1024.0, "written_bytes_per_launch": w * kw * 1024.0,
             "bytes_per_launch": (f * kf + w * kw) * 1024.0, "dispatches_seen": [nf, nw],
             "calibration": {"FETCH_SIZE_factor": kf, "WRITE_SIZE_factor": kw,
                             "how": "1 GiB device copy (bench.py --copy-probe) read by the same counters"},
             "commit": a.commit, "plan": a.plan}
    data = json.load(open(a.json)) if os.path.exists(a.json) else {}
    data[a.name] = entry
    json.dump(data, open(a.json, "w"), indent=1)
    return json.dumps({a.name: entry}, indent=1)


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    for name in ("trace", "pmc"):
        p = sub.add_parser(name)
        p.add_argument("csv")
    p = sub.add_parser("traffic")
    for k in ("name", "kernel", "fetch", "write", "copy-fetch", "copy-write", "json", "commit", "plan"):
        p.add_argument("--" + k, required=True)
    a = ap.parse_args(argv)
    print({"trace": lambda: trace(a.csv), "pmc": lambda: pmc(a.csv), "traffic": lambda: traffic(a)}[a.cmd]())
    return 0


if __name__ == "__main__":
    sys.exit(main())
