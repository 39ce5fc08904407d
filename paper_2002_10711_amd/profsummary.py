"""Turns rocprofv3 result databases into the short summaries kept under ``profiles/``.

    python -m paper_2002_10711_amd.profsummary trace  RESULTS.db
        per-kernel table of a ``--kernel-trace --stats`` run (calls, total, average us)
    python -m paper_2002_10711_amd.profsummary pmc    RESULTS.db [RESULTS.db ...]
        per-kernel averages of every counter of ``--pmc`` runs
    python -m paper_2002_10711_amd.profsummary dispatches RESULTS.db [--match NAME]
        the counters of a ``--pmc`` run dispatch by dispatch, in dispatch order
    python -m paper_2002_10711_amd.profsummary traffic --workload NAME --fetch FETCH.db
            --write WRITE.db [--out profiles/hbm_traffic.json]
        HBM bytes per launch of the workload's kernels from a FETCH_SIZE and a WRITE_SIZE run
        (KiB per dispatch), each scaled by what the same counter reads for the plain 256 MiB
        device copy that ``bench.py --copy-probe`` adds to the run; merged into the JSON file
        that bench.py quotes, stamped with a fingerprint of the kernel sources.

The databases are what ``rocprofv3 -d DIR -o run`` leaves as ``DIR/run_results.db``.
"""
import argparse
import collections
import json
import os
import sqlite3
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

# kernel name (prefix) -> the benchmark's name for the stage it implements
STAGE_OF = [
    ("weight_transform", "weight_transform"),
    ("fused_fwd", "fused_forward"),
    ("gemm_out", "gemm_output"),
    ("input_transform", "input_transform"),
    ("output_transform", "output_transform"),
]
COPY_KERNEL = "__amd_rocclr_copyBuffer"
COPY_KIB = 256 * 1024


def short(name):
    return name.replace("wino::(anonymous namespace)::", "").replace("void ", "").split("(")[0]


def trace_table(db_path):
    cur = sqlite3.connect(db_path).cursor()
    rows = ["| kernel | calls | total us | avg us | % |", "|---|---|---|---|---|"]
    for name, calls, tot, avg, pct in cur.execute("select * from top_kernels"):
        rows.append("| %s | %d | %.1f | %.3f | %.1f |" % (short(name), calls, tot, avg, pct))
    return "\n".join(rows)


def pmc_averages(db_path):
    """{(kernel, counter): (average per dispatch, dispatches)}"""
    cur = sqlite3.connect(db_path).cursor()
    cols = [d[0] for d in cur.execute("select * from counters_collection limit 1").description]
    ki, ci, vi = cols.index("kernel_name"), cols.index("counter_name"), cols.index("value")
    di = cols.index("dispatch_id") if "dispatch_id" in cols else None
    # a counter is reported once per hardware instance (XCD, shader engine ...): sum those
    # of one dispatch, then average over dispatches
    per = collections.defaultdict(float)
    for row in cur.execute("select * from counters_collection"):
        per[(short(row[ki]), row[ci], row[di] if di is not None else 0)] += row[vi]
    agg = collections.defaultdict(lambda: [0.0, 0])
    for (k, c, _), v in per.items():
        a = agg[(k, c)]
        a[0] += v
        a[1] += 1
    return {kc: (v / n, n) for kc, (v, n) in agg.items()}


def dispatch_table(db_path, match):
    """One row per dispatch, in dispatch order, of the kernels whose name contains `match`:
    every collected counter summed over its hardware instances."""
    cur = sqlite3.connect(db_path).cursor()
    cols = [d[0] for d in cur.execute("select * from counters_collection limit 1").description]
    ki, ci, vi, di = (cols.index(c) for c in ("kernel_name", "counter_name", "value", "dispatch_id"))
    per = collections.OrderedDict()
    for row in cur.execute("select * from counters_collection order by dispatch_id"):
        if match in row[ki]:
            key = (row[di], short(row[ki]), row[ci])
            per[key] = per.get(key, 0.0) + row[vi]
    lines = ["| dispatch | kernel | counter | value |", "|---|---|---|---|"]
    lines += ["| %d | %s | %s | %.1f |" % (d, k, c, v) for (d, k, c), v in per.items()]
    return "\n".join(lines)


def pmc_table(db_paths):
    rows = ["| kernel | counter | average per dispatch | dispatches |", "|---|---|---|---|"]
    for p in db_paths:
        for (k, c), (v, n) in sorted(pmc_averages(p).items()):
            rows.append("| %s | %s | %.1f | %d |" % (k, c, v, n))
    return "\n".join(rows)


def csrc_fingerprint():
    import hashlib
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2002_10711_amd", "csrc")
    for f in sorted(os.listdir(d)):
        if f.endswith((".hip", ".h", ".cpp")):
            h.update(f.encode())
            h.update(open(os.path.join(d, f), "rb").read())
    return h.hexdigest()[:16]


def traffic(workload, fetch_db, write_db, out_path, staged_gemm="gemm_tiled_kernel"):
    f, w = pmc_averages(fetch_db), pmc_averages(write_db)

    def one(table, counter):
        return {k: v for (k, c), (v, _) in table.items() if c == counter}
    fetch, write = one(f, "FETCH_SIZE"), one(w, "WRITE_SIZE")
    copy_f = [v for k, v in fetch.items() if k.startswith(COPY_KERNEL)]
    copy_w = [v for k, v in write.items() if k.startswith(COPY_KERNEL)]
    if not copy_f or not copy_w:
        raise SystemExit("no %s dispatches in the runs: was bench.py given --copy-probe?" % COPY_KERNEL)
    sf, sw = COPY_KIB / copy_f[0], COPY_KIB / copy_w[0]
    rows = ["| kernel | FETCH_SIZE avg (KiB) | WRITE_SIZE avg (KiB) | HBM bytes per launch |",
            "|---|---|---|---|"]
    result = {}
    for k in sorted(set(fetch) | set(write)):
        fb, wb_ = fetch.get(k, 0.0), write.get(k, 0.0)
        total = int(round((fb * sf + wb_ * sw) * 1024))
        rows.append("| `%s` | %.1f | %.1f | %d |" % (k, fb, wb_, total))
        stage = None
        if k.startswith(staged_gemm) and "true, true" in k:
            stage = "gemm"                      # the Winograd-domain GEMM (blocked U)
        for prefix, st in STAGE_OF:
            if k.startswith(prefix):
                stage = st
        if stage and stage not in result:
            result[stage] = total
    data = {}
    if os.path.exists(out_path):
        data = json.load(open(out_path))
    fp = csrc_fingerprint()
    if data.get("_meta", {}).get("csrc_sha256_16") != fp:
        # figures measured on other sources are dropped: bench.py would not quote them
        data = {}
    data["_meta"] = {
        "csrc_sha256_16": fp,
        "comment": "HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (KiB per "
                   "dispatch), each scaled by what the same counter reads for a plain 256 MiB "
                   "device copy in the same run; written by paper_2002_10711_amd.profsummary",
    }
    data[workload] = result
    json.dump(data, open(out_path, "w"), indent=1)
    return "\n".join(rows) + "\n\nScale factors from the copy: reads x %.3f, writes x %.3f.\n" % (sf, sw)


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawTextHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    t = sub.add_parser("trace")
    t.add_argument("db")
    p = sub.add_parser("pmc")
    p.add_argument("db", nargs="+")
    dd = sub.add_parser("dispatches")
    dd.add_argument("db")
    dd.add_argument("--match", default="")
    h = sub.add_parser("traffic")
    h.add_argument("--workload", required=True)
    h.add_argument("--fetch", required=True)
    h.add_argument("--write", required=True)
    h.add_argument("--out", default=os.path.join(ROOT, "profiles", "hbm_traffic.json"))
    a = ap.parse_args()
    if a.cmd == "trace":
        print(trace_table(a.db))
    elif a.cmd == "pmc":
        print(pmc_table(a.db))
    elif a.cmd == "dispatches":
        print(dispatch_table(a.db, a.match))
    else:
        print(traffic(a.workload, a.fetch, a.write, a.out))


if __name__ == "__main__":
    sys.exit(main())
