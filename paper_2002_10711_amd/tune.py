"""Measures every kernel sequence of the int8 forward over a grid of layer shapes and writes
the table the library's dispatch reads (the paper picks the algorithm per layer from a table
of measured latencies, Sec. 5.3; this is the same idea for the kernel sequences behind one
algorithm).

    python -m paper_2002_10711_amd.tune --sweep [--out profiles/dispatch_sweep.json]
        on the MI355X: times wino_conv2d_fwd_seq for every sequence that can run each grid
        point (HIP-graph replays, events on the launch stream) and stores all times
    python -m paper_2002_10711_amd.tune --sweep --only trow [--m 6]
        the same for the named sequences only (and one tile size only): their times replace
        or join the ones the stored sweep holds for every grid point, the rest stays
    python -m paper_2002_10711_amd.tune --emit [--sweep-file profiles/dispatch_sweep.json]
        anywhere: writes paper_2002_10711_amd/csrc/dispatch_table.h from the stored times
        (rebuild the library afterwards)

Grid: m in {2, 4, 6}; C in {64, 128, 256, 512}; K in {64, 128, max(256, C)} (the three classes
of output channels the dispatch distinguishes); square images of 4, 8, 16, 32, 56 pixels;
batch 32, 64, 128 and 256.  Inputs are random codes: the kernels' run time does not depend on values.
"""
import argparse
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SWEEP_FILE = os.path.join(ROOT, "profiles", "dispatch_sweep.json")
TABLE_FILE = os.path.join(ROOT, "paper_2002_10711_amd", "csrc", "dispatch_table.h")
SEQ_IDS = {"fused": 1, "col": 2, "col2": 3, "lds": 4, "regs": 5, "staged": 6, "trow": 7}
MAX_WORKSPACE = 3 << 30


def grid():
    for m in (2, 4, 6):
        for C in (64, 128, 256, 512):
            for K in (64, 128, max(256, C)):
                for hw in (4, 8, 16, 32, 56):
                    for N in (32, 64, 128, 256):
                        yield dict(m=m, C=C, K=K, H=hw, N=N)


def kclass(Kp):
    return 0 if Kp <= 64 else 1 if Kp <= 128 else 2


def derived(pt):
    m, H = pt["m"], pt["H"]
    th = -(-H // m)                      # pad 1: Ho = H
    return dict(T=pt["N"] * th * th, Cp=-(-pt["C"] // 64) * 64, Kp=-(-pt["K"] // 64) * 64)


def sweep(out_path, budget_ms, only=None, only_m=None, base_path=None):
    import torch
    from paper_2002_10711_amd import binding as wb
    dev = torch.device("cuda:0")
    stream = torch.cuda.Stream()
    rng = np.random.default_rng(7)
    rows = []
    old = {}
    if only:
        # (a partial sweep: start from the stored rows and time the named sequences again)
        for r in json.load(open(base_path or out_path))["grid"]:
            old[(r["m"], r["C"], r["K"], r["H"], r["N"])] = r
    for pt in grid():
        m, C, K, H, N = pt["m"], pt["C"], pt["K"], pt["H"], pt["N"]
        key = (m, C, K, H, N)
        if only and (key not in old or (only_m and m != only_m)):
            if key in old:
                rows.append(old[key])
            continue
        BT, G, AT = wb.wino_cook_toom(m)
        desc = wb.Desc(N, C, K, H, H, 1, m, wb.WINO_I8, BT=BT, G=G, AT=AT)
        if only and not any(wb.wino_fwd_sequence(desc, SEQ_IDS[nm]) == SEQ_IDS[nm] for nm in only):
            r = dict(old[key])
            r["times_us"] = {k: v for k, v in r["times_us"].items() if k not in only}
            rows.append(r)
            continue
        ws_bytes = wb.wino_workspace_bytes(desc)
        if ws_bytes > MAX_WORKSPACE:
            continue
        quant = wb.make_quant(0.05, 0.3, 0.01, 0.2, 0.0, 127)
        x = torch.from_numpy(rng.integers(-127, 128, (N, C, H, H), dtype=np.int8)).to(dev)
        g = torch.from_numpy(rng.standard_normal((K, C, 3, 3)).astype(np.float32) * 0.05).to(dev)
        U = torch.empty(wb.wino_weights_bytes(desc), dtype=torch.uint8, device=dev)
        ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
        y = torch.empty((N, K, H, H), dtype=torch.int8, device=dev)
        with torch.cuda.stream(stream):
            wb.wino_transform_weights(desc, quant, g, U, stream=stream)
        stream.synchronize()
        times = dict(old[key]["times_us"]) if only else {}
        for name, sid in SEQ_IDS.items():
            if only and name not in only:
                continue
            if wb.wino_fwd_sequence(desc, sid) != sid:
                times.pop(name, None)
                continue

            def fn():
                wb.wino_conv2d_fwd_seq(desc, quant, x, U, y, ws, sid, stream=stream)
            with torch.cuda.stream(stream):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                for _ in range(2):
                    fn()
                e0.record(stream)
                fn()
                e1.record(stream)
                stream.synchronize()
                est = max(e0.elapsed_time(e1), 1e-3)          # ms, one host-launched call
                per = int(min(10, max(1, budget_ms / 4 / est)))
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph, stream=stream):
                    for _ in range(per):
                        fn()
                reps = int(max(2, budget_ms / (est * per)))
                best = None
                for _ in range(3):
                    graph.replay()
                    e0.record(stream)
                    for _ in range(reps):
                        graph.replay()
                    e1.record(stream)
                    stream.synchronize()
                    t = e0.elapsed_time(e1) / (reps * per) * 1e3
                    best = t if best is None else min(best, t)
                del graph
            times[name] = round(best, 3)
        row = dict(pt)
        row.update(derived(pt))
        row["times_us"] = times
        rows.append(row)
        print(json.dumps(row), flush=True)
        del x, g, U, ws, y
    from paper_2002_10711_amd.profsummary import csrc_fingerprint
    json.dump({"_meta": {"device": torch.cuda.get_device_name(0), "csrc_sha256_16": csrc_fingerprint(),
                         "method": "HIP-graph replays of wino_conv2d_fwd_seq, best of 3 runs, us per forward"},
               "grid": rows}, open(out_path, "w"), indent=0)


def table_text(data):
    lines = ["// Generated by `python -m paper_2002_10711_amd.tune --emit` from profiles/dispatch_sweep.json;",
             "// do not edit.  One row per measured grid point: tile size, padded input channels, class of",
             "// output channels, image height, tiles; then the sequences that ran there, fastest first.",
             "static const DispatchRow kDispatch[] = {"]
    for r in data["grid"]:
        order = sorted(r["times_us"], key=lambda k: r["times_us"][k])
        rank = ", ".join(str(SEQ_IDS[k]) for k in order)
        lines.append("    {%d, %d, %d, %d, %d, {%s}}," % (r["m"], r["Cp"], kclass(r["Kp"]), r["H"], r["T"], rank))
    lines.append("};")
    return "\n".join(lines) + "\n"


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawTextHelpFormatter)
    ap.add_argument("--sweep", action="store_true")
    ap.add_argument("--emit", action="store_true")
    ap.add_argument("--out", default=SWEEP_FILE)
    ap.add_argument("--sweep-file", default=SWEEP_FILE)
    ap.add_argument("--budget-ms", type=float, default=12.0, help="timed GPU work per sequence and run")
    ap.add_argument("--only", default="", help="comma-separated sequence names: time only these, keep the rest")
    ap.add_argument("--m", type=int, default=0, help="with --only: grid points of this tile size only")
    a = ap.parse_args()
    if a.sweep:
        sweep(a.out, a.budget_ms, [x for x in a.only.split(",") if x] or None, a.m or None, a.sweep_file)
    if a.emit:
        open(TABLE_FILE, "w").write(table_text(json.load(open(a.sweep_file))))
        print("wrote", TABLE_FILE)
    if not a.sweep and not a.emit:
        ap.error("nothing to do: --sweep and/or --emit")


if __name__ == "__main__":
    sys.exit(main())
