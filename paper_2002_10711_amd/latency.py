"""Per-shape latency table and algorithm choice on the GPU (paper, Sec. 5.3 "Impact of
Winograd on Latency", Fig. 6, and the latency look-up that wiNAS consumes, Sec. 4).

The paper times 3x3 convolutions with im2row and with F2 / F4 / F6 Winograd while varying
the output width/height (112x112 down to 2x2) and inCh -> outCh (3 -> 32 up to
512 -> 512), in FP32 and INT8, and reads off which algorithm to use where.  This module
does the same sweep through the C ABI on the MI355X: forward only, weights prepared
beforehand (the paper treats the weight transform as amortised), inputs resident in HBM,
each call replayed from a HIP graph.  It is a timing tool: values are seeded noise and the
int8 scales are loose bounds (no stage saturates badly, nothing is calibrated) -- parity
is the business of tests/, not of this file.

    python -m paper_2002_10711_amd.latency --out profiles/latency_table.md

`choose_algorithm(table, ...)` returns the fastest entry for a shape, the way a
latency-aware search would query the table.
"""
import argparse
import json

import numpy as np

ALGORITHMS = ("im2row", "F2", "F4", "F6")
SIZES = (112, 56, 32, 28, 16, 14, 8, 7, 4, 2)
CHANNELS = ((3, 32), (32, 32), (64, 64), (128, 128), (256, 256), (512, 512))


def shape_key(C, K, size, dtype):
    return "%s:%d->%d@%d" % (dtype, C, K, size)


def choose_algorithm(table, C, K, size, dtype):
    """Fastest algorithm for a shape that is in the table: (name, microseconds)."""
    row = table[shape_key(C, K, size, dtype)]
    name = min((a for a in ALGORITHMS if row.get(a) is not None), key=lambda a: row[a])
    return name, row[name]


def _timed(fn, stream, reps, warmup):
    """microseconds per call: 10 calls per HIP graph, replayed."""
    import torch
    per = 10
    with torch.cuda.stream(stream):
        for _ in range(2):
            fn()
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            for _ in range(per):
                fn()
        for _ in range(max(1, warmup // per)):
            graph.replay()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record(stream)
        n = max(1, reps // per)
        for _ in range(n):
            graph.replay()
        e1.record(stream)
        torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / (n * per)


def time_shape(N, C, K, size, dtype, reps=100, warmup=20, seed=0):
    """Latencies in microseconds of one NxCxsizexsize -> K convolution (pad 1), per algorithm."""
    import torch
    from . import binding as wb
    dev = torch.device("cuda:0")
    i8 = dtype == "int8"
    dt = wb.WINO_I8 if i8 else wb.WINO_F32
    rng = np.random.default_rng(seed)
    H = W = size
    if i8:
        xh = rng.integers(0, 128, size=(N, C, H, W), dtype=np.int8)
    else:
        xh = np.maximum(rng.standard_normal((N, C, H, W), dtype=np.float32), 0)
    g = (rng.standard_normal((K, C, 3, 3)) * np.sqrt(2.0 / (9 * C))).astype(np.float32)
    x = torch.from_numpy(xh).to(dev)
    gd = torch.from_numpy(g).to(dev)
    y = torch.empty((N, K, H, W), dtype=torch.int8 if i8 else torch.float32, device=dev)
    stream = torch.cuda.Stream()
    out = {}
    gmax = float(np.abs(g).max())
    # im2row baseline (weights packed once)
    s_x, s_w = 1.0 / 32, gmax / 127
    s_y = s_x * s_w * 127 * np.sqrt(9 * C)
    wq = np.clip(np.rint(g / np.float32(s_w)), -127, 127).astype(np.int8) if i8 else g
    wdev = torch.from_numpy(wq).to(dev)
    wp = torch.empty(wb.conv2d_ref_packed_weights_bytes(C, K, dt), dtype=torch.uint8, device=dev)
    rws = torch.empty(wb.conv2d_ref_workspace_bytes(N, C, K, H, W, 1, 1, dt), dtype=torch.uint8,
                      device=dev)
    with torch.cuda.stream(stream):
        wb.conv2d_ref_pack_weights(C, K, dt, wdev, wp, stream=stream)
    out["im2row"] = _timed(lambda: wb.conv2d_ref_gpu(N, C, K, H, W, 1, 1, dt, x, wp, y, s_x, s_w,
                                                     s_y, 127, rws, stream=stream),
                           stream, reps, warmup)
    del rws, wp
    for m in (2, 4, 6):
        BT, G, AT = wb.wino_cook_toom(m)
        desc = wb.Desc(N, C, K, H, W, 1, m, dt, BT=BT, G=G, AT=AT)
        quant = None
        if i8:
            # loose bounds from the matrices' absolute row sums: nothing overflows its stage
            nb = float(np.abs(BT).sum(axis=1).max()) ** 2
            ng = float(np.abs(G).sum(axis=1).max()) ** 2
            na = float(np.abs(AT).sum(axis=1).max()) ** 2
            s_v = s_x * nb
            s_u = gmax * ng / 127
            quant = wb.make_quant(s_x, s_v, s_u, s_u * s_v * 127 * np.sqrt(C) * na / 16)
        U = torch.empty(wb.wino_weights_bytes(desc), dtype=torch.uint8, device=dev)
        ws = torch.empty(wb.wino_workspace_bytes(desc), dtype=torch.uint8, device=dev)
        with torch.cuda.stream(stream):
            wb.wino_transform_weights(desc, quant, gd, U, stream=stream)
        out["F%d" % m] = _timed(lambda: wb.wino_conv2d_fwd(desc, quant, x, U, y, ws, stream=stream),
                                stream, reps, warmup)
        del U, ws
    return out


def sweep(N=32, sizes=SIZES, channels=CHANNELS, dtypes=("int8", "f32"), reps=100, warmup=20,
          max_bytes=2 << 30, log=None):
    """{shape key: {algorithm: microseconds, "best": name}} over the sweep; shapes whose
    largest intermediate (F2's int32 / fp32 Hadamard-stage tensor, 16 N size^2 K bytes, or
    the im2row matrix) would exceed max_bytes are skipped."""
    table = {}
    for dtype in dtypes:
        for C, K in channels:
            for size in sizes:
                e = 1 if dtype == "int8" else 4
                if max(N * size * size * 9 * max(C, 4) * e, 16 * N * size * size * max(C, K)) > max_bytes:
                    continue
                row = time_shape(N, C, K, size, dtype, reps, warmup)
                row["best"] = min(ALGORITHMS, key=lambda a: row[a])
                table[shape_key(C, K, size, dtype)] = row
                if log:
                    log("%-22s " % shape_key(C, K, size, dtype) +
                        " ".join("%s %8.1f" % (a, row[a]) for a in ALGORITHMS) + "  -> " + row["best"])
    return table


def to_markdown(table, N):
    lines = ["| dtype | inCh->outCh | size | im2row us | F2 us | F4 us | F6 us | best | speedup vs im2row |",
             "|---|---|---|---|---|---|---|---|---|"]
    for key, row in table.items():
        dtype, rest = key.split(":")
        ch, size = rest.split("@")
        lines.append("| %s | %s | %sx%s | %.1f | %.1f | %.1f | %.1f | %s | %.2f |" % (
            dtype, ch, size, size, row["im2row"], row["F2"], row["F4"], row["F6"], row["best"],
            row["im2row"] / row[row["best"]]))
    return "\n".join(lines)


def main():
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--batch", type=int, default=32)
    ap.add_argument("--reps", type=int, default=100)
    ap.add_argument("--out", default=None, help="write the markdown table (and .json beside it)")
    ap.add_argument("--quick", action="store_true", help="three sizes, two channel settings")
    a = ap.parse_args()
    sizes = (32, 8, 4) if a.quick else SIZES
    channels = ((3, 32), (64, 64)) if a.quick else CHANNELS
    table = sweep(a.batch, sizes, channels, reps=a.reps, log=lambda s: print(s, flush=True))
    md = ("# Latency of 3x3 convolutions per shape and algorithm (forward, batch %d, pad 1)\n\n"
          "Command: `python -m paper_2002_10711_amd.latency --batch %d --reps %d --out <this file>` "
          "on one MI355X.\nMicroseconds per call, weights prepared beforehand, HIP-graph replay; "
          "`best` is what `choose_algorithm` returns.\n\n" % (a.batch, a.batch, a.reps)) + \
        to_markdown(table, a.batch) + "\n"
    if a.out:
        with open(a.out, "w") as f:
            f.write(md)
        with open(a.out.rsplit(".", 1)[0] + ".json", "w") as f:
            json.dump({"batch": a.batch, "table": table}, f, indent=1)
    else:
        print(md)


if __name__ == "__main__":
    main()
