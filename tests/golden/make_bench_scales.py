"""Writes tests/golden/bench_scales.json: the static quantizer scales of every int8
benchmark workload, calibrated through the CPU oracle only (max-abs / 127 per stage,
standing in for the paper's warmed-up moving averages, Table 1 caption).

    python tests/golden/make_bench_scales.py [workload names: only these are (re)computed]

The benchmark reads this file so that its GPU leg never touches the oracle.  Nothing
here calls the HIP library."""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_2002_10711_amd import workloads  # noqa: E402


def main():
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "bench_scales.json")
    out = {}
    layers = (workloads.config2("i8") + workloads.config2("i16") + workloads.config2("i8w16") +
              workloads.config3() + workloads.config4() + workloads.config5())
    if len(sys.argv) > 1:
        out = json.load(open(path))
        layers = [L for L in layers if L.name in sys.argv[1:]]
    for L in layers:
        X, g = workloads.make_inputs(L)
        if L.stride == 1:
            BT, G, AT = oracle.cook_toom(L.m, dtype=np.float32)
            if L.flex_sigma > 0:
                BT, G, AT = workloads.perturb_transforms(BT, G, AT, L.flex_sigma, L.seed)
            sc = oracle.calibrate(X, g, BT, G, AT, pad=L.pad, qmax=workloads.STAGE_QMAX[L.dtype])
        else:
            # im2row baseline layer: input, weight and output scales
            s_x = np.float32(np.abs(X).max() / 127)
            s_w = np.float32(np.abs(g).max() / 127)
            acc, _ = oracle.conv2d_direct_q(oracle.quantize_tensor(X, s_x),
                                            oracle.quantize_tensor(g, s_w), 1.0,
                                            stride=L.stride, pad=L.pad)
            s_y = np.float32(np.float32(s_x * s_w) * np.float32(np.abs(acc).max()) / 127)
            sc = dict(s_x=float(s_x), s_w=float(s_w), s_y=float(s_y))
        # every layer also gets baseline scales, for the speedup ratio
        if "s_w" not in sc:
            sc["s_w"] = float(np.float32(np.abs(g).max() / 127))
        out[L.name] = sc
        print(L.name, sc, flush=True)
    with open(path, "w") as f:
        json.dump(out, f, indent=1, sort_keys=True)


if __name__ == "__main__":
    main()
