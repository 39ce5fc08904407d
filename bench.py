#!/usr/bin/env python3
"""Benchmark of the Winograd-aware convolution forward path on one MI355X.

A step is one pass of the whole hot path over one batch: weight transform
G g G^T, input transform B^T d B, the per-position GEMMs and the output transform
A^T M A, int8 with a quantizer after every stage.  The default workload is the
CIFAR ResNet-18 stage-1 convolution (batch 64, 32x32, 64->64 channels,
F(4x4,3x3)); inputs are synthetic (seeded ReLU(N(0,1)) activations, Kaiming
weights) and resident in HBM before the timed region starts.

Prints ONE JSON line: direct-convolution-equivalent TOPS of the whole step, the
roofline of the dominant kernel (per-kernel durations measured with events on the
launch stream), the speedup over the im2row baseline, and the CPU oracle timed on
the host cores as a reported baseline.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2002_10711_amd import workloads  # noqa: E402

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_PEAK = {"int8": 5000.0, "f32": 157.3, "f16": 2500.0}   # dense TOP/s, TFLOP/s
WIDE = ("i16", "i8w16")    # dtypes with 16-bit codes in the Winograd domain
HBM_TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")


def pick_workload(name):
    table = {}
    for L in (workloads.config2("i8") + workloads.config2("f32") + workloads.config2("i16") +
              workloads.config2("i8w16") + workloads.config3() +
              workloads.config4() + workloads.config5()):
        table[L.name] = L
    if name not in table:
        raise SystemExit("unknown workload %r; choose from %s" % (name, sorted(table)))
    return table[name]


ALU_PEAK_TFLOPS = 78.6         # fp32 vector without packed ops: 256 CU x 64 lanes x 2 x 2.4 GHz


def algorithmic(L, BT, AT):
    """Bytes / operations the method itself must move / do, per kernel launch.
    `ops` are the GEMM's multiply-adds (x2); `alu` are the transforms' fp32 operations:
    one fused multiply-add (2 flops) per nonzero matrix entry and vector element, one
    int->float conversion per accumulator, four operations per quantized element
    (scale, round, saturate, convert)."""
    wide = L.dtype in WIDE
    e = 1 if L.dtype in ("i8", "i8w16") else 2 if L.dtype == "i16" else 4   # X, Y element
    ew = 2 if wide else e                                                   # U, V element
    quantized = L.dtype != "f32"
    qops = 4 if quantized else 0
    n = L.m + 2
    P = n * n
    TH, TW = -(-L.Ho // L.m), -(-L.Wo // L.m)
    T = L.N * TH * TW
    nzb, nza = int(np.count_nonzero(BT)), int(np.count_nonzero(AT))
    x_b, y_b = L.N * L.C * L.H * L.W * e, L.N * L.K * L.Ho * L.Wo * e
    v_b, u_b, m_b = P * T * L.C * ew, P * L.C * L.K * ew, (8 if wide else 4) * P * T * L.K
    # wide modes: a 16-bit product is four int8 digit products on the matrix cores
    mm = 2 * P * T * L.C * L.K * (4 if wide else 1)
    alu_in = T * L.C * (2 * 2 * n * nzb + qops * P)
    alu_out = T * L.K * (2 * (n + L.m) * nza + (P if quantized else 0) + qops * L.m * L.m)
    alu_w = L.K * L.C * (2 * (3 * 3 * n + 3 * n * n) + qops * P)
    return {
        "weight_transform": dict(bytes=9 * L.C * L.K * 4 + u_b, ops=0, alu=alu_w),
        "input_transform": dict(bytes=x_b + v_b, ops=0, alu=alu_in),
        "gemm": dict(bytes=v_b + u_b + m_b, ops=mm, alu=0),
        "output_transform": dict(bytes=m_b + y_b, ops=0, alu=alu_out),
        # GEMM and output transform in one kernel: M is never stored
        "gemm_output": dict(bytes=v_b + u_b + y_b, ops=mm, alu=alu_out),
        # the whole forward in one kernel: neither V nor M is stored
        "fused_forward": dict(bytes=x_b + u_b + y_b, ops=mm, alu=alu_in + alu_out),
    }


def roofline_entry(name, alg, us, dtype, traffic):
    """The bound is whichever of HBM, MFMA and vector-ALU peak needs the longest time
    for the kernel's algorithmic bytes / GEMM operations / transform operations."""
    mf = MFMA_PEAK["int8" if dtype == "i8" or dtype in WIDE else "f32"]
    t = {"hbm": alg["bytes"] / (HBM_PEAK_GBS * 1e9), "mfma": alg["ops"] / (mf * 1e12),
         "alu": alg["alu"] / (ALU_PEAK_TFLOPS * 1e12)}
    bound = max(t, key=t.get)
    sec = us * 1e-6
    if bound == "hbm":
        ent = dict(bound="hbm", achieved=alg["bytes"] / sec / 1e9, peak=HBM_PEAK_GBS, unit="GB/s")
    elif bound == "mfma":
        ent = dict(bound="mfma", achieved=alg["ops"] / sec / 1e12, peak=mf,
                   unit="TOP/s" if dtype == "i8" else "TFLOP/s")
    else:
        # (frac_of_packed_peak: against the 157.3 TFLOP/s the chip reaches with packed fp32
        # instructions, which this build may not use)
        ent = dict(bound="alu", achieved=alg["alu"] / sec / 1e12, peak=ALU_PEAK_TFLOPS, unit="TFLOP/s",
                   frac_of_packed_peak=alg["alu"] / sec / 1e12 / (2 * ALU_PEAK_TFLOPS))
    ent.update(kernel=name, frac=ent["achieved"] / ent["peak"], avg_us=us,
               algorithmic_bytes=alg["bytes"], algorithmic_ops=alg["ops"],
               algorithmic_alu_ops=alg["alu"], hbm_frac=alg["bytes"] / sec / 1e9 / HBM_PEAK_GBS,
               mfma_frac=alg["ops"] / sec / 1e12 / mf, traffic=traffic)
    return ent


def gpu_leg(L, steps, warmup, use_graph, cold=False):
    import torch
    from paper_2002_10711_amd import binding as wb
    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU (no CPU fallback exists)")
    wb.lib()
    dev = torch.device("cuda:0")
    i8 = L.dtype == "i8"
    wide = L.dtype in WIDE
    qm = workloads.STAGE_QMAX.get(L.dtype)
    scales = json.load(open(os.path.join(ROOT, "tests", "golden", "bench_scales.json")))[
        L.name.replace("_f32", "_i8")]
    X, g = workloads.make_inputs(L)
    BT, G, AT = wb.wino_cook_toom(L.m)
    if L.flex_sigma > 0:
        BT, G, AT = workloads.perturb_transforms(BT, G, AT, L.flex_sigma, L.seed)
    dt = {"i8": wb.WINO_I8, "f32": wb.WINO_F32, "i16": wb.WINO_I16, "i8w16": wb.WINO_I8W16}[L.dtype]
    desc = wb.Desc(L.N, L.C, L.K, L.H, L.W, L.pad, L.m, dt, BT=BT, G=G, AT=AT)
    quant = None
    ydt = torch.float32
    if i8 or wide:
        quant = wb.make_quant(scales["s_x"], scales["s_v"], scales["s_u"], scales["s_y"], 0.0, qm["y"],
                              qmax_u=qm["u"], qmax_v=qm["v"], qmax_m=qm["m"], qmax_y=qm["y"])
        # input codes of the previous layer's quantizer (input preparation, not the path)
        xh = np.clip(np.rint(X / np.float32(scales["s_x"])), -qm["x"], qm["x"]).astype(
            np.int16 if L.dtype == "i16" else np.int8)
        ydt = torch.int16 if L.dtype == "i16" else torch.int8
    else:
        xh = X
    x = torch.from_numpy(xh).to(dev)
    gd = torch.from_numpy(g).to(dev)
    U = torch.empty(wb.wino_weights_bytes(desc), dtype=torch.uint8, device=dev)
    ws = torch.empty(wb.wino_workspace_bytes(desc), dtype=torch.uint8, device=dev)
    y = torch.empty((L.N, L.K, L.Ho, L.Wo), dtype=ydt, device=dev)
    stream = torch.cuda.Stream()          # default priority

    def step():
        wb.wino_transform_weights(desc, quant, gd, U, stream=stream)
        wb.wino_conv2d_fwd(desc, quant, x, U, y, ws, stream=stream)

    def fwd_only():
        wb.wino_conv2d_fwd(desc, quant, x, U, y, ws, stream=stream)

    def timed(fn, k, w):
        """ms per call of fn over exactly k timed calls (w untimed ones first)."""
        with torch.cuda.stream(stream):
            if use_graph:
                # one HIP graph holds `per` consecutive calls; k / per replays are timed
                per = max(d for d in range(1, 11) if k % d == 0)
                for _ in range(3):
                    fn()
                stream.synchronize()
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph, stream=stream):
                    for _ in range(per):
                        fn()
                runner, reps, wreps = graph.replay, k // per, -(-w // per)
            else:
                runner, reps, wreps = fn, k, w
            for _ in range(wreps):
                runner()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record(stream)
            for _ in range(reps):
                runner()
            e1.record(stream)
            torch.cuda.synchronize()
        return e0.elapsed_time(e1) / k       # ms per call

    ms_step = timed(step, steps, warmup)
    ms_fwd = timed(fwd_only, steps, warmup)

    # per-kernel durations: the same step, with events between the kernels
    nk = wb.wino_fwd_num_kernels(desc)
    if nk == 1:
        stages = [("weight_transform", None), ("fused_forward", wb.WINO_STAGE_ALL)]
    elif nk == 3:
        stages = [("weight_transform", None), ("input_transform", wb.WINO_STAGE_INPUT),
                  ("gemm", wb.WINO_STAGE_GEMM), ("output_transform", wb.WINO_STAGE_OUTPUT)]
    else:
        stages = [("weight_transform", None), ("input_transform", wb.WINO_STAGE_INPUT),
                  ("gemm_output", wb.WINO_STAGE_GEMM | wb.WINO_STAGE_OUTPUT)]
    ksteps = max(20, min(steps, 2000))
    kwarm = max(10, min(warmup, 500))
    # (the forward once, so that every stage finds its predecessor's output)
    wb.wino_transform_weights(desc, quant, gd, U, stream=stream)
    for _, mask in stages[1:]:
        wb.wino_conv2d_fwd_stages(desc, quant, x, U, y, ws, mask, stream=stream)
    stream.synchronize()

    def time_stages(stages):
        """us per launch of every stage: each stage on its own, 10 back-to-back calls per HIP
        graph (host launches with --no-graph), events around the replays on the stream the
        kernels run on.  A stage reads what the previous one left in the workspace, so
        repeating it changes nothing."""
        acc = {}
        for name, mask in stages:
            if mask is None:
                fn = lambda: wb.wino_transform_weights(desc, quant, gd, U, stream=stream)
            else:
                fn = lambda mask=mask: wb.wino_conv2d_fwd_stages(desc, quant, x, U, y, ws, mask,
                                                                 stream=stream)
            acc[name] = timed(fn, ksteps - ksteps % 10, kwarm) * 1e3
        return acc

    acc = time_stages(stages)
    # the four kernels of the unfused path, one call each (the paper's kernels a-d as
    # separate launches, V and M through memory), whatever the forward call itself uses
    acc_staged = acc if nk == 3 else time_stages(
        [("weight_transform", None), ("input_transform", wb.WINO_STAGE_INPUT),
         ("gemm", wb.WINO_STAGE_GEMM), ("output_transform", wb.WINO_STAGE_OUTPUT)])

    # im2row baseline on the same layer, forward only (weights packed once)
    # (the baseline has int8 and fp32 forms: 8-bit activations are compared with the int8
    # one, the int16 workload has no baseline)
    s_w = scales.get("s_w", 1.0)
    rdt = wb.WINO_F32 if L.dtype == "f32" else wb.WINO_I8
    ms_ref = None
    if L.dtype != "i16":
        if rdt == wb.WINO_I8:
            wq = np.clip(np.rint(g / np.float32(s_w)), -127, 127).astype(np.int8)
        else:
            wq = g
        wdev = torch.from_numpy(wq).to(dev)
        wp = torch.empty(wb.conv2d_ref_packed_weights_bytes(L.C, L.K, rdt), dtype=torch.uint8, device=dev)
        rws = torch.empty(wb.conv2d_ref_workspace_bytes(L.N, L.C, L.K, L.H, L.W, 1, L.pad, rdt),
                          dtype=torch.uint8, device=dev)
        with torch.cuda.stream(stream):
            wb.conv2d_ref_pack_weights(L.C, L.K, rdt, wdev, wp, stream=stream)

        def ref_fwd():
            wb.conv2d_ref_gpu(L.N, L.C, L.K, L.H, L.W, 1, L.pad, rdt, x, wp, y, scales["s_x"], s_w,
                              scales["s_y"], 127, rws, stream=stream)

        ms_ref = timed(ref_fwd, max(10, steps // 4), max(2, warmup // 4))
    extra = {}
    if cold:
        # cold: every call finds neither X, U nor anything else in L2 / Infinity Cache
        # (256 MB): a 1 GiB fill runs between the calls, outside the event pairs
        big = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        n = 30
        with torch.cuda.stream(stream):
            def event_timed(flush):
                ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
                      for _ in range(n)]
                for a, b in ev:
                    if flush:
                        big.fill_(1)
                    a.record(stream)
                    fwd_only()
                    b.record(stream)
                torch.cuda.synchronize()
                ts = sorted(a.elapsed_time(b) for a, b in ev)
                return ts[len(ts) // 2]
            event_timed(True)
            extra["cold_fwd_ms"] = event_timed(True)
            extra["warm_fwd_host_launch_ms"] = event_timed(False)
            # plain device copy of 1 GiB (reads + writes counted): the HBM rate a kernel sees
            dst = torch.empty_like(big)
            for _ in range(2):
                dst.copy_(big)
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(stream)
            for _ in range(5):
                dst.copy_(big)
            b.record(stream)
            torch.cuda.synchronize()
            extra["measured_copy_GBps"] = 5 * 2 * (1 << 30) / (a.elapsed_time(b) * 1e-3) / 1e9
            # matrix-core probe: independent MFMAs only, 8 workgroups per compute unit
            probe = torch.empty(2048 * 256, dtype=torch.float32, device=dev)
            for name, pdt in (("measured_mfma_int8_TOPS", wb.WINO_I8), ("measured_mfma_f32_TFLOPS", wb.WINO_F32)):
                wb.wino_debug_mfma_loop(pdt, 2048, 2000, probe, stream=stream)
                a.record(stream)
                ops = wb.wino_debug_mfma_loop(pdt, 2048, 2000, probe, stream=stream)
                b.record(stream)
                torch.cuda.synchronize()
                extra[name] = ops / (a.elapsed_time(b) * 1e-3) / 1e12
        del big, dst
    return dict(extra=extra, ms_step=ms_step, ms_fwd=ms_fwd, ms_ref=ms_ref, kernel_us=acc, staged_us=acc_staged,
                BT=BT, AT=AT)


def ref_only_leg(L, steps, warmup):
    """ms per forward of the im2row baseline on a layer (stride 1 or 2), weights packed once."""
    import torch
    from paper_2002_10711_amd import binding as wb
    dev = torch.device("cuda:0")
    sc = json.load(open(os.path.join(ROOT, "tests", "golden", "bench_scales.json")))[L.name]
    X, g = workloads.make_inputs(L)
    xh = np.clip(np.rint(X / np.float32(sc["s_x"])), -127, 127).astype(np.int8)
    wq = np.clip(np.rint(g / np.float32(sc["s_w"])), -127, 127).astype(np.int8)
    x, wdev = torch.from_numpy(xh).to(dev), torch.from_numpy(wq).to(dev)
    y = torch.empty((L.N, L.K, L.Ho, L.Wo), dtype=torch.int8, device=dev)
    wp = torch.empty(wb.conv2d_ref_packed_weights_bytes(L.C, L.K, wb.WINO_I8), dtype=torch.uint8, device=dev)
    rws = torch.empty(wb.conv2d_ref_workspace_bytes(L.N, L.C, L.K, L.H, L.W, L.stride, L.pad, wb.WINO_I8),
                      dtype=torch.uint8, device=dev)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        wb.conv2d_ref_pack_weights(L.C, L.K, wb.WINO_I8, wdev, wp, stream=stream)

        def fn():
            wb.conv2d_ref_gpu(L.N, L.C, L.K, L.H, L.W, L.stride, L.pad, wb.WINO_I8, x, wp, y,
                              sc["s_x"], sc["s_w"], sc["s_y"], 127, rws, stream=stream)
        for _ in range(3):
            fn()
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            for _ in range(5):
                fn()
        for _ in range(max(1, warmup // 5)):
            graph.replay()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record(stream)
        n = max(1, steps // 5)
        for _ in range(n):
            graph.replay()
        e1.record(stream)
        torch.cuda.synchronize()
    return e0.elapsed_time(e1) / (n * 5)


def stack_line(steps, warmup):
    """The 16 3x3 convolutions of CIFAR ResNet-18 (batch 256, int8) one after the other:
    stride-1 layers on their Winograd tile, stride-2 layers on the im2row baseline; forward
    only, weights prepared beforehand (the paper's deployment setting, Sec. 5.3)."""
    layers = workloads.config5()
    rows, t_wino, t_ref, ops = [], 0.0, 0.0, 0
    for L in layers:
        if L.stride == 1:
            r = gpu_leg(L, steps, warmup, True)
            fwd, ref = r["ms_fwd"], r["ms_ref"]
        else:
            fwd = ref = ref_only_leg(L, steps, warmup)
        rows.append(dict(layer=L.name, fwd_us=fwd * 1e3, im2row_us=ref * 1e3))
        t_wino += fwd
        t_ref += ref
        ops += L.direct_ops
    return {
        "metric": "direct-conv-equiv TOPS, CIFAR ResNet-18 3x3 conv stack forward (13 Winograd + 3 im2row layers)",
        "value": ops / (t_wino * 1e-3) / 1e12, "unit": "TOPS", "n_gpus": 1, "steps": steps,
        "warmup": warmup, "ms_per_step": t_wino, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": "cfg5 stack: 16 layers, N=256, 64/128/256/512 channels at 32/16/8/4, "
                               "per-layer m from the seed", "launch": "hip-graph replay per layer"},
        "im2row_stack_ms": t_ref, "speedup_vs_im2row": t_ref / t_wino, "layers": rows,
    }


def cpu_leg(L):
    """The oracle as it stands, on the host cores, whole quantized forward
    (weight stage included) on the first images of the same workload."""
    import oracle
    oracle.build()
    n_img = min(L.N, 16)
    from dataclasses import replace
    Ls = replace(L, N=n_img)
    X, g = workloads.make_inputs(L)
    X = X[:n_img]
    BT, G, AT = oracle.cook_toom(L.m, dtype=np.float32)
    if L.flex_sigma > 0:
        BT, G, AT = workloads.perturb_transforms(BT, G, AT, L.flex_sigma, L.seed)
    if L.dtype != "f32":
        sc = json.load(open(os.path.join(ROOT, "tests", "golden", "bench_scales.json")))[L.name]
        qm = workloads.STAGE_QMAX[L.dtype]
        xq = oracle.quantize_tensor(X, sc["s_x"], qm["x"])
        fn = lambda: oracle.winograd_q(xq, g, BT, G, AT, sc, pad=L.pad, qmax=qm)
    else:
        fn = lambda: oracle.winograd_f64(X, g, BT, G, AT, L.pad)
    fn()
    t0 = time.perf_counter()
    reps = 0
    while time.perf_counter() - t0 < 10.0 or reps < 3:
        fn()
        reps += 1
    dt = (time.perf_counter() - t0) / reps
    return dict(value=Ls.direct_ops / dt / 1e12, unit="TOPS (direct-conv-equivalent)",
                cores=oracle.num_threads(), kind="oracle",
                sample="first %d of %d images of %s, %d repetitions, %.3f s each; quantized "
                       "pipeline incl. weight stage, OpenMP over tiles" % (n_img, L.N, L.name, reps, dt))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5000)
    ap.add_argument("--warmup", type=int, default=2000)
    ap.add_argument("--workload", default="cfg2_i8")
    ap.add_argument("--no-graph", action="store_true", help="launch every step from the host "
                    "instead of replaying a captured HIP graph of one step")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--stack", action="store_true", help="time the whole CIFAR ResNet-18 conv "
                    "stack (config 5: 16 layers, batch 256, int8) layer by layer, forward only, "
                    "and print its total instead of one workload's line")
    ap.add_argument("--flex", type=float, default=0.0, help="perturb the Cook-Toom matrices by "
                    "seeded N(0, FLEX) noise (dense 'learned' transforms, paper Sec. 3.2): a timing "
                    "option, the stored scales are not recalibrated")
    ap.add_argument("--cold", action="store_true", help="also time the forward with L2 and "
                    "Infinity Cache evicted before every call (a 1 GiB buffer is overwritten in "
                    "between) and measure the plain-copy HBM rate; adds cold_fwd_ms, "
                    "warm_fwd_host_launch_ms, measured_copy_GBps and the measured matrix-core "
                    "rates (MFMA-only loop) to the JSON line")
    ap.add_argument("--copy-probe", action="store_true", help="also run a plain 256 MiB device "
                    "copy a few times: the reference kernel against which rocprofv3's "
                    "FETCH_SIZE / WRITE_SIZE counters are scaled")
    a = ap.parse_args()
    if a.gpus != 1:
        raise SystemExit("bench.py: this build runs on ONE GPU only (the path needs no exchange "
                         "step: tiles are independent, so more GPUs would each take a share of the batch); "
                         "got --gpus %d" % a.gpus)
    if a.stack:
        print(json.dumps(stack_line(max(20, a.steps // 5), max(5, a.warmup // 5))))
        return
    L = pick_workload(a.workload)
    if a.flex > 0:
        from dataclasses import replace
        L = replace(L, flex_sigma=a.flex)
    if L.stride != 1:
        raise SystemExit("workload %s is an im2row (stride-2) layer, not a Winograd one" % L.name)
    if a.copy_probe:
        import torch
        src = torch.zeros(256 << 20, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    r = gpu_leg(L, a.steps, a.warmup, not a.no_graph, a.cold)
    alg = algorithmic(L, r["BT"], r["AT"])
    traffic = {}
    if os.path.exists(HBM_TRAFFIC_FILE):
        traffic = json.load(open(HBM_TRAFFIC_FILE)).get(L.name, {})
    kernels = [roofline_entry(k, alg[k], us, L.dtype, traffic.get(k)) for k, us in r["kernel_us"].items()]
    dominant = max(kernels, key=lambda e: e["avg_us"])
    out = {
        "metric": "direct-conv-equiv TOPS, int8 F(4x4,3x3) ResNet-18 layer (whole path incl. weight transform)"
                  if L.name == "cfg2_i8" else "direct-conv-equiv TOPS, whole Winograd path incl. weight transform",
        "value": L.direct_ops / (r["ms_step"] * 1e-3) / 1e12,
        "unit": "TOPS",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": r["ms_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {"i8": "int8", "f32": "f32", "i16": "int16", "i8w16": "int8 data, int16 Winograd domain"}[L.dtype],
        "data": "synthetic",
        "config": {"workload": "%s: N=%d C=%d K=%d %dx%d pad=%d F(%dx%d,3x3) %s" % (
            L.name, L.N, L.C, L.K, L.H, L.W, L.pad, L.m, L.m, L.dtype),
            "launch": "hip-graph replay (up to 10 steps per graph)" if not a.no_graph else "host launches"},
        "fwd_only_ms": r["ms_fwd"],
        "fwd_only_tops": L.direct_ops / (r["ms_fwd"] * 1e-3) / 1e12,
        "im2row_baseline_ms": r["ms_ref"],
        "speedup_vs_im2row": r["ms_ref"] / r["ms_fwd"] if r["ms_ref"] else None,
        "roofline": {k: dominant[k] for k in ("bound", "achieved", "peak", "unit", "frac", "traffic",
                                               "kernel", "avg_us")},
        "kernels": kernels,
        "staged_kernels": [roofline_entry(k, alg[k], us, L.dtype, traffic.get(k))
                           for k, us in r["staged_us"].items()],
    }
    out.update(r["extra"])
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_leg(L)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
