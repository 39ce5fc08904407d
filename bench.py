#!/usr/bin/env python3
"""Benchmark of the Winograd-aware convolution forward path on one MI355X.

A step is one pass of the whole hot path over one batch: weight transform
G g G^T, input transform B^T d B, the per-position GEMMs and the output transform
A^T M A, int8 with a quantizer after every stage.  The default workload is the
CIFAR ResNet-18 stage-1 convolution (batch 64, 32x32, 64->64 channels,
F(4x4,3x3)); inputs are synthetic (seeded ReLU(N(0,1)) activations, Kaiming
weights) and resident in HBM before the timed region starts.

Prints ONE JSON line: direct-convolution-equivalent TOPS of the whole step; the
roofline of the dominant kernel -- its algorithmic bytes against the HBM peak or its GEMM
operations against the matrix-core peak, whichever of the two needs longer (`hbm_frac` and
`mfma_frac` give both; the vector-ALU figure is an extra) -- with per-kernel durations
measured with events on the launch stream; the same for the two largest layers of the
ResNet-18 stack (`largest`); the speedup over the im2row baseline; and the CPU oracle timed
on the host cores as a reported baseline.
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
MFMA_PEAK = {"int8": 5000.0, "f32": 157.3, "bf16": 2500.0}   # dense TOP/s, TFLOP/s
FLOAT = ("f32", "bf16")     # float activations, no quantizer (bf16: bf16 operands in the GEMM)
WIDE = ("i16", "i8w16")    # dtypes with 16-bit codes in the Winograd domain
HBM_TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")


def pick_workload(name):
    table = {}
    for L in (workloads.config2("i8") + workloads.config2("f32") + workloads.config2("bf16") +
              workloads.config2("i16") +
              workloads.config2("i8w16") + workloads.config3() +
              workloads.config4() + workloads.config5()):
        table[L.name] = L
    if name.startswith("layer:"):
        # an ad-hoc int8 layer "layer:N,C,K,H,m" (square image, stride 1, pad 1): for scaling
        # studies of one kernel beyond the sizes the named configurations hold
        try:
            N, C, K, H, m = (int(v) for v in name[6:].split(","))
        except ValueError:
            raise SystemExit("ad-hoc layers are written layer:N,C,K,H,m")
        return workloads.Layer("layer_%d_%dto%d_s%d_F%d" % (N, C, K, H, m), N, C, K, H, H, m=m, seed=7)
    if name not in table:
        raise SystemExit("unknown workload %r; choose from %s (or layer:N,C,K,H,m)" % (name, sorted(table)))
    return table[name]


def bench_scales(name):
    """Quantizer scales of a named workload (calibrated by the oracle, stored by
    tests/golden/make_bench_scales.py).  Ad-hoc layers get fixed, uncalibrated ones: the
    kernels' run time does not depend on the values."""
    table = json.load(open(os.path.join(ROOT, "tests", "golden", "bench_scales.json")))
    if name in table:
        return table[name]
    if name.startswith("layer_"):
        return {"s_x": 0.03, "s_w": 0.002, "s_v": 0.25, "s_u": 0.01, "s_y": 0.1}
    raise SystemExit("no stored scales for workload %r" % name)


ALU_PEAK_TFLOPS = 78.6         # fp32 vector without packed ops: 256 CU x 64 lanes x 2 x 2.4 GHz


def exact_input_stage(L):
    """True where the input transform runs on the matrix cores (int8, F2 / F4, Cook-Toom B^T:
    the kernels with the exact Kronecker form), so that its work is MFMA work, not vector-ALU."""
    return L.dtype == "i8" and L.m in (2, 4) and L.flex_sigma == 0


def algorithmic(L, BT, AT):
    """Bytes / operations the method itself must move / do, per kernel launch.
    `ops` are the GEMM's multiply-adds (x2): the figure the matrix-core roofline prices.
    `mfma_issued` adds the operations the matrix cores are given for the input transform
    where it runs there (one 16x16x64 MFMA per 16 positions, 16 windows and 64 patch bytes).
    `alu` are the fp32 operations issued on the vector ALU: one fused multiply-add
    (2 flops) per nonzero matrix entry and vector element of a transform that runs there,
    one int->float conversion per accumulator, four operations per quantized element
    (scale, round, saturate, convert)."""
    wide = L.dtype in WIDE
    e = 1 if L.dtype in ("i8", "i8w16") else 2 if L.dtype == "i16" else 4   # X, Y element
    ew = 2 if wide or L.dtype == "bf16" else e                              # U, V element
    quantized = L.dtype not in FLOAT
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
    if exact_input_stage(L):
        kron = T * L.C * (-(-P // 16)) * 16 * 64 * 2       # operations given to the matrix cores
        alu_in = T * L.C * qops * P                         # only the quantizer is vector-ALU work
    else:
        kron = 0
        alu_in = T * L.C * (2 * 2 * n * nzb + qops * P)
    alu_out = T * L.K * (2 * (n + L.m) * nza + (P if quantized else 0) + qops * L.m * L.m)
    alu_w = L.K * L.C * (2 * (3 * 3 * n + 3 * n * n) + qops * P)
    return {
        "weight_transform": dict(bytes=9 * L.C * L.K * 4 + u_b, ops=0, alu=alu_w, mfma_issued=0),
        "input_transform": dict(bytes=x_b + v_b, ops=0, alu=alu_in, mfma_issued=kron),
        "gemm": dict(bytes=v_b + u_b + m_b, ops=mm, alu=0, mfma_issued=mm),
        "output_transform": dict(bytes=m_b + y_b, ops=0, alu=alu_out, mfma_issued=0),
        # GEMM and output transform in one kernel: M is never stored
        "gemm_output": dict(bytes=v_b + u_b + y_b, ops=mm, alu=alu_out, mfma_issued=mm),
        # the whole forward in one kernel: neither V nor M is stored
        "fused_forward": dict(bytes=x_b + u_b + y_b, ops=mm, alu=alu_in + alu_out,
                              mfma_issued=mm + kron),
    }


def roofline_entry(name, alg, us, dtype, traffic):
    """The kernel against the roofline that bounds it: its algorithmic bytes at the HBM peak
    or its GEMM operations at the dense matrix-core peak of its dtype, whichever needs the
    longer time.  Both fractions are reported (`hbm_frac`, `mfma_frac`); `alu` is an extra:
    the fp32 operations issued on the vector ALU against its peak (78.6 TFLOP/s without packed
    instructions, which this build may not use)."""
    mf = MFMA_PEAK["int8" if dtype == "i8" or dtype in WIDE else dtype]
    sec = us * 1e-6
    hbm = alg["bytes"] / sec / 1e9
    mfma = alg["ops"] / sec / 1e12
    if alg["bytes"] / (HBM_PEAK_GBS * 1e9) >= alg["ops"] / (mf * 1e12):
        ent = dict(bound="hbm", achieved=hbm, peak=HBM_PEAK_GBS, unit="GB/s")
    else:
        ent = dict(bound="mfma", achieved=mfma, peak=mf,
                   unit="TOP/s" if dtype == "i8" or dtype in WIDE else "TFLOP/s")
    alu = alg["alu"] / sec / 1e12
    ent.update(kernel=name, frac=ent["achieved"] / ent["peak"], avg_us=us,
               hbm_frac=hbm / HBM_PEAK_GBS, mfma_frac=mfma / mf,
               algorithmic_bytes=alg["bytes"], algorithmic_ops=alg["ops"],
               mfma_issued_ops=alg["mfma_issued"], mfma_issued_frac=alg["mfma_issued"] / sec / 1e12 / mf,
               alu=dict(ops=alg["alu"], achieved=alu, peak=ALU_PEAK_TFLOPS, unit="TFLOP/s",
                        frac=alu / ALU_PEAK_TFLOPS),
               traffic=traffic)
    return ent


def csrc_fingerprint():
    """sha256 over the kernel sources: measured HBM traffic is only quoted for the very
    sources it was measured on."""
    import hashlib
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2002_10711_amd", "csrc")
    for f in sorted(os.listdir(d)):
        if f.endswith((".hip", ".h", ".cpp")):
            h.update(f.encode())
            h.update(open(os.path.join(d, f), "rb").read())
    return h.hexdigest()[:16]


def measured_traffic(workload):
    """HBM bytes per launch and kernel from profiles/hbm_traffic.json (rocprofv3 FETCH_SIZE /
    WRITE_SIZE, written by paper_2002_10711_amd.profsummary), or {} with a note if the kernel
    sources have changed since they were measured."""
    if not os.path.exists(HBM_TRAFFIC_FILE):
        return {}, "no traffic file"
    data = json.load(open(HBM_TRAFFIC_FILE))
    fp = data.get("_meta", {}).get("csrc_sha256_16")
    if fp != csrc_fingerprint():
        return {}, "kernel sources changed since the counters were read (measured at %s)" % fp
    return data.get(workload, {}), "rocprofv3 FETCH_SIZE + WRITE_SIZE, csrc %s" % fp


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
    scales = bench_scales(L.name.replace("_f32", "_i8").replace("_bf16", "_i8"))
    X, g = workloads.make_inputs(L)
    BT, G, AT = wb.wino_cook_toom(L.m)
    if L.flex_sigma > 0:
        BT, G, AT = workloads.perturb_transforms(BT, G, AT, L.flex_sigma, L.seed)
    dt = {"i8": wb.WINO_I8, "f32": wb.WINO_F32, "i16": wb.WINO_I16, "i8w16": wb.WINO_I8W16,
          "bf16": wb.WINO_BF16}[L.dtype]
    desc = wb.Desc(L.N, L.C, L.K, L.H, L.W, L.pad, L.m, dt, BT=BT, G=G, AT=AT)
    quant = None
    ydt = torch.float32
    if i8 or wide:
        quant = wb.make_quant(scales["s_x"], scales["s_v"], scales["s_u"], scales["s_y"], 0.0, qm["y"],
                              qmax_u=qm["u"], qmax_v=qm["v"], qmax_m=qm["m"], qmax_y=qm["y"])
        # input codes of the previous layer's quantizer (input preparation, not the path)
        xh = workloads.input_codes(X, scales["s_x"], qm["x"], np.int16 if L.dtype == "i16" else np.int8)
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
    # (the bf16 variant exists as one kernel only)
    acc_staged = acc if nk == 3 else {} if L.dtype == "bf16" else time_stages(
        [("weight_transform", None), ("input_transform", wb.WINO_STAGE_INPUT),
         ("gemm", wb.WINO_STAGE_GEMM), ("output_transform", wb.WINO_STAGE_OUTPUT)])

    # im2row baseline on the same layer, forward only (weights packed once)
    # (the baseline has int8 and fp32 forms: 8-bit activations are compared with the int8
    # one, the int16 workload has no baseline)
    s_w = scales.get("s_w", 1.0)
    rdt = wb.WINO_F32 if L.dtype in FLOAT else wb.WINO_I8
    ms_ref = ms_ref_rows = None
    if L.dtype != "i16":
        if rdt == wb.WINO_I8:
            wq = workloads.input_codes(g, s_w)
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

        # the same baseline with the row matrix written out (three kernels)
        def ref_rows_fwd():
            wb.conv2d_ref_gpu_rows(L.N, L.C, L.K, L.H, L.W, 1, L.pad, rdt, x, wp, y, scales["s_x"],
                                   s_w, scales["s_y"], 127, rws, stream=stream)

        ms_ref_rows = timed(ref_rows_fwd, max(10, steps // 8), max(2, warmup // 8))
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
    return dict(extra=extra, ms_step=ms_step, ms_fwd=ms_fwd, ms_ref=ms_ref, ms_ref_rows=ms_ref_rows, kernel_us=acc, staged_us=acc_staged,
                BT=BT, AT=AT)


def load_probe():
    """Bytes per cycle and compute unit (at the 2.1 GHz the chip sustains, 256 compute units)
    that the vector memory path delivers, per load form, wavefronts per workgroup and
    footprint: 16 KB per workgroup stays in the L1, 64 KB in the XCD's L2 (16 MB in all), 256 KB
    (64 MB in all) in neither."""
    import torch
    from paper_2002_10711_amd import binding as wb
    dev = torch.device("cuda:0")
    stream = torch.cuda.Stream()
    wgs = 256
    buf = torch.ones(wgs * (256 << 10), dtype=torch.uint8, device=dev)
    out = torch.empty(wgs * 1024, dtype=torch.float32, device=dev)
    names = {0: "16 B/lane", 1: "8 B/lane", 2: "4 B/lane", 3: "16 B/lane into LDS"}
    rows = []
    with torch.cuda.stream(stream):
        for kb in (16, 64, 256):
            for waves in (4, 8, 16):
                for mode in (0, 1, 2, 3):
                    if mode in (1, 2) and waves != 4:
                        continue
                    iters = 400
                    wb.wino_debug_load_loop(mode, waves, wgs, kb << 10, 50, buf, out, stream=stream)
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record(stream)
                    nbytes = wb.wino_debug_load_loop(mode, waves, wgs, kb << 10, iters, buf, out, stream=stream)
                    e1.record(stream)
                    stream.synchronize()
                    tbs = nbytes / (e0.elapsed_time(e1) * 1e-3) / 1e12
                    rows.append({"load": names[mode], "waves_per_workgroup": waves, "workgroups": wgs,
                                 "footprint_kb_per_workgroup": kb, "TB_per_s": round(tbs, 2),
                                 "bytes_per_clk_per_cu": round(tbs * 1e12 / 2.1e9 / 256, 1)})
    print(json.dumps({"probe": "vector memory path (wino_debug_load_loop)", "rows": rows}))


def ref_only_leg(L, steps, warmup):
    """ms per forward of the im2row baseline on a layer (stride 1 or 2), weights packed once."""
    import torch
    from paper_2002_10711_amd import binding as wb
    dev = torch.device("cuda:0")
    sc = bench_scales(L.name)
    X, g = workloads.make_inputs(L)
    xh = workloads.input_codes(X, sc["s_x"])
    wq = workloads.input_codes(g, sc["s_w"])
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
        "im2row_stack_ms": t_ref, "speedup_vs_im2row": t_ref / t_wino,
        # the faster of the two per layer: what a latency-aware choice of the algorithm per
        # layer (the paper's search, Sec. 4) would run on this machine
        "best_per_layer_ms": sum(min(r["fwd_us"], r["im2row_us"]) for r in rows) * 1e-3,
        "layers": rows,
    }


LARGEST = {
    # the layer with the most bytes through the transforms, and the GEMM-dominated one
    "transforms": "cfg5_l00_64to64_s32_F4",
    "gemm": "cfg5_l15_512to512_s4_F2",
}


def largest_block(steps, warmup, use_graph):
    """The two largest layers of the ResNet-18 stack (batch 256): forward time, and every
    kernel of the forward and of the same layer as four separate kernels against its
    roofline."""
    out = {}
    for role, name in LARGEST.items():
        L = pick_workload(name)
        r = gpu_leg(L, steps, warmup, use_graph)
        alg = algorithmic(L, r["BT"], r["AT"])
        traffic, note = measured_traffic(L.name)
        keys = ("kernel", "avg_us", "bound", "frac", "hbm_frac", "mfma_frac", "mfma_issued_frac",
                "algorithmic_bytes", "algorithmic_ops", "traffic")

        def rows(us):
            return [{k: e[k] for k in keys} for e in
                    (roofline_entry(k, alg[k], t, L.dtype, traffic.get(k)) for k, t in us.items())]
        out[role] = dict(workload="%s: N=%d C=%d K=%d %dx%d F(%dx%d,3x3) int8" % (
            L.name, L.N, L.C, L.K, L.H, L.W, L.m, L.m), steps=steps,
            fwd_us=r["ms_fwd"] * 1e3, fwd_tops=L.direct_ops / (r["ms_fwd"] * 1e-3) / 1e12,
            im2row_us=r["ms_ref"] * 1e3 if r["ms_ref"] else None,
            kernels=rows(r["kernel_us"]), staged_kernels=rows(r["staged_us"]), traffic_source=note)
    return out


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_leg(L):
    """The oracle as it stands, on the host cores, on the first images of the same workload:
    the quantized pipeline (weight stage included) with OpenMP -- the headline `value` -- and
    next to it the fp64 direct convolution and the fp64 literal Winograd, each with OpenMP on
    all cores and on one thread (fewer images, stated)."""
    import oracle
    oracle.build()
    from dataclasses import replace
    X, g = workloads.make_inputs(L)
    BT, G, AT = oracle.cook_toom(L.m, dtype=np.float32)
    if L.flex_sigma > 0:
        BT, G, AT = workloads.perturb_transforms(BT, G, AT, L.flex_sigma, L.seed)
    threads = oracle.num_threads()

    def timed(fn, budget):
        fn()
        t0 = time.perf_counter()
        reps = 0
        while time.perf_counter() - t0 < budget or reps < 2:
            fn()
            reps += 1
        return (time.perf_counter() - t0) / reps, reps

    def tops(n_img, dt):
        return replace(L, N=n_img).direct_ops / dt / 1e12

    n_omp, n_one = min(L.N, 16), min(L.N, 2)
    runs = {}
    if L.dtype not in FLOAT:
        sc = bench_scales(L.name)
        qm = workloads.STAGE_QMAX[L.dtype]
        xq = oracle.quantize_tensor(X[:n_omp], sc["s_x"], qm["x"])
        main_fn = lambda n: (lambda: oracle.winograd_q(xq[:n], g, BT, G, AT, sc, pad=L.pad, qmax=qm))
        main_name = "quantized_pipeline"
    else:
        main_fn = lambda n: (lambda: oracle.winograd_f64(X[:n], g, BT, G, AT, L.pad))
        main_name = "winograd_f64"
    legs = [(main_name, main_fn, 8.0, 3.0),
            ("direct_f64", lambda n: (lambda: oracle.conv2d_direct_f64(X[:n], g, 1, L.pad)), 3.0, 2.0)]
    if L.dtype not in FLOAT:
        legs.append(("winograd_f64", lambda n: (lambda: oracle.winograd_f64(X[:n], g, BT, G, AT, L.pad)),
                     3.0, 2.0))
    for name, mk, b_omp, b_one in legs:
        oracle.set_num_threads(threads)
        dt, reps = timed(mk(n_omp), b_omp)
        runs[name + "_openmp"] = dict(tops=tops(n_omp, dt), threads=threads, images=n_omp,
                                      seconds_per_pass=dt, passes=reps)
        oracle.set_num_threads(1)
        dt, reps = timed(mk(n_one), b_one)
        runs[name + "_1_thread"] = dict(tops=tops(n_one, dt), threads=1, images=n_one,
                                        seconds_per_pass=dt, passes=reps)
    oracle.set_num_threads(threads)
    head = runs[main_name + "_openmp"]
    return dict(value=head["tops"], unit="TOPS (direct-conv-equivalent)", cores=threads,
                kind="oracle", cpu_model=cpu_model(),
                sample="first %d of %d images of %s, %d passes of %.3f s; %s incl. weight stage, "
                       "OpenMP over tiles; `runs` holds the fp64 direct convolution and the fp64 "
                       "literal Winograd as well, each with OpenMP and on one thread (first %d images)"
                       % (n_omp, L.N, L.name, head["passes"], head["seconds_per_pass"],
                          main_name.replace("_", " "), n_one),
                runs=runs)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5000)
    ap.add_argument("--warmup", type=int, default=2000)
    ap.add_argument("--workload", default="cfg2_i8")
    ap.add_argument("--no-graph", action="store_true", help="launch every step from the host "
                    "instead of replaying a captured HIP graph of one step")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-largest", action="store_true", help="skip the `largest` block (the two "
                    "largest layers of the ResNet-18 stack, timed next to the default workload)")
    ap.add_argument("--stack", action="store_true", help="time the whole CIFAR ResNet-18 conv "
                    "stack (config 5: 16 layers, batch 256, int8) layer by layer, forward only, "
                    "and print its total instead of one workload's line")
    ap.add_argument("--flex", type=float, default=0.0, help="perturb the Cook-Toom matrices by "
                    "seeded N(0, FLEX) noise (dense 'learned' transforms, paper Sec. 3.2): a timing "
                    "option, the stored scales are not recalibrated")
    ap.add_argument("--load-probe", action="store_true", help="only measure what the vector memory "
                    "path of a compute unit delivers (wino_debug_load_loop) for footprints that fit "
                    "the L1, the L2 and neither, and print the table as one JSON line")
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
    if a.load_probe:
        load_probe()
        return
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
    traffic, traffic_note = measured_traffic(L.name)
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
        "dtype": {"i8": "int8", "f32": "f32", "i16": "int16", "i8w16": "int8 data, int16 Winograd domain",
                  "bf16": "f32 data, bf16 operands in the Winograd-domain GEMM"}[L.dtype],
        "data": "synthetic",
        "config": {"workload": "%s: N=%d C=%d K=%d %dx%d pad=%d F(%dx%d,3x3) %s" % (
            L.name, L.N, L.C, L.K, L.H, L.W, L.pad, L.m, L.m, L.dtype),
            "launch": "hip-graph replay (up to 10 steps per graph)" if not a.no_graph else "host launches"},
        "fwd_only_ms": r["ms_fwd"],
        "fwd_only_tops": L.direct_ops / (r["ms_fwd"] * 1e-3) / 1e12,
        "im2row_baseline_ms": r["ms_ref"],
        # (the baseline as built: for int8 one kernel that gathers the im2row rows in LDS,
        # multiplies and requantizes; its own matrix-core fraction next to the ratio, so
        # that a weak baseline shows; `im2row_rows_ms` is the form that writes the row matrix)
        "im2row_rows_ms": r["ms_ref_rows"],
        "im2row_baseline_tops": L.direct_ops / (r["ms_ref"] * 1e-3) / 1e12 if r["ms_ref"] else None,
        "im2row_baseline_mfma_frac": (L.direct_ops / (r["ms_ref"] * 1e-3) / 1e12 /
                                      MFMA_PEAK["f32" if L.dtype in FLOAT else "int8"])
        if r["ms_ref"] else None,
        "speedup_vs_im2row": r["ms_ref"] / r["ms_fwd"] if r["ms_ref"] else None,
        "roofline": {k: dominant[k] for k in ("bound", "achieved", "peak", "unit", "frac", "traffic",
                                               "kernel", "avg_us")},
        "hbm_frac": dominant["hbm_frac"], "mfma_frac": dominant["mfma_frac"],
        "traffic_source": traffic_note,
        "kernels": kernels,
        "staged_kernels": [roofline_entry(k, alg[k], us, L.dtype, traffic.get(k))
                           for k, us in r["staged_us"].items()],
        "timing_note": "ms_per_step and fwd_only_ms: HIP graphs of whole steps; per-kernel avg_us: "
                       "each stage in a graph of its own of ten back-to-back launches, which "
                       "includes the gap between two launches that a step graph partly hides",
    }
    if a.workload == "cfg2_i8" and not a.no_largest:
        out["largest"] = largest_block(max(200, a.steps // 5), max(50, a.warmup // 5), not a.no_graph)
    out.update(r["extra"])
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_leg(L)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
