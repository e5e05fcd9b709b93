#!/usr/bin/env python3
"""Benchmark of the group-wise int8 quantized Winograd convolution on one MI355X.

A step is one forward pass (input transform + quantization, int8 contraction
with per-group dequantization, output transform + bias) over every layer of
the workload, inputs and prepared weights resident in HBM.  The step's kernel
launches are captured once into a HIP graph (the layers are a few microseconds
each, so host launch cost would otherwise dominate) and the timed region
replays that graph.  The weight transform is the method's offline stage: it
runs once before the timed region and is timed separately (per layer in
"layers", and as a second whole-job figure "with_offline_stage" that re-runs
it inside every step).

Prints ONE JSON line.  `value` = direct-equivalent int8 TOPS of the layer set
(2*N*H*W*Cin*Cout*9 per layer / measured time).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
INT8_PEAK_TOPS = 5000.0        # MI355X published dense int8 MFMA rate
VALU_PEAK_OPS = 256 * 64 * 2.4e9   # fp32 vector operations per second without packed math: 256 CUs x 4 SIMDs x 16 lanes


def k1_bytes(lay):
    n2, G = lay.n ** 2, lay.Cin // lay.group_size
    return 4 * lay.N * lay.H * lay.W * lay.Cin + n2 * lay.tiles * (lay.Cin + 4 * G)


def k2_bytes(lay):
    n2, G = lay.n ** 2, lay.Cin // lay.group_size
    return (n2 * lay.tiles * (lay.Cin + 4 * G) + n2 * lay.Cout * (lay.Cin + 4 * G)
            + 4 * lay.N * lay.H * lay.W * lay.Cout)


def k3_bytes(lay):
    n2, G = lay.n ** 2, lay.Cin // lay.group_size
    return 36 * lay.Cin * lay.Cout + n2 * lay.Cout * (lay.Cin + 4 * G)


def measured_traffic(kernel, cfg):
    """HBM bytes per step of the dominant kernel as measured with rocprofv3 --pmc
    (FETCH_SIZE + WRITE_SIZE, calibrated against a copy kernel); read from the
    committed summary, None when there is none for this kernel and layer set."""
    path = os.path.join(ROOT, "profiles", f"{kernel}_cfg{cfg}_hbm_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_step:"):
                return int(float(line.split(":")[1]))
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=2, help="layer set 1..5 (2 = the headline one); 6 = an extra large GEMM-shaped layer at "
                         "two group sizes, outside the five configurations (no host baseline)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--eager", action="store_true",
                    help="launch the step from Python instead of replaying a HIP graph (for profilers)")
    ap.add_argument("--only-steps", action="store_true",
                    help="launch warmup+steps steps eagerly, print the launch count and exit (for counter "
                         "runs: every dispatch in the process then belongs to a step)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a 256 MiB device-to-device copy three times (known HBM traffic, "
                         "used to calibrate the FETCH_SIZE / WRITE_SIZE counters) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
                 "(the path would shard without communication over tiles or output channels)")

    import numpy as np
    import torch
    from paper_2412_19867_amd import wq, workloads

    wq.lib()   # fails loudly when the HIP library is missing; there is no fallback
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.copy_calibration:
        src = torch.ones(64 << 20, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": src.numel() * 4, "copy_bytes_written": src.numel() * 4}))
        return
    stream = torch.cuda.current_stream()

    layers = workloads.CONFIGS[args.config]
    items = []      # one entry per conv launched in a step (a layer with repeat=r gives r chained convs)
    for lay in layers:
        d = workloads.make_layer_data(lay)
        kw = {}
        if d.u_B is not None:
            AT, BT, G = wq.scaled_transforms(lay.m, d.u_B, d.u_G)
            kw = dict(AT=AT, BT=BT, G=G)
        plan = wq.Plan(lay.N, lay.H, lay.W, lay.Cin, lay.Cout, lay.m, lay.group_size, **kw)
        x = torch.from_numpy(d.x).cuda()
        w, b = torch.from_numpy(d.w).cuda(), torch.from_numpy(d.bias).cuda()
        for r in range(lay.repeat):
            # conv r of a stack reads conv r-1's output (Cin == Cout) and has its own weight blob
            it = dict(lay=lay, plan=plan, x=x, w=w, b=b, blob=plan.alloc_blob(),
                      ws=plan.alloc_workspace(), y=plan.alloc_output(), data=d, first=(r == 0))
            plan.weight_prepare(w, b, it["blob"])
            items.append(it)
            x = it["y"]
    torch.cuda.synchronize()

    def step(with_offline=False):
        for it in items:
            if with_offline:
                it["plan"].weight_prepare(it["w"], it["b"], it["blob"])
            it["plan"].forward(it["x"], it["blob"], it["ws"], it["y"])

    if args.only_steps:
        for _ in range(args.warmup + args.steps):
            step()
        torch.cuda.synchronize()
        print(json.dumps({"steps_launched": args.warmup + args.steps, "convs_per_step": len(items),
                          "offline_stage_launches": len(items)}))
        return

    side = torch.cuda.Stream()

    def capture(fn):
        """Record fn's launches on a side stream into a HIP graph."""
        with torch.cuda.stream(side):
            fn()
            side.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                fn()
        torch.cuda.synchronize()
        return g

    def timed_replays(g, steps, warmup):
        with torch.cuda.stream(side):
            for _ in range(warmup):
                g.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                g.replay()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) / steps

    # Three ways to launch the same K steps; the timed figure is the fastest one, named in
    # "launch".  (a) one graph per step, replayed K times; (b) one graph holding 10 steps,
    # replayed K/10 times (a replay costs several microseconds of its own, which a 120 us
    # step notices); (c) plain launches from Python, which run asynchronously ahead of the GPU.
    def timed_eager(steps, warmup):
        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    timings = {}
    if args.eager:
        timings["eager launches from Python"] = timed_eager(args.steps, args.warmup)
    else:
        g_step = capture(step)
        timings["one HIP graph replay per step"] = timed_replays(g_step, args.steps, args.warmup)
        if args.steps % 10 == 0:
            g10 = capture(lambda: [step() for _ in range(10)])
            timings["HIP graph of 10 steps, replayed steps/10 times"] = \
                timed_replays(g10, args.steps // 10, max(1, args.warmup // 10)) / 10
        timings["eager launches from Python"] = timed_eager(args.steps, args.warmup)
    launch_mode = min(timings, key=timings.get)
    sec = timings[launch_mode]
    n_convs = len(items)
    direct_ops = sum(it['lay'].direct_ops for it in items)
    value = direct_ops / sec / 1e12

    g_off = capture(lambda: step(True))
    sec_off = timed_replays(g_off, max(10, args.steps // 4), 3)

    # ---- the same step with cold caches: consecutive steps use different copies of every buffer
    # (inputs, weight blobs, workspaces, outputs), enough copies to exceed the 256 MB Infinity Cache
    # twice over, so nothing a step reads is left over from the step before.  Reported beside the
    # warm figure, which is the timed one: inside a network the activations a layer reads were
    # written just before and are warm, its weights are not.
    footprint = sum(it["x"].numel() * 4 * it["first"] + it["blob"].numel() + it["ws"].numel()
                    + it["y"].numel() * 4 for it in items)
    cold = None
    n_sets = min(8, -(-(512 << 20) // footprint)) if footprint < (512 << 20) else 1
    if n_sets > 1:
        sets = [items]
        for _ in range(n_sets - 1):
            clone, x_prev = [], None
            for it in items:
                c = dict(it)
                c["x"] = it["x"].clone() if it["first"] else x_prev
                c["blob"], c["ws"], c["y"] = it["blob"].clone(), torch.empty_like(it["ws"]), torch.empty_like(it["y"])
                x_prev = c["y"]
                clone.append(c)
            sets.append(clone)

        def step_of(k):
            for it in sets[k % n_sets]:
                it["plan"].forward(it["x"], it["blob"], it["ws"], it["y"])

        for k in range(n_sets * 2):
            step_of(k)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(args.steps):
            step_of(k)
        torch.cuda.synchronize()
        sec_cold = (time.perf_counter() - t0) / args.steps
        cold = dict(buffer_sets=n_sets, footprint_mb_per_set=round(footprint / 1e6, 1),
                    ms_per_step=round(sec_cold * 1e3, 4), value=round(direct_ops / sec_cold / 1e12, 2),
                    unit="TOPS", launch="eager launches from Python")
        del sets

    # ---- per-kernel durations: HIP events on the replay stream around a graph that
    # launches ONE kernel REPS times back to back (so the figure is device time, not
    # host launch cost) ----
    REPS = 20

    def kernel_us(fn):
        g = capture(lambda: [fn() for _ in range(REPS)])
        with torch.cuda.stream(side):
            g.replay()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(side)
            for _ in range(5):
                g.replay()
            e1.record(side)
            torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / (5 * REPS)

    k1_us = [kernel_us(lambda it=it: it["plan"].input_transform(it["x"], it["ws"])) for it in items]
    k2_us = [kernel_us(lambda it=it: it["plan"].contract_output(it["ws"], it["blob"], it["y"]))
             for it in items]
    k3_us = [kernel_us(lambda it=it: it["plan"].weight_prepare(it["w"], it["b"], it["blob"]))
             for it in items]
    # layers whose stages 2+3 run as two kernels: each kernel on its own
    split_us = {k: (kernel_us(lambda it=it: it["plan"].contract(it["ws"], it["blob"])),
                    kernel_us(lambda it=it: it["plan"].output_transform(it["ws"], it["blob"], it["y"])))
                for k, it in enumerate(items) if it["plan"].layout.k2_kernels == 2}

    per_layer = []
    for k, it in enumerate(items):
        lay = it["lay"]
        t_us = k1_us[k] + k2_us[k]
        per_layer.append(dict(
            layer=lay.name, us=round(t_us, 2), k1_us=round(k1_us[k], 2), k2_us=round(k2_us[k], 2),
            direct_equiv_tops=round(lay.direct_ops / t_us / 1e6, 1),
            k1_hbm_frac=round(k1_bytes(lay) / (k1_us[k] * 1e-6) / 1e9 / HBM_PEAK_GBS, 3),
            k2_hbm_frac=round(k2_bytes(lay) / (k2_us[k] * 1e-6) / 1e9 / HBM_PEAK_GBS, 3),
            k2_mfma_frac=round(2 * lay.n ** 2 * lay.tiles * lay.Cin * lay.Cout
                               / (k2_us[k] * 1e-6) / 1e12 / INT8_PEAK_TOPS, 4),
            # the ceilings of stages 2+3: bytes, MFMA work, and the plain-ALU work the method
            # forces (3 fp32 vector operations per output element, tap and group for the
            # dequantization, unpacked: 256 CUs x 64 lanes x 2.4 GHz), each as time / measured time
            k2_valu_frac=round(3 * lay.n ** 2 * lay.tiles * (lay.Cin // lay.group_size) * lay.Cout
                               / (k2_us[k] * 1e-6) / VALU_PEAK_OPS, 4),
            k2_kernels=it["plan"].layout.k2_kernels, k3_us=round(k3_us[k], 2),
            k3_hbm_frac=round(k3_bytes(lay) / (k3_us[k] * 1e-6) / 1e9 / HBM_PEAK_GBS, 3)))

    # per-kernel totals over one step.  Stages 2+3 of a layer are one fused kernel or,
    # for layers with few tiles, a tiled GEMM followed by an output-transform kernel.
    kernels = {}

    def account(name, us, nbytes, launches):
        k = kernels.setdefault(name, dict(us=0.0, bytes=0, launches=0))
        k["us"] += us
        k["bytes"] += nbytes
        k["launches"] += launches

    for k, it in enumerate(items):
        lay = it["lay"]
        account("k_input_transform", k1_us[k], k1_bytes(lay), 1)
        if it["plan"].layout.k2_kernels == 1:
            account("k_contract_output", k2_us[k], k2_bytes(lay), 1)
        else:
            # the fp32 product tensor M is written by the GEMM and read back by the transform
            m_bytes = 4 * lay.n ** 2 * lay.tiles * lay.Cout
            y_bytes = 4 * lay.N * lay.H * lay.W * lay.Cout
            account("k_gemm_dequant", split_us[k][0], k2_bytes(lay) - y_bytes + m_bytes, 1)
            account("k_output_transform", split_us[k][1], m_bytes + y_bytes, 1)
    dom = max(kernels, key=lambda name: kernels[name]["us"])
    dk = kernels[dom]
    achieved = dk["bytes"] / (dk["us"] * 1e-6) / 1e9
    roofline = dict(bound="hbm", kernel=dom, achieved=round(achieved, 1), peak=HBM_PEAK_GBS,
                    unit="GB/s", frac=round(achieved / HBM_PEAK_GBS, 4),
                    traffic=measured_traffic(dom, args.config),
                    algorithmic_bytes_per_step=dk["bytes"],
                    avg_launch_us=round(dk["us"] / dk["launches"], 2),
                    launches_per_step=dk["launches"],
                    kernels={name: dict(us_per_step=round(v["us"], 2), launches=v["launches"],
                                        algorithmic_bytes=v["bytes"],
                                        hbm_frac=round(v["bytes"] / (v["us"] * 1e-6) / 1e9 / HBM_PEAK_GBS, 4))
                             for name, v in kernels.items()})

    # ---- the paper's runtime comparison point on the same layers: the group-wise quantized
    # standard (direct) convolution, same quantizer and groups, no transforms
    d_items = []
    for it in items:
        lay = it["lay"]
        dp = wq.DirectPlan(lay.N, lay.H, lay.W, lay.Cin, lay.Cout, lay.group_size)
        dit = dict(plan=dp, blob=dp.alloc_blob(), ws=dp.alloc_workspace(), x=it["x"], y=it["y"])
        dp.weight_prepare(it["w"], it["b"], dit["blob"])
        d_items.append(dit)
    torch.cuda.synchronize()

    def direct_step():
        for dit in d_items:
            dit["plan"].forward(dit["x"], dit["blob"], dit["ws"], dit["y"])

    # same launch choices as for the Winograd step (graph per step / graph of 10 steps)
    sec_direct = timed_replays(capture(direct_step), max(10, args.steps // 2), 5)
    if args.steps % 10 == 0:
        g10d = capture(lambda: [direct_step() for _ in range(10)])
        sec_direct = min(sec_direct, timed_replays(g10d, max(2, args.steps // 20), 1) / 10)
    dq_us = [kernel_us(lambda dit=dit: dit["plan"].quantize(dit["x"], dit["ws"])) for dit in d_items]
    dc_us = [kernel_us(lambda dit=dit: dit["plan"].conv(dit["ws"], dit["blob"], dit["y"])) for dit in d_items]
    direct = dict(value=round(direct_ops / sec_direct / 1e12, 2), unit="TOPS",
                  ms_per_step=round(sec_direct * 1e3, 4),
                  winograd_over_direct=round(sec_direct / sec, 3),
                  layers=[dict(layer=it["lay"].name, quantize_us=round(dq_us[k], 2),
                               conv_us=round(dc_us[k], 2)) for k, it in enumerate(items)])
    # the step above overwrote y with the direct path's outputs; restore the Winograd results
    step()
    torch.cuda.synchronize()

    # ---- the same quantized GEMM core as a linear layer (one tap): one attention-sized projection
    lin_R, lin_C, lin_g = 4096, 1280, 64
    lp = wq.DirectPlan(lin_R, 1, 1, lin_C, lin_C, lin_g, linear=True)
    lblob, lws, ly = lp.alloc_blob(), lp.alloc_workspace(), lp.alloc_output()
    lx = torch.randn(lin_R, lin_C, device="cuda")
    lp.weight_prepare(torch.randn(lin_C, lin_C, device="cuda") * 0.02, None, lblob)
    lq_us = kernel_us(lambda: lp.quantize(lx, lws))
    lc_us = kernel_us(lambda: lp.conv(lws, lblob, ly))
    # the same layer with 4-bit weight codes (W4A8), and a decode-sized batch of 16 rows against a
    # 5120 x 5120 weight matrix, where the weights are the traffic
    lp4 = wq.DirectPlan(lin_R, 1, 1, lin_C, lin_C, lin_g, linear=True, weight_bits=4)
    lblob4 = lp4.alloc_blob()
    lp4.weight_prepare(torch.randn(lin_C, lin_C, device="cuda") * 0.02, None, lblob4)
    lc4_us = kernel_us(lambda: lp4.conv(lws, lblob4, ly))
    sm_R, sm_C = 16, 5120
    small = {}
    for bits in (8, 4):
        sp = wq.DirectPlan(sm_R, 1, 1, sm_C, sm_C, lin_g, linear=True, weight_bits=bits)
        sblob, sws, sy = sp.alloc_blob(), sp.alloc_workspace(), sp.alloc_output()
        sp.weight_prepare(torch.randn(sm_C, sm_C, device="cuda") * 0.02, None, sblob)
        sp.quantize(torch.randn(sm_R, sm_C, device="cuda"), sws)
        small[f"w{bits}a8_gemm_us"] = round(kernel_us(lambda: sp.conv(sws, sblob, sy)), 2)
    linear = dict(shape=f"{lin_R}x{lin_C}->{lin_C}, g={lin_g}", quantize_us=round(lq_us, 2),
                  gemm_us=round(lc_us, 2),
                  int8_tops=round(2 * lin_R * lin_C * lin_C / ((lq_us + lc_us) * 1e-6) / 1e12, 1),
                  w4a8_gemm_us=round(lc4_us, 2),
                  w4a8_tops=round(2 * lin_R * lin_C * lin_C / ((lq_us + lc4_us) * 1e-6) / 1e12, 1),
                  small_batch=dict(shape=f"{sm_R}x{sm_C}->{sm_C}, g={lin_g}", **small))

    cpu_baseline = None
    if not args.no_cpu_baseline and args.config != 6:
        import oracle
        from oracle import cook_toom as ct
        prepared = []
        for it in items:
            if not it["first"]:
                continue
            lay, d = it["lay"], it["data"]
            if d.u_B is not None:
                AT, BT, G = (M.astype(np.float32) for M in ct.scaled_matrices(lay.m, d.u_B, d.u_G))
            else:
                AT, BT, G = (M.astype(np.float32) for M in ct.standard_matrices(lay.m))
            Wq, sW = oracle.weight_transform_quant(d.w, G, lay.m, lay.group_size)
            prepared.append((lay, d, AT, BT, Wq, sW))

        def cpu_pass():
            for lay, d, AT, BT, Wq, sW in prepared:
                Xq, sX = oracle.input_transform_quant(d.x, BT, lay.m, lay.group_size)
                M = oracle.contract(Xq, sX, Wq, sW, lay.group_size)
                oracle.output_transform(M, AT, d.bias, lay.N, lay.H, lay.W, lay.m)

        cpu_pass()
        t0 = time.perf_counter()
        passes = 0
        while passes < 3 or (time.perf_counter() - t0 < 10 and passes < 50):
            cpu_pass()
            passes += 1
        cpu_sec = (time.perf_counter() - t0) / passes
        cpu_ops = sum(l.direct_ops for l in layers)
        cpu_baseline = dict(value=round(cpu_ops / cpu_sec / 1e12, 5), unit="TOPS",
                            cores=oracle.threads(), kind="oracle",
                            sample=f"{passes} forward passes over the full layer set (one conv per "
                                   f"layer, weights prepared beforehand), {cpu_sec:.2f} s per pass",
                            ms_per_pass=round(cpu_sec * 1e3, 1))

    out = dict(
        metric="direct-equivalent int8 TOPS of the group-wise quantized Winograd conv layer set "
               "(2*N*H*W*Cin*Cout*9 per layer / time); per-layer us in 'layers'",
        value=round(value, 2), unit="TOPS", n_gpus=1, steps=args.steps, warmup=args.warmup,
        ms_per_step=round(sec * 1e3, 4), us_per_layer=round(sec * 1e6 / n_convs, 2),
        launch=launch_mode, ms_per_step_by_launch={k: round(v * 1e3, 4) for k, v in timings.items()},
        higher_is_better=True, scaling="weak", vs_baseline=None, dtype="int8",
        data="synthetic",
        config=dict(workload=f"configs[{args.config - 1}]: " + "; ".join(l.name for l in layers),
                    winograd=f"F({layers[0].m},3)", group_size=layers[0].group_size,
                    batch=layers[0].N, convs_per_step=n_convs),
        roofline=roofline, cpu_baseline=cpu_baseline, direct_conv_same_layers=direct,
        cold_cache=cold, quantized_linear_layer=linear,
        with_offline_stage=dict(value=round(direct_ops / sec_off / 1e12, 2), unit="TOPS",
                                ms_per_step=round(sec_off * 1e3, 4)),
        layers=per_layer)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
