#!/usr/bin/env python3
"""Benchmark of the group-wise int8 quantized Winograd convolution on one MI355X.

A step is one forward pass (input transform + quantization, int8 contraction
with per-group dequantization, output transform + bias) over every convolution
of the workload, inputs and prepared weights resident in HBM, all launches on
one stream.  The headline workload is the largest single-GPU configuration:
configs[4], the SDXL-scale stack (12 chained 3x3 convolutions at 128x128, 64x64
and 32x32 latent resolution, F(4,3), groups of 64).  The K timed steps are
launched in three ways (one HIP graph replay per step, one replay of a graph
holding several steps, plain launches); every way is timed REPEATS times and
its median taken, and the fastest way's median is the reported figure.  The
weight transform is the method's offline stage: it runs once before the timed
region and is timed separately ("with_offline_stage" re-runs it inside every
step).

Prints ONE JSON line.  `value` = direct-equivalent int8 TOPS of the workload
(2*N*H*W*Cin*Cout*9 per convolution / measured time).
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
INT8_PEAK_TOPS = 5000.0        # MI355X published dense int8 MFMA rate
VALU_PEAK_OPS = 78.65e12       # fp32 vector operations per second: the published 157.3 TFLOP/s counts a multiply-add as two
REPEATS = 10                   # timed repetitions of the --steps block per launch mode (median reported)


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


def k2_ceilings_us(lay):
    """The three lower bounds of stages 2+3 in microseconds: algorithmic bytes at the HBM peak, the
    Winograd-domain int8 multiply-adds at the MFMA peak, and the plain vector-ALU work the method
    forces (3 fp32 operations per output element, tap and group for the dequantization)."""
    n2, G = lay.n ** 2, lay.Cin // lay.group_size
    return dict(hbm=k2_bytes(lay) / (HBM_PEAK_GBS * 1e9) * 1e6,
                mfma=2 * n2 * lay.tiles * lay.Cin * lay.Cout / (INT8_PEAK_TOPS * 1e12) * 1e6,
                valu=3 * n2 * lay.tiles * G * lay.Cout / VALU_PEAK_OPS * 1e6)


def library_sources_sha256():
    """Hash of the kernel sources the library is built from: a counter summary under profiles/
    names the hash it was measured with, and is ignored when the sources have changed since."""
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2412_19867_amd", "csrc")
    for name in sorted(os.listdir(d)):
        if name.endswith((".hip", ".h", ".cpp")):
            h.update(name.encode())
            h.update(open(os.path.join(d, name), "rb").read())
    return h.hexdigest()[:16]


def measured_traffic(kernel, cfg):
    """HBM bytes per step of a kernel from rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE, calibrated
    against a copy kernel), read from the committed summary profiles/<kernel>_cfg<N>_hbm_traffic.txt.
    Returns (bytes or None, note)."""
    path = os.path.join(ROOT, "profiles", f"{kernel}_cfg{cfg}_hbm_traffic.txt")
    try:
        fields = dict(line.split(":", 1) for line in open(path) if ":" in line and not line.startswith("#"))
    except OSError:
        return None, "no counter summary for this kernel and workload under profiles/"
    sha = fields.get("library_sources_sha256", "").strip()
    if sha != library_sources_sha256():
        return None, f"profiles/{os.path.basename(path)} was measured with other kernel sources ({sha}): ignored"
    return int(float(fields["traffic_bytes_per_step"])), f"profiles/{os.path.basename(path)}"


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=5,
                    help="layer set 1..5 (5 = the headline one, configs[4]); 6 = an extra large GEMM-shaped "
                         "layer at two group sizes, outside the five configurations (no host baseline)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the comparison layer, the linear layer and the other configurations")
    ap.add_argument("--eager", action="store_true",
                    help="launch the step from Python instead of replaying a HIP graph (for profilers)")
    ap.add_argument("--only-steps", action="store_true",
                    help="launch warmup+steps steps eagerly, print the launch count and exit (for counter "
                         "runs: every dispatch in the process then belongs to a step)")
    ap.add_argument("--k2-variant", default=None,
                    help="force this kernel variant of stages 2+3 on every layer it applies to, or "
                         "'i:name,j:name' on layers i, j of the set (for before/after profiles; the "
                         "default is the plan's own choice per layer)")
    ap.add_argument("--integer-transforms", type=int, default=0, choices=(0, 1, 2),
                    help="run the workload with the fully-integer input and output transforms (1: one "
                         "scale per transform matrix, 2: per matrix row) instead of the fp32 ones")
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

    side = torch.cuda.Stream()

    def build_items(cfg, integer_mode=0):
        """One entry per convolution launched in a step (a layer with repeat=r gives r chained convs)."""
        items = []
        for li, lay in enumerate(workloads.CONFIGS[cfg]):
            d = workloads.make_layer_data(lay)
            kw = {}
            if d.u_B is not None:
                AT, BT, G = wq.scaled_transforms(lay.m, d.u_B, d.u_G)
                kw = dict(AT=AT, BT=BT, G=G)
            plan = wq.Plan(lay.N, lay.H, lay.W, lay.Cin, lay.Cout, lay.m, lay.group_size, **kw)
            if integer_mode:
                plan.set_integer_transforms(integer_mode)
            if args.k2_variant:
                # "name" = every layer, "i:name,j:name" = layers i, j of the set
                want = dict(v.split(":") for v in args.k2_variant.split(",")) if ":" in args.k2_variant \
                    else {str(li): args.k2_variant}
                if str(li) in want:
                    try:
                        plan.tune(0, want[str(li)])
                    except wq.WqError:
                        pass   # not applicable to this layer: the plan's own choice stays
            x = torch.from_numpy(d.x).cuda()
            w, b = torch.from_numpy(d.w).cuda(), torch.from_numpy(d.bias).cuda()
            for r in range(lay.repeat):
                # conv r of a stack reads conv r-1's output (Cin == Cout) and has its own weight blob
                it = dict(lay=lay, plan=plan, x=x, w=w, b=b, blob=plan.alloc_blob(),
                          ws=None, y=plan.alloc_output(), data=d, first=(r == 0))
                plan.weight_prepare(w, b, it["blob"])
                items.append(it)
                x = it["y"]
        # One workspace for all convolutions of the step, as large as the largest needs: they run one
        # after the other on one stream and a forward pass writes every workspace byte before it reads
        # it.  (Per-convolution workspaces measure 0.8 % slower: the dead intermediates of one layer
        # are overwritten in the caches by the next instead of being written back to memory.)
        ws_all = torch.empty(max(it["plan"].layout.ws_bytes for it in items), dtype=torch.uint8, device="cuda")
        for it in items:
            it["ws"] = ws_all[:it["plan"].layout.ws_bytes]
        torch.cuda.synchronize()
        return items

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

    def timed(run_once, calls, warmup_calls, repeats=REPEATS):
        """Median over `repeats` of (wall time of `calls` back-to-back calls) / calls, each repetition
        bracketed by synchronisations."""
        with torch.cuda.stream(side):
            for _ in range(warmup_calls):
                run_once()
            torch.cuda.synchronize()
            samples = []
            for _ in range(repeats):
                t0 = time.perf_counter()
                for _ in range(calls):
                    run_once()
                torch.cuda.synchronize()
                samples.append((time.perf_counter() - t0) / calls)
        return statistics.median(samples), samples

    def time_step(step, steps, warmup, eager_only=False):
        """The three launch modes of K steps; returns {mode: median seconds per step} and the spreads."""
        timings, spread = {}, {}

        def put(name, med_samples, per_call=1):
            med, samples = med_samples
            timings[name] = med / per_call
            spread[name] = [round(min(samples) / per_call * 1e3, 4), round(max(samples) / per_call * 1e3, 4)]

        if not eager_only:
            g_step = capture(step)
            put("one HIP graph replay per step", timed(g_step.replay, steps, warmup))
            group = 10 if steps % 10 == 0 else (5 if steps % 5 == 0 else 1)
            if group > 1:
                gN = capture(lambda: [step() for _ in range(group)])
                put(f"HIP graph of {group} steps, replayed steps/{group} times",
                    timed(gN.replay, steps // group, max(1, warmup // group)), group)
        put("eager launches from Python", timed(step, steps, warmup))
        return timings, spread

    items = build_items(args.config, args.integer_transforms)
    layers = workloads.CONFIGS[args.config]

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
                          "kernels": sorted({it["plan"].k2_variant_name for it in items})}))
        return

    timings, spread = time_step(step, args.steps, args.warmup, eager_only=args.eager)
    launch_mode = min(timings, key=timings.get)
    sec = timings[launch_mode]
    n_convs = len(items)
    direct_ops = sum(it['lay'].direct_ops for it in items)
    value = direct_ops / sec / 1e12

    g_off = capture(lambda: step(True))
    sec_off, _ = timed(g_off.replay, max(5, args.steps // 4), 2, repeats=5)
    footprint = sum(it["x"].numel() * 4 * it["first"] + it["blob"].numel()
                    + it["y"].numel() * 4 for it in items) + max(it["ws"].numel() for it in items)

    # ---- per-kernel durations, measured inside the real sequence: an instrumented step launches
    # every kernel of every convolution in order on the replay stream with a HIP event between
    # consecutive kernels.  A spacer (a few fills of a 1 GiB buffer) in front keeps the GPU busy
    # while the host enqueues the whole step, so that an interval holds its kernel (plus what
    # an event costs, measured on empty intervals of the same pass and subtracted) and no host
    # launch gap; it also leaves the caches as cold as they are when
    # the step is replayed back to back (a step moves 1.9 GB on the headline workload).  Median
    # of REPS instrumented steps.  The offline weight stage is timed on its own (back to back).
    REPS = 15
    spacer = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")

    def kernel_calls(it):
        plan = it["plan"]
        calls = [("k1", lambda: plan.input_transform(it["x"], it["ws"]))]
        if plan.layout.k2_kernels == 1:
            calls.append(("k2a", lambda: plan.contract_output(it["ws"], it["blob"], it["y"])))
        else:
            calls.append(("k2a", lambda: plan.contract_output_part(it["ws"], it["blob"], it["y"], 1)))
            calls.append(("k2b", lambda: plan.contract_output_part(it["ws"], it["blob"], it["y"], 2)))
        return calls

    event_cost = []

    def in_step_kernel_us():
        samples = [dict() for _ in items]
        with torch.cuda.stream(side):
            for rep in range(REPS + 2):
                for _ in range(4):
                    spacer.fill_(rep & 1)
                marks = []
                ev = torch.cuda.Event(enable_timing=True)
                ev.record(side)
                for i, it in enumerate(items):
                    for key, fn in kernel_calls(it):
                        fn()
                        nxt = torch.cuda.Event(enable_timing=True)
                        nxt.record(side)
                        marks.append((i, key, ev, nxt))
                        ev = nxt
                # what an event itself costs: intervals between records with nothing in between
                empty = []
                for _ in range(6):
                    nxt = torch.cuda.Event(enable_timing=True)
                    nxt.record(side)
                    empty.append((ev, nxt))
                    ev = nxt
                torch.cuda.synchronize()
                if rep >= 2:   # the first two passes warm up
                    cost = statistics.median(a.elapsed_time(b) * 1e3 for a, b in empty[1:])
                    event_cost.append(cost)
                    for i, key, a, b in marks:
                        samples[i].setdefault(key, []).append(max(0.0, a.elapsed_time(b) * 1e3 - cost))
        return [{k: statistics.median(v) for k, v in d.items()} for d in samples]

    def kernel_us(fn):
        g = capture(lambda: [fn() for _ in range(20)])
        out = []
        with torch.cuda.stream(side):
            g.replay()
            for _ in range(5):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(side)
                g.replay()
                e1.record(side)
                torch.cuda.synchronize()
                out.append(e0.elapsed_time(e1) * 1e3 / 20)
        return statistics.median(out)

    in_step = in_step_kernel_us()
    # identical convolutions of a stack (same plan, same shapes): the mean over the stack
    by_plan = {}
    for it, t in zip(items, in_step):
        by_plan.setdefault(id(it["plan"]), []).append(t)
    stack_mean = {pid: {k: sum(t[k] for t in ts) / len(ts) for k in ts[0]} for pid, ts in by_plan.items()}
    cache = {}

    def per_plan(it, key, fn):
        k = (id(it["plan"]), key)
        if k not in cache:
            cache[k] = kernel_us(fn)
        return cache[k]

    FIRST_KERNEL = {"fused": "k_contract_output", "gemm": "k_gemm_dequant", "lds_full": "k_wino_lds",
                    "lds_row": "k_wino_lds", "lds_tap": "k_wino_lds"}
    SECOND_KERNEL = {"gemm": "k_output_transform", "lds_row": "k_row_finish", "lds_tap": "k_output_transform"}

    per_layer, kernels = [], {}

    def account(name, us, nbytes):
        k = kernels.setdefault(name, dict(us=0.0, bytes=0, launches=0))
        k["us"] += us
        k["bytes"] += nbytes
        k["launches"] += 1

    for it in items:
        lay, plan = it["lay"], it["plan"]
        fam = plan.k2_variant_name.rsplit("_", 1)[0]
        t = stack_mean[id(plan)]
        k1, k2 = t["k1"], t["k2a"] + t.get("k2b", 0.0)
        k3 = per_plan(it, "k3", lambda: plan.weight_prepare(it["w"], it["b"], it["blob"]))
        ceil = k2_ceilings_us(lay)
        k1_ceiling = k1_bytes(lay) / (HBM_PEAK_GBS * 1e9) * 1e6
        k2_ceiling = max(ceil.values())
        row = dict(layer=lay.name, us=round(k1 + k2, 2), k1_us=round(k1, 2), k2_us=round(k2, 2),
                   direct_equiv_tops=round(lay.direct_ops / (k1 + k2) / 1e6, 1),
                   k2_variant=plan.k2_variant_name, k2_kernels=plan.layout.k2_kernels,
                   k1_hbm_frac=round(k1_ceiling / k1, 3),
                   k2_hbm_frac=round(ceil["hbm"] / k2, 3), k2_mfma_frac=round(ceil["mfma"] / k2, 4),
                   k2_valu_frac=round(ceil["valu"] / k2, 3),
                   # the layer against its binding ceilings: stage 1 by bytes, stages 2+3 by the largest of
                   # bytes, MFMA work and the dequantization's vector-ALU work
                   ceiling_us=round(k1_ceiling + k2_ceiling, 2),
                   ceiling_frac=round((k1_ceiling + k2_ceiling) / (k1 + k2), 3),
                   k2_bound=max(ceil, key=ceil.get),
                   k3_us=round(k3, 2), k3_hbm_frac=round(k3_bytes(lay) / (k3 * 1e-6) / 1e9 / HBM_PEAK_GBS, 3))
        account("k_input_transform", k1, k1_bytes(lay))
        if plan.layout.k2_kernels == 1:
            account(FIRST_KERNEL[fam], k2, k2_bytes(lay))
        else:
            a_us, b_us = t["k2a"], t["k2b"]
            # the fp32 intermediate (the n*n Winograd-domain products, or the n*m row sums of the row
            # form) is written by the first kernel and read back by the second
            per_elem = lay.n * lay.m if fam == "lds_row" else lay.n ** 2
            mid_bytes = 4 * per_elem * lay.tiles * lay.Cout
            y_bytes = 4 * lay.N * lay.H * lay.W * lay.Cout
            account(FIRST_KERNEL[fam], a_us, k2_bytes(lay) - y_bytes + mid_bytes)
            account(SECOND_KERNEL[fam], b_us, mid_bytes + y_bytes)
            row.update(k2_first_us=round(a_us, 2), k2_second_us=round(b_us, 2))
        per_layer.append(row)

    dom = max(kernels, key=lambda name: kernels[name]["us"])
    dk = kernels[dom]
    achieved = dk["bytes"] / (dk["us"] * 1e-6) / 1e9
    traffic, traffic_note = measured_traffic(dom, args.config)
    roofline = dict(bound="hbm", kernel=dom, achieved=round(achieved, 1), peak=HBM_PEAK_GBS,
                    unit="GB/s", frac=round(achieved / HBM_PEAK_GBS, 4),
                    traffic=traffic, traffic_source=traffic_note,
                    algorithmic_bytes_per_step=dk["bytes"],
                    avg_launch_us=round(dk["us"] / dk["launches"], 2),
                    launches_per_step=dk["launches"],
                    timing="HIP events between the kernels of an instrumented step on the replay stream "
                           "(median of %d steps, the cost of an event, %.1f us, subtracted)"
                           % (REPS, statistics.median(event_cost)),
                    note="every configured layer is bound by bytes when its kernels are priced one by one "
                         "(algorithmic bytes / HBM peak exceeds MFMA time and, except where 'k2_bound' says "
                         "otherwise, the dequantization's vector-ALU time); 'layers[].ceiling_frac' prices "
                         "each layer against the largest of the three",
                    kernels={name: dict(us_per_step=round(v["us"], 2), launches=v["launches"],
                                        algorithmic_bytes=v["bytes"],
                                        hbm_frac=round(v["bytes"] / (v["us"] * 1e-6) / 1e9 / HBM_PEAK_GBS, 4))
                             for name, v in kernels.items()})
    sum_ceiling = sum(r["ceiling_us"] for r in per_layer)
    ceiling = dict(step_ceiling_us=round(sum_ceiling, 1), step_us=round(sec * 1e6, 1),
                   frac=round(sum_ceiling / (sec * 1e6), 3))

    direct = linear = others = integer = None
    if not args.no_extras:
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

        d_timings, _ = time_step(direct_step, max(5, args.steps // 2), 2)
        sec_direct = min(d_timings.values())
        direct = dict(value=round(direct_ops / sec_direct / 1e12, 2), unit="TOPS",
                      ms_per_step=round(sec_direct * 1e3, 4),
                      winograd_over_direct=round(sec_direct / sec, 3),
                      note="the paper reports 31.3 % less runtime for the Winograd layers on an Arm CPU: "
                           "another machine and another layer mix")
        del d_items
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
        lp4 = wq.DirectPlan(lin_R, 1, 1, lin_C, lin_C, lin_g, linear=True, weight_bits=4)
        lblob4 = lp4.alloc_blob()
        lp4.weight_prepare(torch.randn(lin_C, lin_C, device="cuda") * 0.02, None, lblob4)
        lc4_us = kernel_us(lambda: lp4.conv(lws, lblob4, ly))
        linear = dict(shape=f"{lin_R}x{lin_C}->{lin_C}, g={lin_g}", quantize_us=round(lq_us, 2),
                      gemm_us=round(lc_us, 2),
                      int8_tops=round(2 * lin_R * lin_C * lin_C / ((lq_us + lc_us) * 1e-6) / 1e12, 1),
                      w4a8_gemm_us=round(lc4_us, 2),
                      w4a8_tops=round(2 * lin_R * lin_C * lin_C / ((lq_us + lc4_us) * 1e-6) / 1e12, 1))

        # ---- the other configurations as sub-blocks: whole-step time and TOPS, same launch choices
        others = {}
        if args.config == 5:
            for c in (1, 2, 3, 4):
                o_items = build_items(c)

                def o_step():
                    for it in o_items:
                        it["plan"].forward(it["x"], it["blob"], it["ws"], it["y"])

                o_t, _ = time_step(o_step, args.steps, args.warmup)
                o_sec = min(o_t.values())
                o_ops = sum(it["lay"].direct_ops for it in o_items)
                others[f"configs[{c - 1}]"] = dict(
                    convs_per_step=len(o_items), ms_per_step=round(o_sec * 1e3, 4),
                    us_per_layer=round(o_sec * 1e6 / len(o_items), 2), value=round(o_ops / o_sec / 1e12, 2),
                    unit="TOPS", launch=min(o_t, key=o_t.get),
                    k2_variants=[it["plan"].k2_variant_name for it in o_items])
                del o_items
                torch.cuda.empty_cache()

        # ---- the same workload with the fully-integer input and output transforms (the "next" path:
        # first and third quantized-stage equations), whole-step time
        if not args.integer_transforms:
            i_items = build_items(args.config, 1)

            def i_step():
                for it in i_items:
                    it["plan"].forward(it["x"], it["blob"], it["ws"], it["y"])

            i_t, _ = time_step(i_step, args.steps, args.warmup)
            i_sec = min(i_t.values())
            integer = dict(value=round(direct_ops / i_sec / 1e12, 2), unit="TOPS", ms_per_step=round(i_sec * 1e3, 4),
                           launch=min(i_t, key=i_t.get), scales="one per transform matrix",
                           k2_variants=sorted({it["plan"].k2_variant_name for it in i_items}),
                           integer_over_fp32_time=round(i_sec / sec, 3))
            del i_items
            torch.cuda.empty_cache()

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

        t0 = time.perf_counter()
        passes = 0
        while passes < 1 or (time.perf_counter() - t0 < 10 and passes < 50):
            cpu_pass()
            passes += 1
        cpu_sec = (time.perf_counter() - t0) / passes
        cpu_ops = sum(l.direct_ops for l in layers)
        cpu_baseline = dict(value=round(cpu_ops / cpu_sec / 1e12, 5), unit="TOPS",
                            cores=oracle.threads(), kind="oracle",
                            sample=f"{passes} forward pass(es) over one convolution per distinct layer shape "
                                   f"({len(prepared)} of the step's {n_convs} convolutions, the same work per "
                                   f"convolution), weights prepared beforehand, {cpu_sec:.2f} s per pass",
                            ms_per_pass=round(cpu_sec * 1e3, 1))

    out = dict(
        metric="direct-equivalent int8 TOPS of the group-wise quantized Winograd conv layer set "
               "(2*N*H*W*Cin*Cout*9 per layer / time); per-layer us in 'layers'",
        value=round(value, 2), unit="TOPS", n_gpus=1, steps=args.steps, warmup=args.warmup,
        ms_per_step=round(sec * 1e3, 4), us_per_layer=round(sec * 1e6 / n_convs, 2),
        launch=launch_mode, repeats=REPEATS, statistic="median of the repeats; value = fastest launch mode's median",
        ms_per_step_by_launch={k: round(v * 1e3, 4) for k, v in timings.items()},
        ms_per_step_min_max_by_launch=spread,
        higher_is_better=True, scaling="weak", vs_baseline=None, dtype="int8",
        data="synthetic",
        config=dict(workload=f"configs[{args.config - 1}]: " + "; ".join(
                        l.name + (f" x{l.repeat} chained" if l.repeat > 1 else "") for l in layers),
                    winograd=f"F({layers[0].m},3)", group_size=layers[0].group_size,
                    batch=layers[0].N, convs_per_step=n_convs,
                    resident_mb=round(footprint / 1e6, 1)),
        roofline=roofline, ceiling=ceiling, cpu_baseline=cpu_baseline, direct_conv_same_layers=direct,
        quantized_linear_layer=linear, other_configs=others, integer_transforms=integer,
        with_offline_stage=dict(value=round(direct_ops / sec_off / 1e12, 2), unit="TOPS",
                                ms_per_step=round(sec_off * 1e3, 4)),
        layers=per_layer)
    if args.k2_variant:
        out["config"]["k2_variant_forced"] = args.k2_variant
    if args.integer_transforms:
        out["config"]["integer_transforms"] = args.integer_transforms
    print(json.dumps(out))


if __name__ == "__main__":
    main()
