#!/usr/bin/env python3
"""Matrix-core / vector-ALU co-issue ceiling of the group-wise dequantized int8 contraction.

Runs wq_microbench_dequant (no memory traffic) for every group size and 1, 2 and 4 waves per
SIMD and prints, per case, the time per 16x16 block and group and the share of the int8 MFMA
peak that rate corresponds to.  The dequantization is 12 vector instructions per block and
group whatever the group size; the MFMA work per group grows with it.

    python -m paper_2412_19867_amd.microbench            # table on stdout

`--cache-probe` instead measures a property of the memory system that a chain of layers runs
into: how fast a kernel reads data it has never touched, depending on whether the last-level
(Infinity) cache holds dirty lines another kernel has just written, or clean ones.

    python -m paper_2412_19867_amd.microbench --cache-probe
"""
from __future__ import annotations

import json
import sys

INT8_PEAK_OPS = 5.0e15        # MI355X dense int8 MFMA, published
CUS, SIMDS = 256, 4


def run(iters: int = 20000):
    import torch
    from paper_2412_19867_amd import wq
    wq.lib()
    rows = []
    names = {0: "mfma_only", 1: "dequant_only", 2: "mfma_then_dequant", 3: "pipelined"}
    for g in (32, 64, 128, 256, 512):
        for nb in (2, 4):
            for wps in (1, 2, 4):
                for mode in (0, 1, 2, 3):
                    wgs = CUS * wps          # one workgroup = 4 waves = one wave per SIMD of a CU
                    wq.microbench_dequant(mode, g, nb, wgs, 200)       # warm-up
                    torch.cuda.synchronize()
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    cyc = wq.microbench_dequant(mode, g, nb, wgs, iters)
                    e1.record()
                    torch.cuda.synchronize()
                    sec = e0.elapsed_time(e1) * 1e-3
                    groups = iters * nb * wgs * 4                       # (block, group) pairs in total
                    macs = groups * 16 * 16 * g if mode != 1 else 0
                    rows.append(dict(group_size=g, blocks_per_wave=nb, waves_per_simd=wps, mode=names[mode],
                                     ns_per_block_group_per_simd=round(sec * 1e9 / (groups / (CUS * SIMDS)), 2),
                                     cycles_per_iter=round(float(cyc[:, 0].double().mean()) / iters, 1),
                                     counter_ghz=round(float(cyc[:, 0].double().sum() / cyc[:, 1].double().sum()) * 0.1, 3),
                                     mfma_peak_frac=round(2 * macs / sec / INT8_PEAK_OPS, 4)))
    return rows


def cache_probe():
    """A read-only stream (a library reduction over int64 words) over `mb` MB of cold data, timed with
    events, after (a) a 1 GiB buffer has just been filled (its lines sit dirty in the caches and are
    written back as the reader's lines displace them), (b) the same buffer has just been read twice
    (clean lines), (c) filled, then 300 MB of it read; and over the same data a second time."""
    import statistics
    import torch
    big = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    big64 = big.view(torch.int64)
    out = torch.zeros(2, dtype=torch.int64, device="cuda")

    def read(t, slot):
        torch.sum(t, dim=0, keepdim=True, out=out[slot:slot + 1])

    def med_us(prepare, data):
        ts = []
        for rep in range(12):
            prepare(rep)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            read(data, 1)
            e1.record()
            torch.cuda.synchronize()
            if rep >= 2:
                ts.append(e0.elapsed_time(e1) * 1e3)
        return statistics.median(ts)

    def dirty(rep):
        big.fill_(rep & 1)

    def clean(rep):
        big.fill_(rep & 1)
        read(big64, 0)
        read(big64, 0)

    def dirty_then_read(rep):
        big.fill_(rep & 1)
        read(big64[: (300 << 20) // 8], 0)

    for mb in (60, 240, 480):
        data = torch.ones(mb << 20, dtype=torch.uint8, device="cuda").view(torch.int64)
        for name, prep in (("1 GiB written just before (dirty lines)", dirty),
                           ("1 GiB read just before (clean lines)", clean),
                           ("1 GiB written, then 300 MB of it read", dirty_then_read),
                           ("the same data read just before", lambda rep: read(data, 1))):
            t = med_us(prep, data)
            print(f"{mb:4d} MB read after [{name:40s}]: {t:7.1f} us = {(mb << 20) / t / 1e6:5.2f} TB/s", flush=True)


def main():
    if "--cache-probe" in sys.argv:
        cache_probe()
        return
    rows = run()
    if "--json" in sys.argv:
        print(json.dumps(rows))
        return
    print(f"{'g':>4} {'blk/wave':>8} {'waves/SIMD':>10} {'mode':>18} {'ns/(block,group)/SIMD':>22} "
          f"{'ticks/iter':>12} {'tick GHz':>9} {'% of int8 MFMA peak':>20}")
    for r in rows:
        print(f"{r['group_size']:>4} {r['blocks_per_wave']:>8} {r['waves_per_simd']:>10} {r['mode']:>18} "
              f"{r['ns_per_block_group_per_simd']:>22} {r['cycles_per_iter']:>12} {r['counter_ghz']:>9} "
              f"{100 * r['mfma_peak_frac']:>19.1f}%")


if __name__ == "__main__":
    main()
