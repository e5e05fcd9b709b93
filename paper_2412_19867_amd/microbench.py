#!/usr/bin/env python3
"""Matrix-core / vector-ALU co-issue ceiling of the group-wise dequantized int8 contraction.

Runs wq_microbench_dequant (no memory traffic) for every group size and 1, 2 and 4 waves per
SIMD and prints, per case, the time per 16x16 block and group and the share of the int8 MFMA
peak that rate corresponds to.  The dequantization is 12 vector instructions per block and
group whatever the group size; the MFMA work per group grows with it.

    python -m paper_2412_19867_amd.microbench            # table on stdout
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


def main():
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
