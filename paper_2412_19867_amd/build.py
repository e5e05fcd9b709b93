"""Builds libwq.so (the C-ABI library of hand-written gfx950 kernels) in-tree.

hipcc cross-compiles for gfx950 without a GPU.  Flags that matter:
  -ffp-contract=off   every fused multiply-add in the kernels is an explicit
                      fmaf; the compiler must not fuse a*b+c on its own (the
                      int8 codes are defined through one rounded product);
  -packed-fp32-ops    disabled: no v_pk_{add,mul,fma}_f32 is generated.
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(ROOT, "_build")
LIB = os.path.join(HERE, "libwq.so")
SOURCES = ["wq_host.cpp", "wq_transform.hip", "wq_contract.hip", "wq_contract_m2.hip",
           "wq_contract_m4.hip", "wq_contract_m6.hip", "wq_contract_lds.hip", "wq_contract_lds_m4.hip", "wq_contract_lds_m4_dump.hip",
           "wq_contract_lds_m6.hip", "wq_contract_lds_m6_dump.hip", "wq_gemm_unfused.hip",
           "wq_direct.hip", "wq_microbench.hip", "wq_static.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-ffp-contract=off",
         "-fvisibility=hidden",   # only the extern "C" entry points of include/wq.h are exported
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def build_library(verbose: bool = False, extra_flags=(), lib_out: str = LIB, build_dir: str = BUILD) -> str:
    os.makedirs(build_dir, exist_ok=True)
    procs = []
    objs = []
    for src in SOURCES:
        obj = os.path.join(build_dir, os.path.splitext(src)[0] + ".o")
        objs.append(obj)
        cmd = [HIPCC, "-x", "hip", *FLAGS, *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)))
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        text = out.decode(errors="replace")
        # hipcc's host pass does not know the gfx target feature; that warning is harmless
        text = "\n".join(l for l in text.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            failed = True
            print(f"--- {src} failed ---\n{text}", file=sys.stderr)
        elif verbose and text.strip():
            print(text)
    if failed:
        raise RuntimeError("hipcc failed")
    cmd = [HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", *objs, "-o", lib_out]
    subprocess.run(cmd, check=True)
    return lib_out


if __name__ == "__main__":
    print(build_library(verbose=True))
