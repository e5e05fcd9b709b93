"""CPU oracle for the group-wise int8 quantized Winograd convolution.

TEST INFRASTRUCTURE ONLY.  Imported by tests/, by the smoke check and by the
benchmark's host-baseline leg; never by the product path.  The arithmetic
lives in qwino_oracle.c (plain C loops) and cook_toom.py (exact rationals);
this file only builds the C file with gcc and marshals numpy arrays to it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

from . import cook_toom  # noqa: F401  (re-exported)

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "qwino_oracle.c")
_LIB = os.path.join(_HERE, "libqwino_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  -ffp-contract=off: every fused
    multiply-add in the fp32 chains is an explicit fmaf()."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared",
               _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_quantize_group.restype = ctypes.c_float
    return _lib


def threads() -> int:
    """Threads the OpenMP loops use (for the benchmark's core count)."""
    n = os.environ.get("OMP_NUM_THREADS")
    return int(n) if n else (os.cpu_count() or 1)


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def direct_conv(x, w, bias=None) -> np.ndarray:
    """3x3 stride-1 zero-pad-1 cross-correlation, fp64 accumulate.  x NHWC, w OIHW."""
    x, w = _f32(x), _f32(w)
    N, H, W, Cin = x.shape
    Cout = w.shape[0]
    assert w.shape == (Cout, Cin, 3, 3)
    b = None if bias is None else _f32(bias)
    y = np.empty((N, H, W, Cout), dtype=np.float64)
    _load().oracle_direct_conv_f64(_p(x), _p(w), _p(b), _p(y), N, H, W, Cin, Cout)
    return y


def winograd_f64(x, w, bias, AT, BT, G, m: int) -> np.ndarray:
    """Un-quantized Winograd convolution in fp64 with the given matrices."""
    x, w = _f32(x), _f32(w)
    N, H, W, Cin = x.shape
    Cout = w.shape[0]
    n = m + 2
    AT, BT, G = _f64(AT), _f64(BT), _f64(G)
    assert AT.shape == (m, n) and BT.shape == (n, n) and G.shape == (n, 3)
    b = None if bias is None else _f32(bias)
    y = np.empty((N, H, W, Cout), dtype=np.float64)
    _load().oracle_winograd_f64(_p(x), _p(w), _p(b), _p(BT), _p(G), _p(AT), _p(y),
                                N, H, W, Cin, Cout, m)
    return y


def quantize_group(v):
    v = _f32(v).ravel()
    q = np.empty(v.size, dtype=np.int8)
    s = _load().oracle_quantize_group(_p(v), int(v.size), _p(q))
    return q, np.float32(s)


def quantize_group_literal(v):
    """The quantizer equation with a division per element (see the C function): for measuring the
    distance of the library's reading from the text, nothing else."""
    v = _f32(v).ravel()
    q = np.empty(v.size, dtype=np.int8)
    L = _load()
    L.oracle_quantize_group_literal.restype = ctypes.c_float
    s = L.oracle_quantize_group_literal(_p(v), int(v.size), _p(q))
    return q, np.float32(s)


def weight_transform_quant(w, G, m: int, g: int, want_float: bool = False):
    w, G = _f32(w), _f32(G)
    Cout, Cin = w.shape[:2]
    n2 = (m + 2) ** 2
    assert Cin % g == 0 and G.shape == (m + 2, 3)
    Wq = np.empty((n2, Cout, Cin), dtype=np.int8)
    sW = np.empty((n2, Cin // g, Cout), dtype=np.float32)
    Wf = np.empty((n2, Cout, Cin), dtype=np.float32) if want_float else None
    _load().oracle_weight_transform_quant(_p(w), _p(G), Cin, Cout, m, g, _p(Wq), _p(sW), _p(Wf))
    return (Wq, sW, Wf) if want_float else (Wq, sW)


def input_transform_quant(x, BT, m: int, g: int, want_float: bool = False):
    x, BT = _f32(x), _f32(BT)
    N, H, W, Cin = x.shape
    n = m + 2
    T = N * (-(-H // m)) * (-(-W // m))
    assert Cin % g == 0 and BT.shape == (n, n)
    Xq = np.empty((n * n, T, Cin), dtype=np.int8)
    sX = np.empty((n * n, T, Cin // g), dtype=np.float32)
    Xf = np.empty((n * n, T, Cin), dtype=np.float32) if want_float else None
    _load().oracle_input_transform_quant(_p(x), _p(BT), N, H, W, Cin, m, g, _p(Xq), _p(sX), _p(Xf))
    return (Xq, sX, Xf) if want_float else (Xq, sX)


def contract(Xq, sX, Wq, sW, g: int, want_P: bool = False):
    n2, T, Cin = Xq.shape
    Cout = Wq.shape[1]
    assert Wq.shape == (n2, Cout, Cin) and sX.shape == (n2, T, Cin // g)
    assert sW.shape == (n2, Cin // g, Cout)
    Xq, Wq = np.ascontiguousarray(Xq, np.int8), np.ascontiguousarray(Wq, np.int8)
    sX, sW = _f32(sX), _f32(sW)
    P = np.empty((n2, T, Cin // g, Cout), dtype=np.int32) if want_P else None
    M = np.empty((n2, T, Cout), dtype=np.float64)
    _load().oracle_contract(_p(Xq), _p(sX), _p(Wq), _p(sW), ctypes.c_long(T), Cin, Cout, n2, g,
                            _p(P), _p(M))
    return (M, P) if want_P else M


def contract_bruteforce(Xq, Wq, g: int) -> np.ndarray:
    n2, T, Cin = Xq.shape
    Cout = Wq.shape[1]
    Xq, Wq = np.ascontiguousarray(Xq, np.int8), np.ascontiguousarray(Wq, np.int8)
    P2 = np.empty((n2, T, Cin // g, Cout), dtype=np.int64)
    _load().oracle_contract_bruteforce(_p(Xq), _p(Wq), ctypes.c_long(T), Cin, Cout, n2, g, _p(P2))
    return P2


def output_transform(M, AT, bias, N: int, H: int, W: int, m: int):
    """Returns (y64, y32)."""
    M, AT = _f64(M), _f32(AT)
    Cout = M.shape[2]
    b = None if bias is None else _f32(bias)
    y64 = np.zeros((N, H, W, Cout), dtype=np.float64)
    y32 = np.zeros((N, H, W, Cout), dtype=np.float32)
    _load().oracle_output_transform(_p(M), _p(AT), _p(b), N, H, W, Cout, m, _p(y64), _p(y32))
    return y64, y32


def qwino_pipeline(x, w, bias, AT, BT, G, m: int, g: int, want_P: bool = False) -> dict:
    """The whole quantized path: offline weight stage, input stage, contraction,
    output stage.  Matrices are taken as fp32 (what the library is handed)."""
    x = _f32(x)
    N, H, W, _ = x.shape
    AT, BT, G = _f32(AT), _f32(BT), _f32(G)
    Wq, sW = weight_transform_quant(w, G, m, g)
    Xq, sX = input_transform_quant(x, BT, m, g)
    res = contract(Xq, sX, Wq, sW, g, want_P=want_P)
    M, P = res if want_P else (res, None)
    y64, y32 = output_transform(M, AT, bias, N, H, W, m)
    return dict(Xq=Xq, sX=sX, Wq=Wq, sW=sW, P=P, M=M, y64=y64, y=y32)


# ---- the group-wise quantized standard (direct) convolution: the paper's runtime comparison point
def quantize_pixels(x, g: int):
    """x [N][H][W][Cin] fp32 -> (xq [N*H*W][Cin] int8, sx [N*H*W][Cin/g] fp32)."""
    x = _f32(x)
    Cin = x.shape[-1]
    P = x.size // Cin
    xq = np.empty((P, Cin), dtype=np.int8)
    sx = np.empty((P, Cin // g), dtype=np.float32)
    _load().oracle_quantize_pixels(_p(x), ctypes.c_long(P), Cin, g, _p(xq), _p(sx))
    return xq, sx


def quantize_filters(w, g: int, bits: int = 8):
    """w [Cout][Cin][3][3] fp32 -> (wq [9][Cout][Cin] int8, sw [9][Cin/g][Cout] fp32);
    bits = 4 gives codes in [-7, 7] (W4A8)."""
    assert bits in (4, 8)
    w = _f32(w)
    Cout, Cin = w.shape[:2]
    wq = np.empty((9, Cout, Cin), dtype=np.int8)
    sw = np.empty((9, Cin // g, Cout), dtype=np.float32)
    _load().oracle_quantize_filters_bits(_p(w), Cin, Cout, g, bits, _p(wq), _p(sw))
    return wq, sw


def direct_qconv(xq, sx, wq, sw, bias, N: int, H: int, W: int, g: int):
    """Returns (y64, y32), both [N][H][W][Cout]."""
    xq, wq = np.ascontiguousarray(xq, np.int8), np.ascontiguousarray(wq, np.int8)
    sx, sw = _f32(sx), _f32(sw)
    Cin, Cout = xq.shape[1], wq.shape[1]
    assert xq.shape[0] == N * H * W and wq.shape == (9, Cout, Cin)
    b = None if bias is None else _f32(bias)
    y64 = np.empty((N, H, W, Cout), dtype=np.float64)
    y32 = np.empty((N, H, W, Cout), dtype=np.float32)
    _load().oracle_direct_qconv(_p(xq), _p(sx), _p(wq), _p(sw), _p(b), N, H, W, Cin, Cout, g,
                                _p(y64), _p(y32))
    return y64, y32


def direct_pipeline(x, w, bias, g: int, weight_bits: int = 8) -> dict:
    """The whole group-wise quantized standard convolution."""
    x = _f32(x)
    N, H, W, _ = x.shape
    xq, sx = quantize_pixels(x, g)
    wq, sw = quantize_filters(w, g, weight_bits)
    y64, y32 = direct_qconv(xq, sx, wq, sw, bias, N, H, W, g)
    return dict(xq=xq, sx=sx, wq=wq, sw=sw, y64=y64, y=y32)


# ---- group-wise quantized linear layer (the 1-tap case of the same quantized GEMM)
def quantize_weight_rows(w, g: int, bits: int = 8):
    """w [Cout][Cin] fp32 -> (wq [Cout][Cin] int8, sw [Cin/g][Cout] fp32);
    bits = 4 gives codes in [-7, 7] (W4A8)."""
    assert bits in (4, 8)
    w = _f32(w)
    Cout, Cin = w.shape
    wq = np.empty((Cout, Cin), dtype=np.int8)
    sw = np.empty((Cin // g, Cout), dtype=np.float32)
    _load().oracle_quantize_weight_rows_bits(_p(w), Cin, Cout, g, bits, _p(wq), _p(sw))
    return wq, sw


def quantize_group_bits(v, bits: int):
    """One group through the `bits`-wide quantizer -> (codes int8, scale)."""
    v = _f32(v).ravel()
    q = np.empty(v.size, dtype=np.int8)
    L = _load()
    L.oracle_quantize_group_bits.restype = ctypes.c_float
    s = L.oracle_quantize_group_bits(_p(v), v.size, bits, _p(q))
    return q, np.float32(s)


def linear_pipeline(x, w, bias, g: int, weight_bits: int = 8) -> dict:
    """x [R][Cin], w [Cout][Cin]: quantize both group-wise, multiply, rescale per group."""
    x, w = _f32(x), _f32(w)
    R, Cin = x.shape
    Cout = w.shape[0]
    xq, sx = quantize_pixels(x, g)
    wq, sw = quantize_weight_rows(w, g, weight_bits)
    b = None if bias is None else _f32(bias)
    y64 = np.empty((R, Cout), dtype=np.float64)
    y32 = np.empty((R, Cout), dtype=np.float32)
    _load().oracle_linear_q(_p(xq), _p(sx), _p(wq), _p(sw), _p(b), ctypes.c_long(R), Cin, Cout, g,
                            _p(y64), _p(y32))
    return dict(xq=xq, sx=sx, wq=wq, sw=sw, y64=y64, y=y32)
