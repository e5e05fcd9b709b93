"""CPU oracle of the FULLY INTEGER group-wise quantized Winograd convolution.

TEST INFRASTRUCTURE ONLY.  Plain numpy, in the order of the three quantized-stage
equations of Section "Learnable Winograd transform scales":

    X~ = s_qB s_qB s_qx  Q(S_B V_B / s_qB) Q(x / s_qx) Q(V_B^T S_B / s_qB)        (input transform)
    Y~ = s_qW s_qX  Q(W / s_qW) Q(X~ / s_qX)   summed over the input channels      (Hadamard stage)
    y~ = s_qA s_qA s_qY  Q(V_A S_A / s_qA) Q(Y~ / s_qY) Q(S_A V_A^T / s_qA)        (output transform)

with Q the uniform symmetric 8-bit quantizer of Section "Related work" and min-max (abs-max)
scales taken dynamically for activations.  Where the text leaves the granularity of a scale open
the reading is the one under which the equation is an integer matrix product with the scales
outside it:

  s_qB, s_qA   ONE scale per transform matrix, abs-max / 127 (the equations write them as scalars
               that appear squared).  `matrix_scales="row"` is the alternative with one scale per
               matrix row (the output index of the product, the only other place a scale can sit
               outside the integer sum); it is offered for comparison, not as the reading.
  s_qx         one dynamic scale per (tile, group of g input channels): the abs-max of the
               group's n x n x g patch values (the groups of the rest of the method, and constant
               over the n x n patch as the integer product B^T d B needs).
  s_qX, s_qW   as in the built path: per (tap, tile, group) and per (tap, out-channel, group).
  s_qY         one dynamic scale per (tile, output channel): the abs-max of its n x n
               Winograd-domain values - the "single scale factor for the entire output tile" the
               section discusses (an 8 x 8 tile is one group of 64).
  rounding     round half to even; x / s evaluated as x * (127 / a) as everywhere in this oracle.
  precision    integer products exact (int64); scales and the de-quantized tensors in fp64,
               except that X~ is rounded once to fp32 before the Hadamard stage's quantizer, which
               is the fp32 quantizer of the built path (oracle.quantize_group).

The weight stage W = G w G^T stays in floating point and is quantized once, offline, exactly as
in the built path (the paper transforms the weights "with high precision").
"""
from __future__ import annotations

import numpy as np

from . import contract, weight_transform_quant, _load, _p, _f32  # noqa: F401  (the built path's stages)

QMAX = 127.0


def quantize_absmax(v: np.ndarray, axes) -> tuple:
    """Symmetric 8-bit quantizer with one abs-max scale over `axes` (kept as size-1 dims).
    Returns (codes int64, scale fp64); an all-zero group gets codes 0 and scale 0."""
    v = np.asarray(v, np.float64)
    a = np.abs(v).max(axis=axes, keepdims=True)
    safe = np.where(a > 0, a, 1.0)
    q = np.clip(np.rint(v * (QMAX / safe)), -QMAX, QMAX).astype(np.int64)
    q = np.where(a > 0, q, 0)
    return q, np.where(a > 0, a / QMAX, 0.0)


def quantize_matrix(Mx: np.ndarray, matrix_scales: str) -> tuple:
    """A transform matrix as int8 codes and its scale(s): one per matrix, or one per row."""
    Mx = np.asarray(Mx, np.float64)
    if matrix_scales == "matrix":
        q, s = quantize_absmax(Mx, (0, 1))
        return q, np.broadcast_to(s, (Mx.shape[0], 1)).copy()
    if matrix_scales == "row":
        return quantize_absmax(Mx, (1,))
    raise ValueError(matrix_scales)


def extract_tiles(x: np.ndarray, m: int) -> np.ndarray:
    """x [N][H][W][C] -> d [T][C][n][n]: the (m+2) x (m+2) input patches of the F(m,3) tiles
    (stride m, one pixel of zero padding, zeros beyond), tile id (b*TH + th)*TW + tw."""
    N, H, W, C = x.shape
    n = m + 2
    TH, TW = -(-H // m), -(-W // m)
    xp = np.zeros((N, TH * m + 2, TW * m + 2, C), x.dtype)
    xp[:, 1:H + 1, 1:W + 1] = x
    d = np.empty((N, TH, TW, C, n, n), x.dtype)
    for th in range(TH):
        for tw in range(TW):
            d[:, th, tw] = xp[:, th * m:th * m + n, tw * m:tw * m + n].transpose(0, 3, 1, 2)
    return d.reshape(N * TH * TW, C, n, n)


def input_transform_int(x, BT, m: int, g: int, matrix_scales: str = "matrix"):
    """First quantized-stage equation.  Returns dict(Xt [n*n][T][C] fp64 (the de-quantized X~),
    Qx, s_qx, QB, s_qB, Xint) - the integer pieces for the pins."""
    d = extract_tiles(np.asarray(x, np.float32), m).astype(np.float64)       # [T][C][n][n]
    T, C, n, _ = d.shape
    dg = d.reshape(T, C // g, g, n, n)
    Qx, s_qx = quantize_absmax(dg, (2, 3, 4))                                 # per (tile, group)
    Qx = Qx.reshape(T, C, n, n)
    QB, s_qB = quantize_matrix(BT, matrix_scales)                             # [n][n], [n][1]
    Xint = np.einsum("ik,tckl,jl->tcij", QB, Qx, QB)                          # exact in int64
    scale = (s_qB * s_qB.T)[None, None] * np.repeat(s_qx.reshape(T, C // g), g, axis=1)[:, :, None, None]
    Xt = (scale * Xint).transpose(2, 3, 0, 1).reshape(n * n, T, C)
    return dict(Xt=Xt, Qx=Qx, s_qx=s_qx.reshape(T, C // g), QB=QB, s_qB=s_qB[:, 0], Xint=Xint)


def quantize_along_channels(Xt32: np.ndarray, g: int):
    """The built path's activation quantizer: X [n*n][T][C] fp32 -> codes int8 and scales
    [n*n][T][C/g] fp32, one group per (tap, tile, g consecutive channels)."""
    n2, T, C = Xt32.shape
    Xq = np.empty((n2, T, C), np.int8)
    sX = np.empty((n2, T, C // g), np.float32)
    lib = _load()
    flat = np.ascontiguousarray(Xt32.reshape(-1, g))
    qf = np.empty_like(flat, dtype=np.int8)
    sf = sX.reshape(-1)
    for k in range(flat.shape[0]):
        sf[k] = lib.oracle_quantize_group(_p(flat[k]), g, _p(qf[k]))
    Xq[...] = qf.reshape(n2, T, C)
    return Xq, sX


def output_transform_int(Yt, AT, bias, N: int, H: int, W: int, m: int, matrix_scales: str = "matrix"):
    """Third quantized-stage equation on Y~ [n*n][T][Cout] (fp64).  Returns dict(y [N][H][W][Cout]
    fp64, QY, s_qY, QA, s_qA, yint)."""
    n = m + 2
    n2, T, Co = Yt.shape
    Y = np.asarray(Yt, np.float64).reshape(n, n, T, Co).transpose(2, 3, 0, 1)   # [T][Co][n][n]
    QY, s_qY = quantize_absmax(Y, (2, 3))                                        # per (tile, out-channel)
    QA, s_qA = quantize_matrix(AT, matrix_scales)                                # [m][n], [m][1]
    yint = np.einsum("ai,toij,bj->toab", QA, QY, QA)                             # exact in int64
    yt = (s_qA * s_qA.T)[None, None] * s_qY * yint                               # [T][Co][m][m]
    TH, TW = -(-H // m), -(-W // m)
    full = yt.reshape(N, TH, TW, Co, m, m).transpose(0, 1, 4, 2, 5, 3).reshape(N, TH * m, TW * m, Co)
    y = full[:, :H, :W].copy()
    if bias is not None:
        y += np.asarray(bias, np.float64)
    return dict(y=y, QY=QY, s_qY=s_qY[:, :, 0, 0], QA=QA, s_qA=s_qA[:, 0], yint=yint)


def fullint_pipeline(x, w, bias, AT, BT, G, m: int, g: int, matrix_scales: str = "matrix") -> dict:
    """The three equations in order.  x [N][H][W][Cin], w [Cout][Cin][3][3]; matrices as given
    (with any learned diagonal scales applied)."""
    x = np.asarray(x, np.float32)
    N, H, W, _ = x.shape
    st1 = input_transform_int(x, BT, m, g, matrix_scales)
    Xq, sX = quantize_along_channels(st1["Xt"].astype(np.float32), g)
    Wq, sW = weight_transform_quant(w, np.asarray(G, np.float32), m, g)
    Yt = contract(Xq, sX, Wq, sW, g)                                             # [n*n][T][Cout] fp64
    st3 = output_transform_int(Yt, AT, bias, N, H, W, m, matrix_scales)
    return dict(y=st3["y"], Yt=Yt, Xt=st1["Xt"], stage1=st1, stage3=st3, Xq=Xq, sX=sX, Wq=Wq, sW=sW)


def sqnr_db(ref: np.ndarray, got: np.ndarray) -> float:
    """10 log10(|ref|^2 / |ref - got|^2): the objective of the scale fine-tuning."""
    ref, got = np.asarray(ref, np.float64), np.asarray(got, np.float64)
    return float(10.0 * np.log10((ref ** 2).sum() / max(((ref - got) ** 2).sum(), 1e-300)))


def tap_relative_std(Yt: np.ndarray, m: int) -> np.ndarray:
    """The dynamic-range diagnostic of Figure "Dynamic ranges across different taps" (a): the
    standard deviation of the Winograd-domain output at each of the n x n locations, relative to
    the mean over the locations.  Yt [n*n][T][Cout]."""
    n = m + 2
    sd = np.asarray(Yt, np.float64).reshape(n * n, -1).std(axis=1).reshape(n, n)
    return sd / sd.mean()
