"""Data-free fine-tuning of the Winograd transform scales (the paper's algorithm box "Data-free
fully group-wise quantized Winograd transform by scales optimization").

One set of diagonal scales S_B, S_G per polynomial point, shared by all layers, is learned by
gradient descent so that the FULLY quantized Winograd convolution (int8 transform matrices, int8
input patches, int8 Winograd-domain operands and output tiles: the three quantized-stage
equations of Section "Learnable Winograd transform scales") reproduces the standard convolution
of the same layer on random Gaussian (or uniform) inputs; S_A = (S_B S_G)^-1 follows from
S_A S_B S_G = I.  The loss is the signal-to-quantization-noise ratio between the two outputs;
every iteration draws K layers and fresh noise, accumulates their gradients and takes one
optimizer step (stochastic gradient descent, as in the paper).

This module is the differentiable model of that pipeline in plain PyTorch (any device): each
quantizer is the uniform symmetric abs-max one with a straight-through gradient.  It shares no
code with the checker under oracle/; tests compare its forward pass with the checker's.
The learned scales are what wq_scaled_transforms / wq_plan_create take.
"""
from __future__ import annotations

from dataclasses import dataclass
from fractions import Fraction as Fr
from typing import List, Optional, Sequence

import torch
import torch.nn.functional as F

# Homogeneous polynomial points (f, g) and the standard diagonal scales of the supplementary
# Section "Standard Winograd transforms" (F(2,3): the same construction with 0, 1, -1, infinity).
POINTS = {
    2: [(0, 1), (1, 1), (-1, 1), (1, 0)],
    4: [(0, 1), (1, 1), (-1, 1), (2, 1), (-2, 1), (1, 0)],
    6: [(0, 1), (1, 1), (-1, 1), (2, 1), (-2, 1), (Fr(1, 2), 1), (Fr(-1, 2), 1), (1, 0)],
}
STANDARD_S_B = {2: [1, 2, 2, -1], 4: [4, -6, -6, 24, 24, 1],
                6: [1, Fr(-9, 2), Fr(-9, 2), 90, 90, Fr(45, 32), Fr(45, 32), 1]}
STANDARD_S_G = {2: [1, Fr(1, 2), Fr(1, 2), 1], 4: [Fr(1, 4), Fr(-1, 6), Fr(-1, 6), Fr(1, 24), Fr(1, 24), 1],
                6: [1, Fr(-2, 9), Fr(-2, 9), Fr(1, 90), Fr(1, 90), Fr(32, 45), Fr(32, 45), 1]}


def _vandermonde(points, b: int):
    """V[i][j] = f_i^j g_i^(b-1-j), exact rationals."""
    return [[(Fr(f) ** j if j else Fr(1)) * (Fr(g) ** (b - 1 - j) if b - 1 - j else Fr(1)) for j in range(b)]
            for f, g in points]


def _inverse(M):
    n = len(M)
    A = [[Fr(v) for v in row] + [Fr(int(i == j)) for j in range(n)] for i, row in enumerate(M)]
    for c in range(n):
        p = next(r for r in range(c, n) if A[r][c] != 0)
        A[c], A[p] = A[p], A[c]
        A[c] = [v / A[c][c] for v in A[c]]
        for r in range(n):
            if r != c and A[r][c] != 0:
                A[r] = [a - A[r][c] * b for a, b in zip(A[r], A[c])]
    return [row[n:] for row in A]


def vandermonde_factors(m: int, dtype=torch.float64):
    """(V_A [m][n], V_B [n][n], V_G [n][3]) with A^T = V_A S_A, B^T = S_B V_B, G = S_G V_G."""
    n, pts = m + 2, POINTS[m]
    Vnn = _vandermonde(pts, n)
    VB = _inverse([[Vnn[j][i] for j in range(n)] for i in range(n)])          # V_{n x n}^{-T}
    VG = _vandermonde(pts, 3)
    Vnm = _vandermonde(pts, m)
    VA = [[Vnm[j][i] for j in range(n)] for i in range(m)]                    # V_{n x m}^T
    t = lambda M: torch.tensor([[float(v) for v in row] for row in M], dtype=dtype)
    return t(VA), t(VB), t(VG)


def _ste_quant(v: torch.Tensor, dims, qmax: float = 127.0) -> torch.Tensor:
    """Uniform symmetric abs-max quantizer over `dims`, de-quantized, straight-through gradient."""
    a = v.detach().abs().amax(dim=dims, keepdim=True)
    s = torch.where(a > 0, a / qmax, torch.ones_like(a))
    q = torch.clamp(torch.round(v.detach() / s), -qmax, qmax) * s
    return v + (q - v.detach())


def _patches(x: torch.Tensor, m: int) -> torch.Tensor:
    """x [N][C][H][W] -> [N][TH][TW][C][n][n]: the (m+2)^2 input patches, stride m, zero pad 1."""
    N, C, H, W = x.shape
    n = m + 2
    TH, TW = -(-H // m), -(-W // m)
    xp = F.pad(x, (1, TW * m + 1 - W, 1, TH * m + 1 - H))
    return xp.unfold(2, n, m).unfold(3, n, m).permute(0, 2, 3, 1, 4, 5)


@dataclass
class WinogradScales:
    """log-magnitudes of S_B and S_G per point (the signs of the standard scales are kept)."""
    m: int
    log_sb: torch.Tensor
    log_sg: torch.Tensor
    sign_sb: torch.Tensor
    sign_sg: torch.Tensor

    @staticmethod
    def standard(m: int, device="cpu", dtype=torch.float64) -> "WinogradScales":
        sb = torch.tensor([float(v) for v in STANDARD_S_B[m]], dtype=dtype, device=device)
        sg = torch.tensor([float(v) for v in STANDARD_S_G[m]], dtype=dtype, device=device)
        return WinogradScales(m, sb.abs().log().requires_grad_(), sg.abs().log().requires_grad_(),
                              sb.sign(), sg.sign())

    def diagonals(self):
        S_B = self.sign_sb * self.log_sb.exp()
        S_G = self.sign_sg * self.log_sg.exp()
        return 1.0 / (S_B * S_G), S_B, S_G          # S_A S_B S_G = I by construction

    def matrices(self, factors):
        VA, VB, VG = factors
        S_A, S_B, S_G = self.diagonals()
        return VA * S_A[None, :], S_B[:, None] * VB, S_G[:, None] * VG       # A^T, B^T, G


def quantized_winograd_conv(x, w, scales: WinogradScales, factors, g: int, matrix_scales: str = "matrix"):
    """The fully quantized Winograd convolution of x [N][Cin][H][W] with w [Cout][Cin][3][3]
    (stride 1, zero pad 1), differentiable in the scales.  Returns [N][Cout][H][W]."""
    m = scales.m
    n = m + 2
    N, C, H, W = x.shape
    Co = w.shape[0]
    AT, BT, G = scales.matrices(factors)
    mdims = (0, 1) if matrix_scales == "matrix" else (1,)
    Bq, Aq = _ste_quant(BT, mdims), _ste_quant(AT, mdims)
    # weights: W = G w G^T in floating point, one scale per (tap, out-channel, group of Cin)
    Wt = torch.einsum("ik,ockl,jl->ocij", G, w, G)                                  # [Co][C][n][n]
    Wq = _ste_quant(Wt.reshape(Co, C // g, g, n, n), (2,)).reshape(Co, C, n, n)
    # first equation: int8 patches (one scale per (tile, group)), int8 B, integer product
    d = _patches(x, m)                                                              # [N][TH][TW][C][n][n]
    TH, TW = d.shape[1], d.shape[2]
    dq = _ste_quant(d.reshape(N, TH, TW, C // g, g, n, n), (4, 5, 6)).reshape(N, TH, TW, C, n, n)
    Xt = torch.einsum("ik,bhwckl,jl->bhwcij", Bq, dq, Bq)
    # second equation: X~ re-quantized per (tap, tile, group), contraction over the input channels
    Xq = _ste_quant(Xt.reshape(N, TH, TW, C // g, g, n, n), (4,)).reshape(N, TH, TW, C, n, n)
    Yt = torch.einsum("ocij,bhwcij->bhwoij", Wq, Xq)                                # [N][TH][TW][Co][n][n]
    # third equation: one scale per (tile, out-channel) output tile, int8 A, integer product
    Yq = _ste_quant(Yt, (4, 5))
    yt = torch.einsum("ai,bhwoij,cj->bhwoac", Aq, Yq, Aq)                           # [N][TH][TW][Co][m][m]
    y = yt.permute(0, 3, 1, 4, 2, 5).reshape(N, Co, TH * m, TW * m)
    return y[:, :, :H, :W]


def sqnr_db(ref: torch.Tensor, got: torch.Tensor) -> torch.Tensor:
    return 10.0 * torch.log10(ref.pow(2).sum() / (ref - got).pow(2).sum().clamp_min(1e-300))


def finetune_scales(layers: Sequence[torch.Tensor], m: int, g: int, epochs: int = 4, batches: int = 25,
                    K: int = 2, lr: float = 0.02, momentum: float = 0.9, noise: str = "gaussian",
                    batch: int = 2, size: int = 24, seed: int = 0, matrix_scales: str = "matrix",
                    log: Optional[List[float]] = None) -> WinogradScales:
    """The algorithm box: `layers` are the pre-trained weights [Cout][Cin][3][3] of the standard
    convolutions; returns the learned scales.  `log` collects the mean SQNR (dB) of each batch."""
    dev, dt = layers[0].device, layers[0].dtype
    gen = torch.Generator(device="cpu").manual_seed(seed)
    factors = tuple(f.to(dev, dt) for f in vandermonde_factors(m, dt))
    scales = WinogradScales.standard(m, dev, dt)
    ref_sb, ref_sg = scales.log_sb.detach().clone(), scales.log_sg.detach().clone()
    opt = torch.optim.SGD([scales.log_sb, scales.log_sg], lr=lr, momentum=momentum)
    for _ in range(epochs):
        for _ in range(batches):
            opt.zero_grad()
            picks = torch.randint(len(layers), (K,), generator=gen).tolist()
            total = 0.0
            for k in picks:
                w = layers[k]
                shape = (batch, w.shape[1], size, size)
                x = torch.randn(shape, generator=gen, dtype=dt) if noise == "gaussian" else \
                    torch.rand(shape, generator=gen, dtype=dt) * 2 - 1
                x = x.to(dev)
                y_ref = F.conv2d(x, w, padding=1)
                y_q = quantized_winograd_conv(x, w, scales, factors, g, matrix_scales)
                s = sqnr_db(y_ref, y_q)
                (-s / K).backward()
                total += float(s.detach())
            opt.step()
            # The pipeline does not depend on a common factor of S_B (or of S_G): the matrices'
            # own quantization scales absorb it.  Keep that free factor where the standard scales
            # have it, so that the magnitudes cannot drift.
            with torch.no_grad():
                scales.log_sb -= (scales.log_sb - ref_sb).mean()
                scales.log_sg -= (scales.log_sg - ref_sg).mean()
            if log is not None:
                log.append(total / K)
    return scales
