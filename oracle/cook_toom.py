"""Exact (rational) construction of the Winograd transform matrices.

TEST INFRASTRUCTURE ONLY - part of the CPU oracle; the HIP library carries its
own tables and never imports this.

Follows Section "Winograd convolution" (A^T = V_{n x m}^T S_A,
B^T = S_B V_{n x n}^{-T}, G = S_G V_{n x r}, with S_A S_B S_G = I) and the
supplementary Section "Standard Winograd transforms" (the Vandermonde matrix
V_{a x b}[i][j] = f_i^j g_i^{b-1-j} of the homogeneous points (f_i, g_i), and
the points / diagonal scales the paper adopts for F(4,3) and F(6,3)).
"""
from __future__ import annotations

from fractions import Fraction as Fr
from typing import List, Sequence, Tuple

import numpy as np

Matrix = List[List[Fr]]

# Points and diagonal scales printed in the supplementary section.
STANDARD = {
    4: dict(
        points=[(0, 1), (1, 1), (-1, 1), (2, 1), (-2, 1), (1, 0)],
        S_A=[1, 1, 1, 1, 1, 1],
        S_B=[4, -6, -6, 24, 24, 1],
        S_G=[Fr(1, 4), Fr(-1, 6), Fr(-1, 6), Fr(1, 24), Fr(1, 24), 1],
    ),
    6: dict(
        points=[(0, 1), (1, 1), (-1, 1), (2, 1), (-2, 1), (Fr(1, 2), 1), (Fr(-1, 2), 1), (1, 0)],
        S_A=[1, 1, 1, 1, 1, 1, 1, 1],
        S_B=[1, Fr(-9, 2), Fr(-9, 2), 90, 90, Fr(45, 32), Fr(45, 32), 1],
        S_G=[1, Fr(-2, 9), Fr(-2, 9), Fr(1, 90), Fr(1, 90), Fr(32, 45), Fr(32, 45), 1],
    ),
    # F(2,3) is not printed in the paper; the same construction with the first
    # three finite points plus infinity and unit-free scales chosen so that the
    # matrices are the familiar small-integer ones.
    2: dict(
        points=[(0, 1), (1, 1), (-1, 1), (1, 0)],
        S_A=[1, 1, 1, -1],
        S_B=[1, 2, 2, -1],
        S_G=[1, Fr(1, 2), Fr(1, 2), 1],
    ),
}


def _pow(x: Fr, k: int) -> Fr:
    return Fr(1) if k == 0 else Fr(x) ** k


def vandermonde(points: Sequence[Tuple], b: int) -> Matrix:
    """V_{a x b} with V[i][j] = f_i^j * g_i^(b-1-j)."""
    return [[_pow(Fr(f), j) * _pow(Fr(g), b - 1 - j) for j in range(b)] for f, g in points]


def inverse(Mx: Matrix) -> Matrix:
    n = len(Mx)
    A = [[Fr(v) for v in row] + [Fr(int(i == j)) for j in range(n)] for i, row in enumerate(Mx)]
    for col in range(n):
        piv = next(r for r in range(col, n) if A[r][col] != 0)
        A[col], A[piv] = A[piv], A[col]
        p = A[col][col]
        A[col] = [v / p for v in A[col]]
        for r in range(n):
            if r != col and A[r][col] != 0:
                f = A[r][col]
                A[r] = [a - f * c for a, c in zip(A[r], A[col])]
    return [row[n:] for row in A]


def transpose(Mx: Matrix) -> Matrix:
    return [list(r) for r in zip(*Mx)]


def cook_toom(points, S_A, S_B, S_G, m: int, r: int = 3):
    """Return (A^T [m x n], B^T [n x n], G [n x r]) as exact fractions."""
    n = m + r - 1
    assert len(points) == n
    V_nm = vandermonde(points, m)
    V_nn = vandermonde(points, n)
    V_nr = vandermonde(points, r)
    AT = [[V_nm[i][a] * Fr(S_A[i]) for i in range(n)] for a in range(m)]      # V^T S_A
    VinvT = transpose(inverse(V_nn))
    BT = [[Fr(S_B[i]) * VinvT[i][k] for k in range(n)] for i in range(n)]      # S_B V^{-T}
    G = [[Fr(S_G[i]) * V_nr[i][k] for k in range(r)] for i in range(n)]        # S_G V
    return AT, BT, G


def identity_defect(AT: Matrix, BT: Matrix, G: Matrix) -> Fr:
    """max |sum_i AT[a][i] G[i][k] BT[i][l] - [l == a+k]|: zero iff the three
    matrices compute the 1-D correlation y[a] = sum_k d[a+k] g[k] exactly."""
    m, n, r = len(AT), len(BT), len(G[0])
    worst = Fr(0)
    for a in range(m):
        for k in range(r):
            for l in range(n):
                s = sum(AT[a][i] * G[i][k] * BT[i][l] for i in range(n))
                worst = max(worst, abs(s - (1 if l == a + k else 0)))
    return worst


def standard_fractions(m: int):
    st = STANDARD[m]
    return cook_toom(st["points"], st["S_A"], st["S_B"], st["S_G"], m)


def to_f64(Mx: Matrix) -> np.ndarray:
    return np.array([[float(v) for v in row] for row in Mx], dtype=np.float64)


def standard_matrices(m: int):
    """(A^T, B^T, G) as float64 arrays."""
    return tuple(to_f64(M) for M in standard_fractions(m))


def scaled_matrices(m: int, u_B, u_G):
    """Matrices with the diagonal scales replaced by u_B*S_B, u_G*S_G and
    S_A = (S_B S_G)^{-1} (the learnable-scale parametrisation); exact
    rationals of the given float scales, then rounded to float64."""
    st = STANDARD[m]
    S_B = [Fr(float(u)) * Fr(s) for u, s in zip(u_B, st["S_B"])]
    S_G = [Fr(float(u)) * Fr(s) for u, s in zip(u_G, st["S_G"])]
    S_A = [1 / (b * g) for b, g in zip(S_B, S_G)]
    return tuple(to_f64(M) for M in cook_toom(st["points"], S_A, S_B, S_G, m))


def matrices_from_scales(m: int, S_B, S_G):
    """Matrices from explicit diagonal S_B, S_G (e.g. the learned values the
    paper tabulates), with S_A = (S_B S_G)^{-1}."""
    st = STANDARD[m]
    S_B = [Fr(float(v)) for v in S_B]
    S_G = [Fr(float(v)) for v in S_G]
    S_A = [1 / (b * g) for b, g in zip(S_B, S_G)]
    return tuple(to_f64(M) for M in cook_toom(st["points"], S_A, S_B, S_G, m))
