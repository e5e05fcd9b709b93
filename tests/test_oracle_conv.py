"""Pins for the oracle's un-quantized convolutions (CPU only).

direct_conv is pinned to a library routine (torch conv2d in fp64) and to
closed forms; the fp64 Winograd path is pinned to direct_conv through the
minimal-filtering identity (exact up to fp64 rounding), including ragged
tile grids, and through the invariance under S_A S_B S_G = I.
"""
import numpy as np
import pytest
import torch

import oracle
from oracle import cook_toom as ct
from conftest import golden_path


def rand_layer(seed, N, H, W, Cin, Cout):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((N, H, W, Cin)).astype(np.float32)
    w = rng.standard_normal((Cout, Cin, 3, 3)).astype(np.float32)
    b = rng.standard_normal(Cout).astype(np.float32)
    return x, w, b


def test_direct_conv_matches_library_cross_correlation():
    x, w, b = rand_layer(1, 2, 7, 9, 5, 4)
    y = oracle.direct_conv(x, w, b)
    ref = torch.nn.functional.conv2d(
        torch.from_numpy(x).double().permute(0, 3, 1, 2), torch.from_numpy(w).double(),
        torch.from_numpy(b).double(), stride=1, padding=1).permute(0, 2, 3, 1).numpy()
    np.testing.assert_allclose(y, ref, rtol=1e-12, atol=1e-12)


def test_direct_conv_closed_forms():
    x, _, _ = rand_layer(2, 1, 6, 5, 3, 3)
    # centre tap = channel identity -> output equals input
    w = np.zeros((3, 3, 3, 3), np.float32)
    for c in range(3):
        w[c, c, 1, 1] = 1.0
    np.testing.assert_array_equal(oracle.direct_conv(x, w), x.astype(np.float64))
    # tap (u=0, v=2) reads the pixel one row up, one column right, zero outside
    w = np.zeros((3, 3, 3, 3), np.float32)
    for c in range(3):
        w[c, c, 0, 2] = 1.0
    y = oracle.direct_conv(x, w)
    ref = np.zeros_like(y)
    ref[:, 1:, :-1, :] = x[:, :-1, 1:, :]
    np.testing.assert_array_equal(y, ref)
    # bias only
    y = oracle.direct_conv(x, np.zeros((2, 3, 3, 3), np.float32), np.array([0.5, -2.0], np.float32))
    assert np.all(y[..., 0] == 0.5) and np.all(y[..., 1] == -2.0)


@pytest.mark.parametrize("m", [2, 4, 6])
@pytest.mark.parametrize("shape", [(1, 8, 8, 3, 2), (2, 7, 9, 4, 5), (1, 13, 5, 2, 3), (1, 1, 1, 1, 1)])
def test_winograd_identity_equals_direct(m, shape):
    x, w, b = rand_layer(10 * m + shape[1], *shape)
    AT, BT, G = ct.standard_matrices(m)
    yw = oracle.winograd_f64(x, w, b, AT, BT, G, m)
    yd = oracle.direct_conv(x, w, b)
    scale = np.abs(yd).max()
    assert np.abs(yw - yd).max() <= 1e-10 * scale


@pytest.mark.parametrize("m", [4, 6])
def test_invariance_under_diagonal_scales(m):
    x, w, b = rand_layer(99 + m, 1, 11, 10, 6, 4)
    rng = np.random.default_rng(5)
    u_B, u_G = rng.uniform(0.5, 2, m + 2), rng.uniform(0.5, 2, m + 2)
    AT, BT, G = ct.scaled_matrices(m, u_B, u_G)
    yd = oracle.direct_conv(x, w, b)
    yw = oracle.winograd_f64(x, w, b, AT, BT, G, m)
    assert np.abs(yw - yd).max() <= 1e-10 * np.abs(yd).max()


def test_invariance_with_the_papers_learned_scales():
    rows = [[float(t) for t in l.split()] for l in open(golden_path("learned_scales_f63.txt"))
            if l.strip() and not l.startswith("#")]
    _, S_B, S_G = (np.array(c) for c in zip(*rows))
    AT, BT, G = ct.matrices_from_scales(6, S_B, S_G)
    x, w, b = rand_layer(123, 1, 12, 12, 4, 4)
    yd = oracle.direct_conv(x, w, b)
    yw = oracle.winograd_f64(x, w, b, AT, BT, G, 6)
    assert np.abs(yw - yd).max() <= 1e-10 * np.abs(yd).max()


def test_winograd_with_a_broken_matrix_is_caught():
    # sensitivity of the pin: a swapped pair in B^T must break the identity
    x, w, b = rand_layer(3, 1, 8, 8, 2, 2)
    AT, BT, G = ct.standard_matrices(4)
    BT = BT.copy()
    BT[[1, 2]] = BT[[2, 1]]
    yd = oracle.direct_conv(x, w, b)
    yw = oracle.winograd_f64(x, w, b, AT, BT, G, 4)
    assert np.abs(yw - yd).max() > 1e-3 * np.abs(yd).max()
