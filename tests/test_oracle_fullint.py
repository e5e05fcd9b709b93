"""Pins of the fully-integer oracle (oracle/fullint.py): the three quantized-stage equations of
Section "Learnable Winograd transform scales" with int8 transform matrices, int8 input patches
and int8 Winograd-domain output tiles.

What fixes it other than itself: exact integer arithmetic in special cases where every quantizer
is lossless (checked against numpy's int64 einsum on independently extracted patches), the patch
extraction against the built path's input stage run with an identity "transform", covariance
under power-of-two rescaling, the quantizer's half-step bound per stage, and the one quantitative
fact the paper fixes for this pipeline: with the learned F(6,3) scales it tabulates the result is
far better than with the standard scales, and the per-tap dynamic range of the Winograd-domain
output flattens (its Figure on dynamic ranges, panels (a) and (c)).
"""
import numpy as np
import pytest

import oracle
from oracle import cook_toom as ct
from oracle import fullint

from conftest import golden_path


def _learned_f63():
    rows = [[float(t) for t in l.split()] for l in open(golden_path("learned_scales_f63.txt"))
            if not l.startswith("#")]
    return ct.matrices_from_scales(6, [r[1] for r in rows], [r[2] for r in rows])


def _patches_by_hand(x, m):
    """Independent extraction: one np.pad and explicit python loops over tiles."""
    N, H, W, C = x.shape
    n = m + 2
    TH, TW = -(-H // m), -(-W // m)
    xp = np.pad(x, ((0, 0), (1, TH * m + 1 - H), (1, TW * m + 1 - W), (0, 0)))
    out = []
    for b in range(N):
        for th in range(TH):
            for tw in range(TW):
                out.append(np.moveaxis(xp[b, th * m:th * m + n, tw * m:tw * m + n, :], 2, 0))
    return np.stack(out)          # [T][C][n][n]


@pytest.mark.parametrize("m", [2, 4, 6])
def test_patch_extraction_matches_the_built_input_stage_with_an_identity_transform(m):
    rng = np.random.default_rng(m)
    x = rng.standard_normal((2, 3 * m + 1, 2 * m + 3, 32)).astype(np.float32)
    n = m + 2
    _, _, Xf = oracle.input_transform_quant(x, np.eye(n, dtype=np.float32), m, 32, want_float=True)
    d = fullint.extract_tiles(x, m)
    assert np.array_equal(Xf.reshape(n, n, d.shape[0], 32).transpose(2, 3, 0, 1), d)
    assert np.array_equal(_patches_by_hand(x, m), d)


def test_f23_matrices_are_exact_in_int8_and_the_f43_f63_ones_are_not():
    AT, BT, G = ct.standard_matrices(2)
    for Mx in (AT, BT):
        q, s = fullint.quantize_matrix(Mx, "matrix")
        assert np.array_equal(q * s, Mx) and np.abs(q).max() == 127
    for m in (4, 6):
        AT, BT, G = ct.standard_matrices(m)
        q, s = fullint.quantize_matrix(BT, "matrix")
        assert np.abs(q * s - BT).max() > 1e-3          # 4 / (5/127) = 101.6 is not an integer
        assert np.abs(q * s - BT).max() <= s.max() / 2 + 1e-12


def test_lossless_input_transform_is_the_exact_integer_product():
    """F(2,3) (matrices exact in int8), integer pixels with abs-max 127 in every (tile, group)
    patch: every quantizer of the first equation is lossless, so X~ must equal B^T d B computed
    exactly in integers."""
    rng = np.random.default_rng(5)
    m, g = 2, 32
    x = rng.integers(-127, 128, size=(2, 6, 8, 64)).astype(np.float32)
    d = _patches_by_hand(x, m)
    T, C = d.shape[:2]
    assert (np.abs(d).reshape(T, C // g, -1).max(axis=2) == 127).all()
    AT, BT, G = ct.standard_matrices(m)
    st = fullint.input_transform_int(x, BT, m, g)
    assert np.array_equal(st["Qx"], d.astype(np.int64)) and np.allclose(st["s_qx"], 1.0)
    want = np.einsum("ik,tckl,jl->tcij", BT.astype(np.int64), d.astype(np.int64), BT.astype(np.int64))
    got = st["Xt"].reshape(m + 2, m + 2, T, C).transpose(2, 3, 0, 1)
    np.testing.assert_allclose(got, want, rtol=1e-13, atol=0)       # s_qB^2 * 127^2 = 1 up to two roundings
    assert np.array_equal(np.rint(got), want)
    # a transposed right factor or a swapped index must show up: the product is not symmetric
    assert not np.array_equal(want, want.transpose(0, 1, 3, 2))


def test_lossless_output_transform_is_the_exact_integer_product():
    rng = np.random.default_rng(6)
    m, n = 2, 4
    N, H, W, Co = 1, 4, 6, 8
    T = N * 2 * 3
    Y = rng.integers(-127, 128, size=(n * n, T, Co)).astype(np.float64)
    Y[0] = 127                                   # every (tile, channel) tile reaches the abs-max
    AT, BT, G = ct.standard_matrices(m)
    st = fullint.output_transform_int(Y, AT, None, N, H, W, m)
    Yt = Y.reshape(n, n, T, Co).transpose(2, 3, 0, 1).astype(np.int64)
    assert np.array_equal(st["QY"], Yt) and np.allclose(st["s_qY"], 1.0)
    want = np.einsum("ai,toij,bj->toab", AT.astype(np.int64), Yt, AT.astype(np.int64))
    got = st["y"].reshape(N, 2, m, 3, m, Co).transpose(0, 1, 3, 5, 2, 4).reshape(T, Co, m, m)
    assert np.array_equal(np.rint(got), want)
    np.testing.assert_allclose(got, want, rtol=1e-13, atol=1e-9)


def test_each_stage_stays_within_its_quantizers_half_steps():
    rng = np.random.default_rng(7)
    m, g = 4, 32
    x = rng.standard_normal((1, 8, 8, 32)).astype(np.float32)
    AT, BT, G = ct.standard_matrices(m)
    st = fullint.input_transform_int(x, BT, m, g)
    d = _patches_by_hand(x, m).astype(np.float64)
    T, C = d.shape[:2]
    step = np.repeat(st["s_qx"], g, axis=1)[:, :, None, None]
    assert (np.abs(d - st["Qx"] * step) <= step / 2 * (1 + 1e-6)).all()
    assert np.abs(st["Qx"]).reshape(T, -1).max(axis=1).min() == 127
    # X~ is the product of the DE-quantized factors (integer product, scales outside)
    Bh = st["QB"] * st["s_qB"][:, None]
    want = np.einsum("ik,tckl,jl->tcij", Bh, st["Qx"] * step, Bh)
    got = st["Xt"].reshape(m + 2, m + 2, T, C).transpose(2, 3, 0, 1)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)


def test_power_of_two_rescaling_of_the_input_passes_straight_through():
    rng = np.random.default_rng(8)
    m, g = 4, 32
    x = rng.standard_normal((1, 9, 7, 64)).astype(np.float32)
    w = (rng.standard_normal((16, 64, 3, 3)) * 0.05).astype(np.float32)
    AT, BT, G = ct.standard_matrices(m)
    a = fullint.fullint_pipeline(x, w, None, AT, BT, G, m, g)
    b = fullint.fullint_pipeline(x * np.float32(8.0), w, None, AT, BT, G, m, g)
    assert np.array_equal(a["stage1"]["Qx"], b["stage1"]["Qx"]) and np.array_equal(a["Xq"], b["Xq"])
    assert np.array_equal(a["stage3"]["QY"], b["stage3"]["QY"])
    assert np.array_equal(a["y"] * 8.0, b["y"])


def test_f23_pipeline_is_close_to_the_convolution_and_bias_is_added_last():
    rng = np.random.default_rng(9)
    x = rng.standard_normal((2, 10, 10, 64)).astype(np.float32)
    w = (rng.standard_normal((24, 64, 3, 3)) * 0.06).astype(np.float32)
    bias = rng.standard_normal(24).astype(np.float32)
    AT, BT, G = ct.standard_matrices(2)
    ref = oracle.direct_conv(x, w, bias)
    got = fullint.fullint_pipeline(x, w, bias, AT, BT, G, 2, 32)
    assert fullint.sqnr_db(ref, got["y"]) > 30.0
    nob = fullint.fullint_pipeline(x, w, None, AT, BT, G, 2, 32)
    np.testing.assert_allclose(got["y"] - nob["y"], np.broadcast_to(bias.astype(np.float64), ref.shape), atol=1e-12)


@pytest.mark.parametrize("matrix_scales", ["matrix", "row"])
def test_learned_f63_scales_beat_the_standard_ones_and_flatten_the_dynamic_range(matrix_scales):
    """The paper's claim for this pipeline, on random Gaussian inputs (the data it fine-tunes on)
    and synthetic weights: standard F(6,3) scales are unusable, the learned ones it tabulates are
    much better, and the per-tap spread of the Winograd-domain output shrinks."""
    rng = np.random.default_rng(10)
    x = rng.standard_normal((1, 24, 24, 64)).astype(np.float32)
    w = (rng.standard_normal((32, 64, 3, 3)) * np.sqrt(2 / (9 * 64))).astype(np.float32)
    ref = oracle.direct_conv(x, w, None)
    std = fullint.fullint_pipeline(x, w, None, *ct.standard_matrices(6), 6, 32, matrix_scales)
    lrn = fullint.fullint_pipeline(x, w, None, *_learned_f63(), 6, 32, matrix_scales)
    s_std, s_lrn = fullint.sqnr_db(ref, std["y"]), fullint.sqnr_db(ref, lrn["y"])
    print(f"{matrix_scales}: SQNR standard {s_std:.1f} dB, learned {s_lrn:.1f} dB")
    assert s_lrn > s_std + 10.0
    r_std, r_lrn = fullint.tap_relative_std(std["Yt"], 6), fullint.tap_relative_std(lrn["Yt"], 6)
    spread = lambda r: r.max() / r.min()
    print(f"per-tap relative std: max/min {spread(r_std):.0f} (standard) -> {spread(r_lrn):.0f} (learned)")
    assert spread(r_std) > 10 * spread(r_lrn)
    # the 'cross': with the standard scales the rows/columns of the points +-2 are the faint ones
    assert r_std[3:5, :].max() < 0.2 and r_std[:, 3:5].max() < 0.2 and r_std[0, 0] > 1.0
