"""Pins for the oracle of the group-wise quantized standard (direct) convolution.

The paper names this layer only as its runtime comparison point (Section
"Runtime improvements") and prints no formula or number for it, so the pins are
mathematical: a library convolution of the de-quantized tensors, a lossless
special case that must reproduce the exact convolution, pure-Python brute force
on sampled outputs, the quantizer's error bound, and the Winograd oracle run as
F(1,3) with identity transforms (which is the same computation, tap by tap).
"""
import numpy as np
import pytest
import torch

import oracle


def _data(seed, N, H, W, Cin, Cout, scale_w=0.1):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((N, H, W, Cin)).astype(np.float32)
    x[..., rng.integers(0, Cin)] *= 20.0
    w = (rng.standard_normal((Cout, Cin, 3, 3)) * scale_w).astype(np.float32)
    b = rng.standard_normal(Cout).astype(np.float32)
    return x, w, b


def _dequant(r, N, H, W, g):
    """fp64 tensors x^ = sx*xq [N][H][W][Cin] and w^ = sw*wq [Cout][Cin][3][3]."""
    Cin = r["xq"].shape[1]
    xh = r["xq"].astype(np.float64) * np.repeat(r["sx"].astype(np.float64), g, axis=1)
    xh = xh.reshape(N, H, W, Cin)
    Cout = r["wq"].shape[1]
    swf = np.repeat(r["sw"].astype(np.float64), g, axis=1)          # [9][Cin][Cout]
    wh = r["wq"].astype(np.float64) * swf.transpose(0, 2, 1)        # [9][Cout][Cin]
    wh = wh.transpose(1, 2, 0).reshape(Cout, Cin, 3, 3)
    return xh, wh


@pytest.mark.parametrize("g", [32, 64])
def test_equals_library_convolution_of_dequantized_tensors(g):
    N, H, W, Cin, Cout = 2, 6, 5, 128, 24
    x, w, b = _data(3, N, H, W, Cin, Cout)
    r = oracle.direct_pipeline(x, w, b, g)
    xh, wh = _dequant(r, N, H, W, g)
    ref = torch.nn.functional.conv2d(torch.from_numpy(xh).permute(0, 3, 1, 2), torch.from_numpy(wh),
                                     torch.from_numpy(b.astype(np.float64)), padding=1)
    ref = ref.permute(0, 2, 3, 1).numpy()
    assert np.abs(r["y64"] - ref).max() <= 1e-12 * np.abs(ref).max()
    assert np.array_equal(r["y"], r["y64"].astype(np.float32))


def test_scales_and_codes_follow_the_group_partition():
    N, H, W, Cin, Cout, g = 1, 3, 4, 96, 8, 32
    x, w, _ = _data(4, N, H, W, Cin, Cout)
    xq, sx = oracle.quantize_pixels(x, g)
    wq, sw = oracle.quantize_filters(w, g)
    xa = np.abs(x.reshape(-1, Cin // g, g)).max(axis=2)
    assert np.array_equal(sx, xa / np.float32(127.0))
    wa = np.abs(w.reshape(Cout, Cin // g, g, 9)).max(axis=2)          # [Cout][groups][9]
    assert np.array_equal(sw, (wa / np.float32(127.0)).transpose(2, 1, 0))
    # every non-zero group uses the full code range and stays within half a step
    assert (np.abs(xq.reshape(-1, Cin // g, g)).max(axis=2) == 127).all()
    assert (np.abs(wq.reshape(9, Cout, Cin // g, g)).max(axis=3) == 127).all()
    err = np.abs(x.reshape(-1, Cin) - np.repeat(sx, g, axis=1) * xq)
    assert (err <= np.repeat(sx, g, axis=1) * 0.5 * (1 + 1e-4)).all()   # s and r each carry one fp32 rounding of the abs-max
    wt = w.transpose(2, 3, 0, 1).reshape(9, Cout, Cin)
    errw = np.abs(wt - np.repeat(sw, g, axis=1).transpose(0, 2, 1) * wq)
    assert (errw <= np.repeat(sw, g, axis=1).transpose(0, 2, 1) * 0.5 * (1 + 1e-4)).all()   # s and r each carry one fp32 rounding of the abs-max


def test_lossless_groups_reproduce_the_exact_convolution():
    """Integer-valued data with abs-max 127 in every group quantizes without error."""
    N, H, W, Cin, Cout, g = 1, 5, 5, 64, 4, 32
    rng = np.random.default_rng(5)
    x = rng.integers(-127, 128, size=(N, H, W, Cin)).astype(np.float32)
    x[..., 0::g] = 127.0
    w = rng.integers(-127, 128, size=(Cout, Cin, 3, 3)).astype(np.float32)
    w[:, 0::g] = -127.0
    x *= np.float32(2.0 ** -3)
    w *= np.float32(2.0 ** -9)
    b = rng.standard_normal(Cout).astype(np.float32)
    r = oracle.direct_pipeline(x, w, b, g)
    ref = oracle.direct_conv(x, w, b)
    assert np.abs(r["y64"] - ref).max() <= 1e-12 * np.abs(ref).max()


def test_sampled_outputs_by_brute_force():
    N, H, W, Cin, Cout, g = 2, 4, 5, 64, 6, 32
    x, w, b = _data(6, N, H, W, Cin, Cout)
    r = oracle.direct_pipeline(x, w, b, g)
    xq, sx, wq, sw = (r[k] for k in ("xq", "sx", "wq", "sw"))
    rng = np.random.default_rng(7)
    picks = [(0, 0, 0, 0), (N - 1, H - 1, W - 1, Cout - 1), (0, 0, W - 1, 1), (1, H - 1, 0, 2)]
    picks += [tuple(int(rng.integers(0, d)) for d in (N, H, W, Cout)) for _ in range(8)]
    for (bi, h, q, o) in picks:
        acc = float(b[o])
        for u in range(3):
            for v in range(3):
                hh, ww = h + u - 1, q + v - 1
                if not (0 <= hh < H and 0 <= ww < W):
                    continue
                pix = (bi * H + hh) * W + ww
                for gi in range(Cin // g):
                    p = 0
                    for c in range(gi * g, (gi + 1) * g):
                        p += int(xq[pix, c]) * int(wq[u * 3 + v, o, c])
                    acc += p * float(sx[pix, gi]) * float(sw[u * 3 + v, gi, o])
        assert abs(acc - r["y64"][bi, h, q, o]) <= 1e-12 * max(1.0, abs(acc))


def test_error_against_the_unquantized_convolution_is_within_the_quantizer_bound():
    N, H, W, Cin, Cout, g = 1, 6, 6, 64, 8, 32
    x, w, b = _data(8, N, H, W, Cin, Cout)
    r = oracle.direct_pipeline(x, w, b, g)
    ref = oracle.direct_conv(x, w, b)
    # |x w - x^ w^| <= |x| sw/2 + |w| sx/2 + sx sw/4 per product, summed over the window
    sxf = np.repeat(r["sx"], g, axis=1).reshape(N, H, W, Cin).astype(np.float64)
    swf = np.repeat(r["sw"], g, axis=1).transpose(2, 1, 0).reshape(Cout, Cin, 3, 3).astype(np.float64)
    ax, aw = np.abs(x).astype(np.float64), np.abs(w).astype(np.float64)
    conv = lambda a, k: torch.nn.functional.conv2d(torch.from_numpy(a).permute(0, 3, 1, 2), torch.from_numpy(k),
                                                   padding=1).permute(0, 2, 3, 1).numpy()
    bound = 0.5 * conv(ax, swf) + 0.5 * conv(sxf, aw) + 0.25 * conv(sxf, swf)
    err = np.abs(r["y64"] - ref)
    assert (err <= bound * (1 + 1e-6) + 1e-12).all()
    assert err.max() > 0          # it is a lossy path
    # a planted mistake (scales of the wrong group) breaks the bound
    bad = dict(r)
    bad_sx = r["sx"][:, ::-1].copy()
    y_bad, _ = oracle.direct_qconv(r["xq"], bad_sx, r["wq"], r["sw"], b, N, H, W, g)
    assert not (np.abs(y_bad - ref) <= bound * (1 + 1e-6) + 1e-12).all()


def test_winograd_oracle_as_F13_with_identity_transforms_is_the_same_computation():
    """F(1,3): B^T = G = I (3x3), A^T = [1 1 1]: tap (u,v) of tile (= pixel) tau is the
    input pixel shifted by (u-1, v-1), so codes, scales and outputs must coincide."""
    N, H, W, Cin, Cout, g = 1, 4, 5, 64, 5, 32
    x, w, b = _data(9, N, H, W, Cin, Cout)
    I3 = np.eye(3, dtype=np.float32)
    AT = np.ones((1, 3), dtype=np.float32)
    rw = oracle.qwino_pipeline(x, w, b, AT, I3, I3, 1, g)
    rd = oracle.direct_pipeline(x, w, b, g)
    assert np.array_equal(rw["Wq"], rd["wq"]) and np.array_equal(rw["sW"], rd["sw"])
    # centre tap of every tile is the pixel itself
    assert np.array_equal(rw["Xq"][4], rd["xq"]) and np.array_equal(rw["sX"][4], rd["sx"])
    assert np.abs(rw["y64"] - rd["y64"]).max() <= 1e-12 * np.abs(rd["y64"]).max()
