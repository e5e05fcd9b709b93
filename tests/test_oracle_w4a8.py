"""Pins for the 4-bit weight quantizer of the W4A8 rows in the paper's tables (weights
4 bits, activations 8 bits, standard convolution and linear layers).  The paper prints no
worked example, so the pins are mathematical: the quantizer against a formula typed out
here in numpy fp64, its range and error bound, the lossless case, the product of the
de-quantized operands, and the expected 127/7 loss of resolution against 8-bit weights."""
import numpy as np

import oracle


def test_quantizer_against_the_definition_in_fp64():
    rng = np.random.default_rng(11)
    for _ in range(50):
        v = (rng.standard_normal(32) * 10.0 ** rng.uniform(-3, 3)).astype(np.float32)
        q, s = oracle.quantize_group_bits(v, 4)
        a = np.abs(v).max()
        assert s == np.float32(a) / np.float32(7.0)
        assert np.abs(q).max() == 7 and q.min() >= -7 and q.max() <= 7
        # codes: round-half-even of v*(7/a); away from ties the fp64 value decides
        t = v.astype(np.float64) * 7.0 / float(a)
        clear = np.abs(t - np.floor(t) - 0.5) > 1e-5
        assert np.array_equal(q[clear], np.rint(t[clear]).astype(np.int8))
        assert (np.abs(v - s * q.astype(np.float32)) <= 0.5 * s * (1 + 1e-5)).all()
    # 8 bits through the same entry point is the int8 quantizer
    v = rng.standard_normal(64).astype(np.float32)
    q8, s8 = oracle.quantize_group_bits(v, 8)
    q8b, s8b = oracle.quantize_group(v)
    assert np.array_equal(q8, q8b) and s8 == s8b


def test_zero_and_tiny_groups():
    q, s = oracle.quantize_group_bits(np.zeros(32, np.float32), 4)
    assert s == 0 and not q.any()
    q, s = oracle.quantize_group_bits(np.full(32, 1e-44, np.float32), 4)   # below 7*FLT_MIN: the zero group
    assert s == 0 and not q.any()
    v = np.zeros(32, np.float32)
    v[5] = -3.5
    q, s = oracle.quantize_group_bits(v, 4)
    assert q[5] == -7 and s == np.float32(0.5) and np.count_nonzero(q) == 1


def test_integer_weights_up_to_seven_are_lossless():
    rng = np.random.default_rng(12)
    R, Cin, Cout, g = 11, 128, 9, 32
    x = rng.integers(-127, 128, size=(R, Cin)).astype(np.float32)
    w = rng.integers(-7, 8, size=(Cout, Cin)).astype(np.float32)
    x[:, 0::g] = 127.0
    w[:, 0::g] = -7.0
    w *= np.float32(2.0 ** -6)
    r = oracle.linear_pipeline(x, w, None, g, weight_bits=4)
    assert np.array_equal(r["wq"], (w * 64).astype(np.int8))
    ref = x.astype(np.float64) @ w.astype(np.float64).T
    assert np.abs(r["y64"] - ref).max() <= 1e-12 * np.abs(ref).max()


def test_linear_equals_numpy_product_of_dequantized_operands():
    rng = np.random.default_rng(13)
    for g in (32, 64):
        x = rng.standard_normal((23, 256)).astype(np.float32)
        w = (rng.standard_normal((17, 256)) * 0.1).astype(np.float32)
        b = rng.standard_normal(17).astype(np.float32)
        r = oracle.linear_pipeline(x, w, b, g, weight_bits=4)
        assert np.abs(r["wq"]).max() == 7
        wa = np.abs(w.reshape(17, 256 // g, g)).max(axis=2)
        assert np.array_equal(r["sw"], (wa / np.float32(7.0)).T)
        xh = r["xq"].astype(np.float64) * np.repeat(r["sx"].astype(np.float64), g, axis=1)
        wh = r["wq"].astype(np.float64) * np.repeat(r["sw"].astype(np.float64), g, axis=0).T
        ref = xh @ wh.T + b.astype(np.float64)
        assert np.abs(r["y64"] - ref).max() <= 1e-12 * np.abs(ref).max()
        # the activations are untouched by the weight width
        r8 = oracle.linear_pipeline(x, w, b, g)
        assert np.array_equal(r["xq"], r8["xq"]) and np.array_equal(r["sx"], r8["sx"])


def test_direct_conv_equals_conv_of_dequantized_operands():
    import torch
    rng = np.random.default_rng(14)
    N, H, W, Cin, Cout, g = 2, 6, 7, 64, 10, 32
    x = rng.standard_normal((N, H, W, Cin)).astype(np.float32)
    w = (rng.standard_normal((Cout, Cin, 3, 3)) * 0.1).astype(np.float32)
    r = oracle.direct_pipeline(x, w, None, g, weight_bits=4)
    assert np.abs(r["wq"]).max() == 7
    xh = (r["xq"].astype(np.float64) * np.repeat(r["sx"].astype(np.float64), g, axis=1)).reshape(N, H, W, Cin)
    swf = np.repeat(r["sw"].astype(np.float64), g, axis=1)            # [9][Cin][Cout]
    wh = r["wq"].astype(np.float64) * swf.transpose(0, 2, 1)           # [9][Cout][Cin]
    wt = torch.from_numpy(wh.reshape(3, 3, Cout, Cin)).permute(2, 3, 0, 1).contiguous()
    ref = torch.nn.functional.conv2d(torch.from_numpy(xh).permute(0, 3, 1, 2), wt, padding=1)
    ref = ref.permute(0, 2, 3, 1).numpy()
    assert np.abs(r["y64"] - ref).max() <= 1e-12 * np.abs(ref).max()


def test_four_bit_weights_lose_about_127_over_7_in_resolution():
    rng = np.random.default_rng(15)
    x = rng.standard_normal((64, 512)).astype(np.float32)
    w = (rng.standard_normal((48, 512)) * 0.05).astype(np.float32)
    ref = x.astype(np.float64) @ w.astype(np.float64).T
    e8 = np.sqrt(np.mean((oracle.linear_pipeline(x, w, None, 32)["y64"] - ref) ** 2))
    e4 = np.sqrt(np.mean((oracle.linear_pipeline(x, w, None, 32, weight_bits=4)["y64"] - ref) ** 2))
    # weight rounding noise scales with the step (x 127/7 = 18); the 8-bit activation noise is common
    assert 8.0 < e4 / e8 < 18.5
