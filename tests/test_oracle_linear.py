"""Pins for the oracle of the group-wise quantized linear layer (Section "Experiments":
the same quantization is applied to every linear layer and attention product).  No number
is printed for it, so the pins are mathematical: numpy's matrix product of the
de-quantized operands, a lossless special case, the quantizer's error bound, and the
direct-convolution oracle on a 1x1 image whose centre tap is the weight matrix."""
import numpy as np

import oracle


def _data(seed, R, Cin, Cout):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((R, Cin)).astype(np.float32)
    x[:, rng.integers(0, Cin)] *= 20.0
    w = (rng.standard_normal((Cout, Cin)) * 0.1).astype(np.float32)
    b = rng.standard_normal(Cout).astype(np.float32)
    return x, w, b


def test_equals_numpy_product_of_dequantized_operands():
    for g in (32, 64, 128):
        x, w, b = _data(1, 37, 256, 19)
        r = oracle.linear_pipeline(x, w, b, g)
        xh = r["xq"].astype(np.float64) * np.repeat(r["sx"].astype(np.float64), g, axis=1)
        wh = r["wq"].astype(np.float64) * np.repeat(r["sw"].astype(np.float64), g, axis=0).T
        ref = xh @ wh.T + b.astype(np.float64)
        assert np.abs(r["y64"] - ref).max() <= 1e-12 * np.abs(ref).max()
        assert np.array_equal(r["y"], r["y64"].astype(np.float32))
        # scales follow the (row, group) partition of the weight matrix
        wa = np.abs(w.reshape(19, 256 // g, g)).max(axis=2)
        assert np.array_equal(r["sw"], (wa / np.float32(127.0)).T)


def test_lossless_groups_reproduce_the_exact_product():
    rng = np.random.default_rng(2)
    R, Cin, Cout, g = 9, 128, 7, 32
    x = rng.integers(-127, 128, size=(R, Cin)).astype(np.float32)
    w = rng.integers(-127, 128, size=(Cout, Cin)).astype(np.float32)
    x[:, 0::g] = 127.0
    w[:, 0::g] = -127.0
    x *= np.float32(0.25)
    w *= np.float32(2.0 ** -10)
    r = oracle.linear_pipeline(x, w, None, g)
    ref = x.astype(np.float64) @ w.astype(np.float64).T
    assert np.abs(r["y64"] - ref).max() <= 1e-12 * np.abs(ref).max()


def test_error_is_within_the_quantizer_bound():
    x, w, b = _data(3, 21, 128, 11)
    g = 32
    r = oracle.linear_pipeline(x, w, b, g)
    ref = x.astype(np.float64) @ w.astype(np.float64).T + b
    sxf = np.repeat(r["sx"].astype(np.float64), g, axis=1)
    swf = np.repeat(r["sw"].astype(np.float64), g, axis=0).T
    bound = 0.5 * np.abs(x) @ swf.T + 0.5 * sxf @ np.abs(w).T + 0.25 * sxf @ swf.T
    err = np.abs(r["y64"] - ref)
    assert (err <= bound * (1 + 1e-4) + 1e-12).all() and err.max() > 0


def test_same_as_the_centre_tap_of_the_direct_convolution_oracle():
    """A 1x1 image: only the centre tap of a 3x3 filter sees it."""
    x, w, b = _data(4, 6, 64, 5)
    g = 32
    w33 = np.zeros((5, 64, 3, 3), dtype=np.float32)
    w33[:, :, 1, 1] = w
    rd = oracle.direct_pipeline(x.reshape(6, 1, 1, 64), w33, b, g)
    rl = oracle.linear_pipeline(x, w, b, g)
    assert np.array_equal(rd["xq"], rl["xq"]) and np.array_equal(rd["wq"][4], rl["wq"])
    assert np.abs(rd["y64"].reshape(6, 5) - rl["y64"]).max() <= 1e-12 * np.abs(rl["y64"]).max()
