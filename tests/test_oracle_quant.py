"""Pins for the oracle's quantized stages (CPU only).

quantizer   invariants that follow from its definition, worked tie cases,
            the lossless special case, zero and sub-normal groups;
transforms  the fp32 chains against the matrix products B^T d B and G g G^T
            evaluated in fp64 on independently extracted tiles;
contract    a different loop nest and numpy's integer einsum;
pipeline    (i) inputs for which quantization is lossless must reproduce the
            un-quantized convolution, (ii) on random inputs the error against
            the un-quantized Winograd result must stay inside the bound that
            follows from |v - s q| <= s/2 element by element - a wrong scale
            index, a dropped group or a transposed operand breaks one of them.
"""
import numpy as np
import pytest

import oracle
from oracle import cook_toom as ct
from paper_2412_19867_amd import workloads

F32 = np.float32
EPS = np.finfo(np.float32).eps


# ------------------------------------------------------------- quantizer
def test_quantizer_worked_ties_round_half_to_even():
    # absmax 127 -> r = 1, s = 1 exactly
    v = np.array([127, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 3.49, 126.5, -126.5, 0, 64.5] + [0] * 20, F32)
    q, s = oracle.quantize_group(v)
    assert s == F32(1.0)
    assert q[:12].tolist() == [127, 0, 2, 2, 0, -2, -2, 3, 126, -126, 0, 64]


def test_quantizer_invariants():
    rng = np.random.default_rng(0)
    for trial in range(200):
        g = [32, 64, 256][trial % 3]
        v = (rng.standard_normal(g) * 10.0 ** rng.uniform(-6, 6)).astype(F32)
        q, s = oracle.quantize_group(v)
        a = np.abs(v).max()
        assert s == F32(a) / F32(127.0)
        assert np.abs(q.astype(np.int32)).max() == 127
        # reconstruction error at most half a step (plus rounding of s and r)
        err = np.abs(v.astype(np.float64) - float(s) * q.astype(np.float64))
        assert err.max() <= 0.5 * float(s) * (1 + 300 * EPS)
        # odd symmetry
        q2, s2 = oracle.quantize_group(-v)
        assert s2 == s and np.array_equal(q2, -q)
        # power-of-two scaling leaves the codes unchanged
        k = int(rng.integers(-20, 20))
        q3, s3 = oracle.quantize_group(np.ldexp(v, k).astype(F32))
        assert np.array_equal(q3, q) and s3 == np.ldexp(s, k)


def test_quantizer_lossless_when_values_are_integers_times_a_power_of_two():
    rng = np.random.default_rng(1)
    ints = rng.integers(-127, 128, size=64)
    ints[5] = 127
    for k in (-9, 0, 7):
        v = np.ldexp(ints.astype(F32), k)
        q, s = oracle.quantize_group(v)
        assert np.array_equal(q.astype(np.int64), ints) and s == np.ldexp(F32(1), k)


def test_quantizer_zero_and_subnormal_groups():
    q, s = oracle.quantize_group(np.zeros(32, F32))
    assert s == 0 and not q.any()
    tiny = np.full(32, 1e-40, F32)          # sub-normal absmax: below 127*FLT_MIN
    q, s = oracle.quantize_group(tiny)
    assert s == 0 and not q.any()
    fl_min = np.finfo(F32).tiny
    v = np.zeros(32, F32)
    v[3] = F32(127) * fl_min                # smallest absmax that is still quantized
    v[4] = -fl_min * F32(64)
    q, s = oracle.quantize_group(v)
    assert s == fl_min and q[3] == 127 and q[4] == -64


# ------------------------------------------------------------ transforms
def tiles_of(x, m):
    """[T, n, n, C] input tiles with the 1-pixel zero border, by numpy padding."""
    N, H, W, C = x.shape
    n = m + 2
    TH, TW = -(-H // m), -(-W // m)
    xp = np.zeros((N, TH * m + 2, TW * m + 2, C), x.dtype)
    xp[:, 1:H + 1, 1:W + 1] = x
    out = np.empty((N * TH * TW, n, n, C), x.dtype)
    for b in range(N):
        for th in range(TH):
            for tw in range(TW):
                out[(b * TH + th) * TW + tw] = xp[b, th * m:th * m + n, tw * m:tw * m + n]
    return out


@pytest.mark.parametrize("m,shape", [(4, (2, 7, 10, 32)), (6, (1, 13, 6, 64)), (2, (1, 5, 5, 32))])
def test_input_transform_is_BT_d_B(m, shape):
    rng = np.random.default_rng(m)
    x = rng.standard_normal(shape).astype(F32)
    u = rng.uniform(0.5, 2, m + 2)
    _, BT, _ = ct.scaled_matrices(m, u, u[::-1])      # asymmetric, non-standard
    BT32 = BT.astype(F32)
    _, _, Xf = oracle.input_transform_quant(x, BT32, m, 32, want_float=True)
    d = tiles_of(x, m).astype(np.float64)             # [T,n,n,C]
    ref = np.einsum("ik,tklc,jl->ijtc", BT32.astype(np.float64), d, BT32.astype(np.float64))
    n = m + 2
    ref = ref.reshape(n * n, d.shape[0], shape[3])
    mag = np.einsum("ik,tklc,jl->ijtc", np.abs(BT32).astype(np.float64), np.abs(d),
                    np.abs(BT32).astype(np.float64)).reshape(ref.shape)
    assert np.all(np.abs(Xf - ref) <= 4 * n * EPS * mag + 1e-30)


@pytest.mark.parametrize("m", [2, 4, 6])
def test_weight_transform_is_G_g_GT(m):
    rng = np.random.default_rng(40 + m)
    w = rng.standard_normal((5, 32, 3, 3)).astype(F32)
    u = rng.uniform(0.5, 2, m + 2)
    _, _, G = ct.scaled_matrices(m, u[::-1], u)
    G32 = G.astype(F32)
    _, _, Wf = oracle.weight_transform_quant(w, G32, m, 32, want_float=True)
    G64 = G32.astype(np.float64)
    ref = np.einsum("ik,ockl,jl->ijoc", G64, w.astype(np.float64), G64).reshape((m + 2) ** 2, 5, 32)
    mag = np.einsum("ik,ockl,jl->ijoc", np.abs(G64), np.abs(w).astype(np.float64),
                    np.abs(G64)).reshape(ref.shape)
    assert np.all(np.abs(Wf - ref) <= 8 * EPS * mag + 1e-30)


def test_stage_outputs_are_the_quantizer_applied_per_group():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((1, 6, 9, 64)).astype(F32)
    x[..., 7] *= 20
    _, BT, _ = ct.standard_matrices(4)
    Xq, sX, Xf = oracle.input_transform_quant(x, BT, 4, 32, want_float=True)
    for t in (0, 7, 35):
        for tau in (0, 3, 5):
            for gi in (0, 1):
                q, s = oracle.quantize_group(Xf[t, tau, gi * 32:(gi + 1) * 32])
                assert s == sX[t, tau, gi]
                assert np.array_equal(q, Xq[t, tau, gi * 32:(gi + 1) * 32])
    w = rng.standard_normal((3, 64, 3, 3)).astype(F32)
    _, _, G = ct.standard_matrices(4)
    Wq, sW, Wf = oracle.weight_transform_quant(w, G, 4, 32, want_float=True)
    for t in (0, 17, 35):
        for o in range(3):
            for gi in (0, 1):
                q, s = oracle.quantize_group(Wf[t, o, gi * 32:(gi + 1) * 32])
                assert s == sW[t, gi, o]
                assert np.array_equal(q, Wq[t, o, gi * 32:(gi + 1) * 32])


# -------------------------------------------------------------- contract
def test_integer_contraction_against_brute_force_and_einsum():
    rng = np.random.default_rng(4)
    n2, T, Cin, Cout, g = 16, 5, 96, 7, 32
    Xq = rng.integers(-127, 128, (n2, T, Cin), dtype=np.int8)
    Wq = rng.integers(-127, 128, (n2, Cout, Cin), dtype=np.int8)
    sX = rng.uniform(0.1, 1, (n2, T, Cin // g)).astype(F32)
    sW = rng.uniform(0.1, 1, (n2, Cin // g, Cout)).astype(F32)
    M, P = oracle.contract(Xq, sX, Wq, sW, g, want_P=True)
    assert np.array_equal(P.astype(np.int64), oracle.contract_bruteforce(Xq, Wq, g))
    ref = np.einsum("atgc,aogc->atgo", Xq.reshape(n2, T, Cin // g, g).astype(np.int64),
                    Wq.reshape(n2, Cout, Cin // g, g).astype(np.int64))
    assert np.array_equal(P.astype(np.int64), ref)
    Mref = np.einsum("atgo,atg,ago->ato", ref.astype(np.float64), sX.astype(np.float64),
                     sW.astype(np.float64))
    np.testing.assert_allclose(M, Mref, rtol=1e-13)
    # extreme codes do not overflow int32 at the largest group the library admits
    Xq = np.full((1, 1, 1024), -127, np.int8)
    Wq = np.full((1, 1, 1024), -127, np.int8)
    _, P = oracle.contract(Xq, np.ones((1, 1, 1), F32), Wq, np.ones((1, 1, 1), F32), 1024, want_P=True)
    assert P[0, 0, 0, 0] == 1024 * 127 * 127


# -------------------------------------------------------------- pipeline
@pytest.mark.parametrize("m,g", [(4, 32), (6, 32), (4, 64)])
def test_pipeline_lossless_case_equals_unquantized(m, g):
    """One non-zero channel per group: every group holds a single value, which
    the quantizer represents as +-127 * (|v|/127) - exact up to fp32 rounding.
    The quantized path must then agree with the direct convolution."""
    rng = np.random.default_rng(m * g)
    Cin, Cout = 2 * g, 6
    x = np.zeros((2, 9, 7, Cin), F32)
    w = np.zeros((Cout, Cin, 3, 3), F32)
    keep = [3, g + 11]
    x[..., keep] = rng.standard_normal((2, 9, 7, 2)).astype(F32)
    w[:, keep] = rng.standard_normal((Cout, 2, 3, 3)).astype(F32)
    b = rng.standard_normal(Cout).astype(F32)
    AT, BT, G = ct.standard_matrices(m)
    out = oracle.qwino_pipeline(x, w, b, AT, BT, G, m, g)
    yd = oracle.direct_conv(x, w, b)
    assert np.abs(out["y64"] - yd).max() <= 2e-5 * np.abs(yd).max()
    assert np.abs(out["y"] - yd).max() <= 2e-5 * np.abs(yd).max()


@pytest.mark.parametrize("m,g,scaled", [(4, 32, False), (6, 32, True), (4, 64, True)])
def test_pipeline_error_stays_inside_the_quantizer_bound(m, g, scaled):
    d = workloads.small_layer(seed=m + g, N=1, H=10, W=9, Cin=2 * g, Cout=8, m=m, group_size=g,
                              row_scales=scaled)
    if scaled:
        AT, BT, G = ct.scaled_matrices(m, d.u_B, d.u_G)
    else:
        AT, BT, G = ct.standard_matrices(m)
    AT, BT, G = AT.astype(F32), BT.astype(F32), G.astype(F32)
    out = oracle.qwino_pipeline(d.x, d.w, d.bias, AT, BT, G, m, g)
    _, _, Xf = oracle.input_transform_quant(d.x, BT, m, g, want_float=True)
    _, _, Wf = oracle.weight_transform_quant(d.w, G, m, g, want_float=True)
    n2, T, Cin = Xf.shape
    Cout = Wf.shape[1]
    half = 0.5 * (1 + 300 * EPS)
    eX = np.repeat(out["sX"].astype(np.float64) * half, g, axis=2)             # [n2,T,Cin]
    eW = np.repeat(out["sW"].transpose(0, 2, 1).astype(np.float64) * half, g, axis=2)  # [n2,Cout,Cin]
    aX, aW = np.abs(Xf).astype(np.float64), np.abs(Wf).astype(np.float64)
    boundM = (np.einsum("atc,aoc->ato", eX, aW) + np.einsum("atc,aoc->ato", aX, eW)
              + np.einsum("atc,aoc->ato", eX, eW))
    Mexact = np.einsum("atc,aoc->ato", Xf.astype(np.float64), Wf.astype(np.float64))
    assert np.all(np.abs(out["M"] - Mexact) <= boundM * (1 + 1e-6))
    # the bound is not vacuous: the error uses a real fraction of it somewhere
    assert (np.abs(out["M"] - Mexact) / (boundM + 1e-300)).max() > 0.02
    # output: same matrices un-quantized in fp64, element-wise bound through |A^T|
    yw = oracle.winograd_f64(d.x, d.w, d.bias, AT, BT, G, m)
    bm = boundM + 16 * EPS * np.einsum("atc,aoc->ato", aX, aW)      # fp32 transform rounding
    by, _ = oracle.output_transform(bm, np.abs(AT), None, 1, 10, 9, m)
    assert np.all(np.abs(out["y64"] - yw) <= by * (1 + 1e-6) + 1e-9)
    # signal-to-quantization-noise floor against the direct convolution
    yd = oracle.direct_conv(d.x, d.w, d.bias)
    sqnr = 10 * np.log10((yd ** 2).sum() / ((out["y64"] - yd) ** 2).sum())
    assert sqnr > 8.0, sqnr      # gross-error floor only; the paper prints no SQNR value
    # fp32 copy of the output is the rounded fp64 one
    assert np.array_equal(out["y"], out["y64"].astype(F32))


def test_pipeline_bound_catches_a_misindexed_scale():
    """Sensitivity of the pin above: permuting the activation scales between
    groups (a plausible indexing slip) must violate the element-wise bound."""
    m, g = 4, 32
    d = workloads.small_layer(seed=11, N=1, H=8, W=8, Cin=64, Cout=4, m=m, group_size=g)
    AT, BT, G = (M.astype(F32) for M in ct.standard_matrices(m))
    Xq, sX, Xf = oracle.input_transform_quant(d.x, BT, m, g, want_float=True)
    Wq, sW, Wf = oracle.weight_transform_quant(d.w, G, m, g, want_float=True)
    M_bad = oracle.contract(Xq, sX[:, :, ::-1].copy(), Wq, sW, g)
    half = 0.5 * (1 + 300 * EPS)
    eX = np.repeat(sX.astype(np.float64) * half, g, axis=2)
    eW = np.repeat(sW.transpose(0, 2, 1).astype(np.float64) * half, g, axis=2)
    aX, aW = np.abs(Xf).astype(np.float64), np.abs(Wf).astype(np.float64)
    boundM = (np.einsum("atc,aoc->ato", eX, aW) + np.einsum("atc,aoc->ato", aX, eW)
              + np.einsum("atc,aoc->ato", eX, eW))
    Mexact = np.einsum("atc,aoc->ato", Xf.astype(np.float64), Wf.astype(np.float64))
    assert np.any(np.abs(M_bad - Mexact) > boundM * 1.5)


@pytest.mark.parametrize("m", [2, 4, 6])
def test_power_of_two_row_scales_change_nothing_but_the_stored_scales(m):
    """With transforms in fp32 and only X and W quantized, a diagonal rescaling of B^T and G
    multiplies every tap by one factor for all channels; the dynamic abs-max scale of each
    group absorbs it and S_A = (S_B S_G)^-1 undoes it.  For powers of two this holds exactly:
    same int8 codes, scales multiplied by the tap's factor, same int32 sums, same output."""
    n = m + 2
    rng = np.random.default_rng(40 + m)
    kB, kG = rng.integers(-3, 4, n), rng.integers(-3, 4, n)
    mats0 = tuple(M.astype(np.float32) for M in ct.standard_matrices(m))
    mats1 = tuple(M.astype(np.float32) for M in ct.scaled_matrices(m, 2.0 ** kB, 2.0 ** kG))
    d = workloads.small_layer(60 + m, 2, 9, 7, 64, 24, m, 32)
    r0 = oracle.qwino_pipeline(d.x, d.w, d.bias, *mats0, m, 32, want_P=True)
    r1 = oracle.qwino_pipeline(d.x, d.w, d.bias, *mats1, m, 32, want_P=True)
    assert np.array_equal(r0["Xq"], r1["Xq"]) and np.array_equal(r0["Wq"], r1["Wq"])
    assert np.array_equal(r0["P"], r1["P"])
    fB = (2.0 ** (kB[:, None] + kB[None, :])).reshape(n * n).astype(np.float32)
    fG = (2.0 ** (kG[:, None] + kG[None, :])).reshape(n * n).astype(np.float32)
    assert np.array_equal(r1["sX"], r0["sX"] * fB[:, None, None])
    assert np.array_equal(r1["sW"], r0["sW"] * fG[:, None, None])
    assert np.array_equal(r0["y64"], r1["y64"])


def test_reciprocal_reading_of_the_quantizer_against_the_literal_division():
    """The library and the oracle evaluate x / s as x * (127 / a) (one division per group).  On
    the Winograd-domain activations and weights of config 1 this differs from the division the
    quantizer equation writes only in codes where x / s lies within a rounding error of a
    half-integer: a few codes in a million, each by exactly one step, and the scales are the
    same numbers.  (The count is quoted in the design doc.)"""
    from paper_2412_19867_amd import workloads
    d = workloads.make_layer_data(workloads.CONFIGS[1][0])
    lay = d.layer
    AT, BT, G = (M.astype(np.float32) for M in ct.standard_matrices(lay.m))
    _, _, Xf = oracle.input_transform_quant(d.x, BT, lay.m, lay.group_size, want_float=True)
    _, _, Wf = oracle.weight_transform_quant(d.w, G, lay.m, lay.group_size, want_float=True)
    total = differ = 0
    for tensor in (Xf, Wf):
        groups = np.ascontiguousarray(tensor.reshape(-1, lay.group_size))
        for row in groups[:: max(1, len(groups) // 20000)]:          # ~20000 groups of each tensor
            qa, sa = oracle.quantize_group(row)
            ql, sl = oracle.quantize_group_literal(row)
            assert sa == sl
            delta = np.abs(qa.astype(np.int32) - ql.astype(np.int32))
            assert delta.max() <= 1
            differ += int(np.count_nonzero(delta))
            total += row.size
    print(f"codes that differ from the literal division: {differ} of {total} ({differ / total:.2e})")
    assert differ / total < 1e-4
