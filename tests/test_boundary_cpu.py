"""Host-side tests of the C-ABI library: they never launch a kernel.

The library loads without a GPU, exports every function include/wq.h declares,
carries standard matrices equal to the oracle's exact construction, and turns
every invalid argument into an error code before any device work.
"""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import cook_toom as ct

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol(wq):
    header = open(os.path.join(ROOT, "include", "wq.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(wq_[a-z_0-9]+)\s*\(", header))
    assert declared == set(wq.EXPORTS)
    L = wq.lib()
    for name in declared:
        assert getattr(L, name) is not None


@pytest.mark.parametrize("m", [2, 4, 6])
def test_standard_tables_equal_the_exact_construction(wq, m):
    AT, BT, G = wq.standard_transforms(m)
    AT0, BT0, G0 = ct.standard_matrices(m)
    np.testing.assert_array_equal(AT, AT0)
    np.testing.assert_array_equal(BT, BT0)
    np.testing.assert_allclose(G, G0, rtol=2e-16)     # thirds and ninths: one rounding each


def test_scaled_transforms_match_the_oracle_parametrisation(wq):
    rng = np.random.default_rng(0)
    for m in (4, 6):
        u_B, u_G = rng.uniform(0.5, 2, m + 2), rng.uniform(0.5, 2, m + 2)
        AT, BT, G = wq.scaled_transforms(m, u_B, u_G)
        AT0, BT0, G0 = ct.scaled_matrices(m, u_B, u_G)
        for a, b in ((AT, AT0), (BT, BT0), (G, G0)):
            assert a.dtype == np.float32
            np.testing.assert_allclose(a, b, rtol=1.2e-7)
    with pytest.raises(ValueError):
        wq.scaled_transforms(4, np.ones(5), np.ones(6))
    with pytest.raises(wq.WqError):
        wq.scaled_transforms(4, np.zeros(6), np.ones(6))
    with pytest.raises(wq.WqError):
        wq.scaled_transforms(4, np.full(6, np.inf), np.ones(6))
    with pytest.raises(wq.WqError):
        wq.scaled_transforms(5, np.ones(7), np.ones(7))
    # the result is a valid triple for wq_plan_create, and the paper's learned F(6,3) scales are too
    rng = np.random.default_rng(1)
    AT, BT, G = wq.scaled_transforms(6, rng.uniform(0.5, 2, 8), rng.uniform(0.5, 2, 8))
    wq.Plan(1, 8, 8, 32, 32, 6, 32, AT=AT, BT=BT, G=G)


def test_only_the_c_abi_is_exported(wq):
    """Hidden visibility: the dynamic symbol table holds the wq_* entry points and nothing else of
    the library's own (no mangled launchers)."""
    import subprocess
    out = subprocess.run(["nm", "-D", "--defined-only", wq.LIB_PATH], capture_output=True, text=True, check=True).stdout
    names = [l.split()[-1] for l in out.splitlines() if l.strip()]
    own = [n for n in names if "wq" in n.lower()]
    assert sorted(own) == sorted(wq.EXPORTS), sorted(set(own) ^ set(wq.EXPORTS))
    assert not [n for n in names if n.startswith("_Z") and "wq_" in n]


def test_plan_tune_is_validated_on_the_host(wq):
    p = wq.Plan(2, 64, 64, 640, 320, 4, 64)
    auto = p.layout.k2_variant
    assert p.layout.k2_kernels in (1, 2) and p.layout.k1_rows in (1, 2, 3, 6)
    for name, code in wq.K2_VARIANTS.items():
        if name in ("auto", "gemm_128x128"):
            continue
        p.tune(0, name)
        assert p.layout.k2_variant == code
        assert p.layout.k2_kernels == (2 if name.startswith(("gemm", "lds_row", "lds_tap")) else 1)
    with pytest.raises(wq.WqError) as e:
        p.tune(0, "gemm_128x128")        # groups of 64: that instance needs 128 and more
    assert e.value.status == 2
    assert p.layout.k2_variant == list(wq.K2_VARIANTS.values())[-1]      # unchanged by the failed call
    with pytest.raises(wq.WqError) as e:
        p.tune(0, 7)                     # not a variant
    assert e.value.status == 1
    with pytest.raises(wq.WqError) as e:
        p.tune(5, "auto")                # 5 tap rows do not divide n = 6
    assert e.value.status == 2
    p.tune(0, "auto")
    assert p.layout.k2_variant == auto
    p.tune(3)
    assert p.layout.k1_rows == 3
    # F(6,3) has no 64x64 fully fused instance; F(2,3) and dense A^T none of the register-tile ones
    with pytest.raises(wq.WqError):
        wq.Plan(1, 12, 12, 64, 64, 6, 32).tune(0, "lds_full_64x64")
    with pytest.raises(wq.WqError):
        wq.Plan(1, 12, 12, 64, 64, 2, 32).tune(0, "fused_32x32")
    assert wq.lib().wq_plan_tune(None, 0, -1) == 1
    # the standard-convolution plan's split override
    d = wq.DirectPlan(1, 8, 8, 64, 64, 32)
    for s in (1, 3, 9):
        assert d.tune(s).layout.splits == s
    with pytest.raises(wq.WqError):
        d.tune(2)
    lin = wq.DirectPlan(8, 1, 1, 256, 64, 32, linear=True)
    assert lin.tune(4).layout.splits == 4
    with pytest.raises(wq.WqError):
        lin.tune(3)


def test_the_plans_own_variant_choice_always_applies(wq):
    """Over a grid of shapes, tile sizes and group sizes (both transform modes): the variant a plan
    picks for itself is a listed one, and forcing exactly that variant is accepted - the selection
    rules never name a kernel instance the shape, group size or matrices rule out."""
    import itertools
    codes = set(wq.K2_VARIANTS.values())
    picked = set()
    shapes = [(1, 8, 8), (1, 20, 36), (2, 64, 64), (2, 128, 128), (8, 96, 96), (32, 14, 14), (32, 56, 56), (4, 33, 17)]
    chans = [(32, 32), (64, 48), (128, 256), (320, 320), (640, 640), (1280, 1280), (960, 320), (256, 1024), (1536, 64)]
    for (N, H, W), (ci, co), m, g in itertools.product(shapes, chans, (2, 4, 6), (32, 64, 128, 256)):
        if ci % g:
            continue
        p = wq.Plan(N, H, W, ci, co, m, g)
        for mode in (0, 1):
            if mode:
                p.set_integer_transforms(mode)
            v = p.layout.k2_variant
            assert v in codes, (N, H, W, ci, co, m, g, mode, v)
            p.tune(0, v)                      # raises WqError if the plan's own choice does not apply
            assert p.layout.k2_variant == v
            picked.add(p.k2_variant_name)
    # the grid reaches every family the rules can pick
    assert {n.rsplit("_", 1)[0] for n in picked} >= {"fused", "gemm", "lds_full", "lds_row", "lds_tap"}


def test_layout_numbers(wq):
    p = wq.Plan(2, 7, 9, 64, 40, 4, 32)
    L = p.layout
    assert (L.n, L.groups, L.TH, L.TW, L.T) == (6, 2, 2, 3, 12)
    assert L.T_pad % 32 == 0 and L.T_pad >= L.T and L.Cout_pad % 32 == 0 and L.Cout_pad >= 40
    assert L.blob_sW_off >= 36 * L.Cout_pad * 64 and L.blob_sW_off % 256 == 0
    assert L.blob_bytes >= L.blob_bias_off + 4 * L.Cout_pad
    assert L.ws_sX_off >= 36 * L.T_pad * 64 and L.ws_bytes >= L.ws_sX_off + 36 * L.T_pad * 2 * 4
    assert L.debug_P_bytes == 36 * 12 * 2 * 40 * 4


def test_argument_errors_are_host_side(wq):
    L = wq.lib()

    def create(*a, mats=(None, None, None)):
        h = ctypes.c_void_p()
        st = L.wq_plan_create(ctypes.byref(h), *a, *mats)
        if st == 0:
            L.wq_plan_destroy(h)
        else:
            assert not h.value
        return st

    assert create(1, 8, 8, 64, 64, 4, 32) == 0
    assert create(1, 8, 8, 64, 64, 3, 32) == 2          # m
    assert create(1, 8, 8, 64, 64, 8, 32) == 2
    assert create(1, 8, 8, 64, 64, 4, 48) == 2          # group size
    assert create(1, 8, 8, 64, 64, 4, 1024) == 2
    assert create(1, 8, 8, 96, 64, 4, 64) == 1          # Cin % g
    assert create(0, 8, 8, 64, 64, 4, 32) == 1
    assert create(1, 8, -1, 64, 64, 4, 32) == 1
    assert L.wq_plan_create(None, 1, 8, 8, 64, 64, 4, 32, None, None, None) == 1
    AT, BT, G = (np.ascontiguousarray(M, np.float32) for M in ct.standard_matrices(4))
    ptr = lambda a: a.ctypes.data
    assert create(1, 8, 8, 64, 64, 4, 32, mats=(ptr(BT), ptr(G), ptr(AT))) == 0
    assert create(1, 8, 8, 64, 64, 4, 32, mats=(ptr(BT), None, ptr(AT))) == 1   # partial set
    bad = BT.copy(); bad[[1, 2]] = bad[[2, 1]]
    assert create(1, 8, 8, 64, 64, 4, 32, mats=(ptr(bad), ptr(G), ptr(AT))) == 3
    bad = G.copy(); bad[3, 1] = np.nan
    assert create(1, 8, 8, 64, 64, 4, 32, mats=(ptr(BT), ptr(bad), ptr(AT))) == 3
    bad = AT.copy(); bad[2, 3] *= 1.01
    assert create(1, 8, 8, 64, 64, 4, 32, mats=(ptr(BT), ptr(G), ptr(bad))) == 3
    # a diagonal rescaling with S_A S_B S_G = I is accepted
    ATs, BTs, Gs = wq.scaled_transforms(4, np.linspace(0.5, 2, 6), np.linspace(2, 0.5, 6))
    assert create(1, 8, 8, 64, 64, 4, 32, mats=(ptr(BTs), ptr(Gs), ptr(ATs))) == 0
    assert L.wq_plan_destroy(None) == 1
    assert L.wq_standard_transforms(5, None, None, None) == 2


def test_forward_errors_before_any_launch(wq):
    L = wq.lib()
    p = wq.Plan(1, 8, 8, 64, 64, 4, 32)
    lay = p.layout
    fake = 0x10000  # never dereferenced: every call below must fail on the host
    big = 1 << 40
    # never prepared
    assert L.wq_conv_forward(p._h, None, fake, fake, big, fake, big, fake) == 4
    assert L.wq_contract_output(p._h, None, fake, big, fake, big, fake) == 4
    # NULL pointers
    assert L.wq_conv_forward(p._h, None, None, fake, big, fake, big, fake) == 1
    assert L.wq_conv_forward(p._h, None, fake, None, big, fake, big, fake) == 1
    assert L.wq_conv_forward(p._h, None, fake, fake, big, None, big, fake) == 1
    assert L.wq_conv_forward(p._h, None, fake, fake, big, fake, big, None) == 1
    assert L.wq_conv_forward(None, None, fake, fake, big, fake, big, fake) == 1
    assert L.wq_input_transform(p._h, None, None, fake, big) == 1
    assert L.wq_weight_prepare(p._h, None, None, None, fake, big) == 1
    # buffers too small
    assert L.wq_conv_forward(p._h, None, fake, fake, lay.blob_bytes - 1, fake, big, fake) == 5
    assert L.wq_conv_forward(p._h, None, fake, fake, big, fake, lay.ws_bytes - 1, fake) == 5
    assert L.wq_input_transform(p._h, None, fake, fake, lay.ws_bytes - 1) == 5
    assert L.wq_weight_prepare(p._h, None, fake, None, fake, lay.blob_bytes - 1) == 5
    assert L.wq_conv_forward_debug(p._h, None, fake, fake, big, fake, big, fake, fake,
                                   lay.debug_P_bytes - 1) == 5
    assert L.wq_conv_forward_debug(p._h, None, fake, fake, big, fake, big, fake, None, big) == 1
    for code in range(7):
        assert wq.status_string(code)
    with pytest.raises(wq.WqError):
        wq.Plan(1, 8, 8, 64, 64, 5, 32)


def test_direct_plan_layout_and_argument_errors(wq):
    p = wq.DirectPlan(2, 7, 9, 64, 40, 32)
    L = p.layout
    assert (L.P, L.groups, L.kstep) == (2 * 7 * 9, 2, 32)
    assert L.Cout_pad % 32 == 0 and L.Cout_pad >= 40
    assert L.blob_sW_off >= 9 * L.Cout_pad * 64 and L.blob_sW_off % 256 == 0
    assert L.blob_bytes >= L.blob_bias_off + 4 * L.Cout_pad
    assert L.ws_sx_off >= L.P * 64 and L.ws_bytes >= L.ws_sx_off + L.P * 2 * 4
    lib = wq.lib()

    def create(*a):
        h = ctypes.c_void_p()
        st = lib.wq_direct_plan_create(ctypes.byref(h), *a)
        if st == 0:
            lib.wq_direct_plan_destroy(h)
        else:
            assert not h.value
        return st

    assert create(1, 8, 8, 64, 64, 32) == 0
    assert create(1, 8, 8, 64, 64, 48) == 2            # group size
    assert create(1, 8, 8, 96, 64, 64) == 1            # Cin % g
    assert create(0, 8, 8, 64, 64, 32) == 1
    assert create(64, 1024, 1024, 64, 64, 32) == 2     # a tensor of 2 GiB or more
    assert lib.wq_direct_plan_create(None, 1, 8, 8, 64, 64, 32) == 1
    # calls without device buffers fail on the host
    h = ctypes.c_void_p()
    assert lib.wq_direct_plan_create(ctypes.byref(h), 1, 8, 8, 64, 64, 32) == 0
    assert lib.wq_direct_quantize(h, None, None, None, 0) == 1
    fake = ctypes.c_void_p(256)
    assert lib.wq_direct_quantize(h, None, fake, fake, 16) == 5          # workspace too small
    assert lib.wq_direct_conv(h, None, fake, 1 << 30, fake, 1 << 30, fake) == 4   # never prepared
    lib.wq_direct_plan_destroy(h)


def test_linear_plan_layout_and_argument_errors(wq):
    p = wq.DirectPlan(50, 1, 1, 128, 40, 64, linear=True)
    L = p.layout
    assert (L.P, L.taps, L.splits, L.groups, L.kstep) == (50, 1, 1, 2, 64)
    assert L.blob_sW_off >= L.Cout_pad * 128 and L.ws_sx_off >= 50 * 128
    lib = wq.lib()
    h = ctypes.c_void_p()
    assert lib.wq_linear_plan_create(ctypes.byref(h), 0, 128, 40, 64) == 1
    assert lib.wq_linear_plan_create(ctypes.byref(h), 8, 100, 40, 64) == 1     # Cin % g
    assert lib.wq_linear_plan_create(ctypes.byref(h), 8, 128, 40, 48) == 2     # group size
    assert lib.wq_linear_plan_create(None, 8, 128, 40, 64) == 1


def test_direct_plan_refuses_more_pixels_than_the_launch_grid_holds(wq):
    lib = wq.lib()
    h = ctypes.c_void_p()
    # 64 pixels per workgroup along the grid's y dimension, which holds 65535 workgroups.
    assert lib.wq_direct_plan_create(ctypes.byref(h), 1, 2048, 2048, 32, 32, 32) == 2   # WQ_ERR_UNSUPPORTED
    assert lib.wq_direct_plan_create(ctypes.byref(h), 1, 2047, 2048, 32, 32, 32) == 0
    lib.wq_direct_plan_destroy(h)


def test_weight_bits_of_direct_and_linear_plans(wq):
    lib = wq.lib()
    h = ctypes.c_void_p()
    assert lib.wq_linear_plan_create_bits(ctypes.byref(h), 8, 64, 8, 32, 5) == 2    # WQ_ERR_UNSUPPORTED
    assert lib.wq_direct_plan_create_bits(ctypes.byref(h), 1, 4, 4, 64, 8, 32, 16) == 2
    p8 = wq.DirectPlan(10, 1, 1, 128, 40, 32, linear=True)
    p4 = wq.DirectPlan(10, 1, 1, 128, 40, 32, linear=True, weight_bits=4)
    assert p8.layout.weight_bits == 8 and p4.layout.weight_bits == 4
    assert p4.layout.blob_sW_off == (64 * 128 // 2 + 255) // 256 * 256       # Cout_pad = 64, two codes per byte
    assert p8.layout.blob_sW_off == 64 * 128
    assert p4.layout.ws_bytes == p8.layout.ws_bytes
    c4 = wq.DirectPlan(1, 5, 5, 64, 16, 32, weight_bits=4)
    assert c4.layout.taps == 9 and c4.layout.blob_sW_off == (9 * 32 * 64 // 2 + 255) // 256 * 256


def test_integer_transform_mode_is_host_state_only(wq):
    """wq_plan_set_integer_transforms: argument checks, the forced two-kernel variant and full tap
    rows, refusal of variants that never hold a Winograd-domain tile, and mode 0 undoing it."""
    assert wq.lib().wq_plan_set_integer_transforms(None, 1) == 1
    p = wq.Plan(2, 64, 64, 640, 320, 4, 64)
    before = (p.layout.k2_variant, p.layout.k1_rows, p.layout.ws_bytes, p.layout.blob_bytes)
    assert wq.lib().wq_plan_set_integer_transforms(p._h, 3) == 1
    for mode in (1, 2):
        p.set_integer_transforms(mode)
        assert p.layout.k2_kernels == 2 and p.layout.k1_rows == 6
        assert p.k2_variant_name.startswith(("gemm", "lds_tap"))
        for name in ("fused_32x16", "lds_row_64x64", "lds_full_64x64"):
            with pytest.raises(wq.WqError) as e:
                p.tune(0, name)
            assert e.value.status == 2
        with pytest.raises(wq.WqError):
            p.tune(3, "auto")                 # the patch scale needs all tap rows in one workgroup
        p.tune(0, "gemm_64x64")
        assert (p.layout.ws_bytes, p.layout.blob_bytes) == before[2:]
    p.set_integer_transforms(0)
    assert (p.layout.k2_variant, p.layout.k1_rows, p.layout.ws_bytes, p.layout.blob_bytes) == before
