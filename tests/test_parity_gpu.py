"""GPU parity: the HIP path (through the C ABI) against the CPU oracle.

Bit-exact on the int8 codes, the fp32 scales (they are defined by one rounded
division) and the int32 group partial sums; fp32 output within 1e-5 of the
layer's largest output magnitude (normwise-max; a per-element relative bound
is ill-posed where the Winograd sums cancel).
"""
import numpy as np
import pytest
import torch

import oracle
from oracle import cook_toom as ct
from paper_2412_19867_amd import workloads

pytestmark = pytest.mark.gpu

Y_TOL = 1e-5


def matrices_for(d, wq):
    lay = d.layer
    if d.u_B is not None:
        lib_mats = wq.scaled_transforms(lay.m, d.u_B, d.u_G)          # what a user would pass
        ora = tuple(M.astype(np.float32) for M in ct.scaled_matrices(lay.m, d.u_B, d.u_G))
        for a, b in zip(lib_mats, ora):
            np.testing.assert_allclose(a, b, rtol=1.2e-7)
        return ora      # both sides get the oracle-built fp32 matrices as *inputs*
    return None


def run_gpu(wq, d, mats, want_P=True, variant=None, k1_rows=0):
    lay = d.layer
    kw = {} if mats is None else dict(AT=mats[0], BT=mats[1], G=mats[2])
    plan = wq.Plan(lay.N, lay.H, lay.W, lay.Cin, lay.Cout, lay.m, lay.group_size, **kw)
    if variant is not None or k1_rows:
        plan.tune(k1_rows, "auto" if variant is None else variant)
        if variant is not None:
            assert plan.k2_variant_name == variant
    L = plan.layout
    blob, ws, y = plan.alloc_blob(), plan.alloc_workspace(), plan.alloc_output()
    y.fill_(float("nan"))
    x = torch.from_numpy(d.x).cuda()
    w = torch.from_numpy(d.w).cuda()
    b = torch.from_numpy(d.bias).cuda() if d.bias is not None else None
    plan.weight_prepare(w, b, blob)
    # the debug entry point launches the same kernel instances as the production one (the dump
    # sits behind a run-time flag inside them); both outputs are checked
    plan.forward(x, blob, ws, y)
    torch.cuda.synchronize()
    P, y_dbg = None, None
    if want_P:
        P = plan.alloc_debug_P()
        y_dbg = plan.alloc_output()
        y_dbg.fill_(float("nan"))
        plan.forward_debug(x, blob, ws, y_dbg, P)
        torch.cuda.synchronize()
    # stage 2 and stage 3 as separate calls (the two-kernel form, whatever the plan defaults to)
    y_split = plan.alloc_output()
    y_split.fill_(float("nan"))
    plan.contract(ws, blob)
    plan.output_transform(ws, blob, y_split)
    torch.cuda.synchronize()
    Wq, sW, bias = plan.blob_views(blob)
    Xq, sX = plan.workspace_views(ws)
    out = dict(M=plan.product_view(ws).cpu().numpy(), y_split=y_split.cpu().numpy(),Wq=Wq[:, :L.Cout].cpu().numpy(), sW=sW[:, :, :L.Cout].cpu().numpy(),
               Xq=Xq[:, :L.T].cpu().numpy(), sX=sX[:, :L.T].cpu().numpy(),
               y=y.cpu().numpy(), P=None if P is None else P.cpu().numpy(),
               y_dbg=None if y_dbg is None else y_dbg.cpu().numpy(), variant=plan.k2_variant_name,
               pad_ok=bool((Wq[:, L.Cout:] == 0).all() and (sW[:, :, L.Cout:] == 0).all()
                           and (Xq[:, L.T:] == 0).all() and (sX[:, L.T:] == 0).all()
                           and (bias[L.Cout:] == 0).all()))
    return out


SEEN_VARIANTS = set()   # kernel instances of stages 2+3 whose int32 sums were compared so far


def check(wq, d, want_P=True, variant=None, k1_rows=0):
    lay = d.layer
    mats = matrices_for(d, wq)
    if mats is None:
        AT, BT, G = ct.standard_matrices(lay.m)
    else:
        AT, BT, G = mats
    ref = oracle.qwino_pipeline(d.x, d.w, d.bias, AT, BT, G, lay.m, lay.group_size, want_P=want_P)
    got = run_gpu(wq, d, mats, want_P=want_P, variant=variant, k1_rows=k1_rows)
    assert got["pad_ok"]
    for key in ("Wq", "Xq"):
        bad = np.count_nonzero(got[key] != ref[key])
        assert bad == 0, f"{lay.name}: {key} differs in {bad} of {ref[key].size} codes"
    for key in ("sW", "sX"):
        assert np.array_equal(got[key].view(np.uint32), ref[key].view(np.uint32)), f"{lay.name}: {key}"
    if want_P:
        assert np.array_equal(got["P"], ref["P"]), f"{lay.name}: int32 partial sums ({got['variant']})"
        SEEN_VARIANTS.add(got["variant"])
    scale = np.abs(ref["y64"]).max()
    worst = 0.0
    m_scale = np.abs(ref["M"]).max()
    m_err = np.abs(got["M"].astype(np.float64) - ref["M"]).max()
    # absolute floor: where the fp32 product of the two scales is sub-normal it carries an
    # error of up to one sub-normal step (2^-149), times |P| <= g*127^2, per group
    m_tol = Y_TOL * m_scale + lay.Cin * 127.0 ** 2 * 2.0 ** -149
    assert m_err <= m_tol, f"{lay.name}: M max|err| {m_err:.3e} > {m_tol:.3e}"
    for key in ("y", "y_dbg", "y_split"):
        if got[key] is None:
            continue
        assert np.isfinite(got[key]).all(), f"{lay.name}: {key} has unwritten or non-finite entries"
        err = np.abs(got[key].astype(np.float64) - ref["y64"]).max()
        assert err <= Y_TOL * scale, f"{lay.name}: {key} max|err| {err:.3e} > {Y_TOL * scale:.3e}"
        worst = max(worst, err / max(scale, 1e-300))
    print(f"{lay.name} [{got['variant']}]: max|err|/max|y| = {worst:.2e}")
    return worst


SMALL = [
    # seed N  H   W  Cin Cout m  g   scaled
    (1, 1, 8, 8, 32, 16, 4, 32, False),
    (2, 2, 7, 10, 64, 48, 4, 32, False),      # ragged tiles, Cout padded
    (3, 1, 13, 6, 64, 33, 6, 32, True),       # odd Cout, learned-scale style matrices
    (4, 3, 9, 9, 128, 64, 4, 64, True),
    (5, 1, 5, 5, 32, 32, 2, 32, False),
    (6, 2, 12, 12, 256, 32, 6, 128, False),
    (7, 1, 6, 20, 512, 16, 4, 256, True),
    (8, 1, 4, 4, 512, 32, 2, 512, False),
    (9, 5, 11, 11, 96, 80, 6, 32, False),     # > 32 tiles: several tile blocks and a tail
    (10, 1, 1, 1, 32, 1, 4, 32, False),       # a single pixel
]


@pytest.mark.parametrize("case", SMALL, ids=lambda c: "s%d_%dx%dx%d_%d-%d_F%d_g%d" % c[:8])
def test_small_layers(wq, case):
    seed, N, H, W, Cin, Cout, m, g, scaled = case
    d = workloads.small_layer(seed, N, H, W, Cin, Cout, m, g, row_scales=scaled)
    check(wq, d)


def test_no_bias_and_repeatability(wq):
    d = workloads.small_layer(21, 2, 9, 7, 64, 32, 4, 32)
    d.bias = None
    check(wq, d)
    a = run_gpu(wq, d, None)
    b = run_gpu(wq, d, None)
    assert np.array_equal(a["y"], b["y"]) and np.array_equal(a["Xq"], b["Xq"])


def test_dense_matrices_take_the_generic_kernels(wq):
    """A valid F(4,3) triple from six finite points has none of the standard
    zeros, so the kernels that skip them cannot be selected."""
    pts = [(0, 1), (1, 1), (-1, 1), (2, 1), (-2, 1), (3, 1)]
    AT, BT, G = ct.cook_toom(pts, [1] * 6, [1] * 6, [1] * 6, 4)
    assert ct.identity_defect(AT, BT, G) == 0
    mats = tuple(ct.to_f64(M).astype(np.float32) for M in (AT, BT, G))
    assert np.count_nonzero(mats[1]) > 24
    d = workloads.small_layer(31, 1, 9, 10, 64, 32, 4, 32)
    lay = d.layer
    ref = oracle.qwino_pipeline(d.x, d.w, d.bias, *mats, lay.m, lay.group_size, want_P=True)
    got = run_gpu(wq, d, mats)
    for key in ("Wq", "Xq", "P"):
        assert np.array_equal(got[key], ref[key]), key
    for key in ("sW", "sX"):
        assert np.array_equal(got[key].view(np.uint32), ref[key].view(np.uint32)), key
    err = np.abs(got["y"].astype(np.float64) - ref["y64"]).max()
    assert err <= Y_TOL * np.abs(ref["y64"]).max()


def test_degenerate_groups(wq):
    """All-zero input, a zero group, a sub-normal group and a group at the
    smallest quantized magnitude."""
    d = workloads.small_layer(41, 1, 8, 8, 64, 32, 4, 32)
    d.x[...] = 0
    check(wq, d)
    d = workloads.small_layer(42, 1, 8, 8, 64, 32, 4, 32)
    d.x[..., :32] = 0                       # one whole group zero everywhere
    d.w[:, 32:] = 0
    check(wq, d)
    d = workloads.small_layer(43, 1, 8, 8, 64, 32, 4, 32)
    d.x[..., :32] *= np.float32(1e-41)      # sub-normal activations in group 0
    d.x[..., 32:] *= np.float32(3e-38)
    check(wq, d)


def test_config1_full(wq):
    check(wq, workloads.make_layer_data(workloads.CONFIGS[1][0]))


FULL = [(c, i) for c in (2, 3, 4, 5) for i in range(len(workloads.CONFIGS[c]))]


@pytest.mark.parametrize("cfg,idx", FULL, ids=lambda v: str(v))
def test_config_layers_full_size(wq, cfg, idx):
    """Every layer of configs 2-5 at full size, in the kernel instances the library picks for it
    (the ones bench.py times), the whole int32 tensor P included (up to 472 MB)."""
    lay = workloads.CONFIGS[cfg][idx]
    check(wq, workloads.make_layer_data(lay))


def test_graph_replay_matches_eager(wq):
    """The forward pass captured in a HIP graph and replayed several times, with
    eager work and synchronisations in between, gives the eager result bit for bit."""
    d = workloads.small_layer(51, 2, 13, 11, 64, 48, 6, 32)
    lay = d.layer
    plan = wq.Plan(lay.N, lay.H, lay.W, lay.Cin, lay.Cout, lay.m, lay.group_size)
    blob, ws = plan.alloc_blob(), plan.alloc_workspace()
    x = torch.from_numpy(d.x).cuda()
    plan.weight_prepare(torch.from_numpy(d.w).cuda(), torch.from_numpy(d.bias).cuda(), blob)
    y_eager = plan.alloc_output()
    plan.forward(x, blob, ws, y_eager)
    torch.cuda.synchronize()
    want = y_eager.clone()
    y = plan.alloc_output()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        plan.forward(x, blob, ws, y)
        side.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            plan.forward(x, blob, ws, y)
    torch.cuda.synchronize()
    for k in range(4):
        y.fill_(float("nan"))
        ws.zero_()                                   # eager work between replays
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            g.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, want), f"replay {k}"
        plan.forward(x, blob, ws, y_eager)           # eager run of the same plan in between
        torch.cuda.synchronize()
        assert torch.equal(y_eager, want)


@pytest.mark.parametrize("idx", [0, 1], ids=["g64", "g256"])
def test_wide_layer_at_reduced_batch(wq, idx):
    """The extra 1280 -> 1280 layer of the benchmark (two-kernel form because of its width;
    groups of 256 accumulate four K-steps per group) with batch 4 instead of 32."""
    lay = workloads.CONFIGS[6][idx]
    import dataclasses
    d = workloads.make_layer_data(lay, N=4)
    d.layer = dataclasses.replace(lay, N=4)
    check(wq, d, want_P=False)


def _random_cases(count, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for k in range(count):
        m = int(rng.choice([2, 4, 6]))
        g = int(rng.choice([32, 32, 64, 128]))
        Cin = g * int(rng.integers(1, 5))
        cases.append((1000 + k, int(rng.integers(1, 4)), int(rng.integers(1, 20)), int(rng.integers(1, 20)),
                      Cin, int(rng.integers(1, 100)), m, g, bool(rng.integers(0, 2))))
    return cases


@pytest.mark.parametrize("case", _random_cases(24, 2024), ids=lambda c: "r%d_%dx%dx%d_%d-%d_F%d_g%d" % c[:8])
def test_random_small_shapes(wq, case):
    """Seeded random shapes: image sizes from 1 to 19, any Cout, one to four groups."""
    seed, N, H, W, Cin, Cout, m, g, scaled = case
    d = workloads.small_layer(seed, N, H, W, Cin, Cout, m, g, row_scales=scaled)
    check(wq, d)


def test_largest_supported_input(wq):
    """An input of exactly 1 GiB (the plan's limit) with a 1 GiB int8 operand tensor: every
    32-bit offset of the transform and contraction kernels is exercised near its top."""
    d = workloads.small_layer(77, 8, 512, 512, 128, 32, 2, 32)
    assert d.x.nbytes == 1 << 30
    lib = wq.lib()
    import ctypes
    h = ctypes.c_void_p()
    assert lib.wq_plan_create(ctypes.byref(h), 8, 512, 513, 128, 32, 2, 32, None, None, None) == 2   # one column more
    check(wq, d, want_P=False)


def test_two_kernel_form_with_more_than_65535_tiles(wq):
    """The GEMM + output-transform kernels with 100352 tiles, more than a grid dimension other
    than x holds."""
    d = workloads.small_layer(79, 32, 112, 112, 128, 32, 2, 128)
    check(wq, d, want_P=False, variant="gemm_64x64")


def test_two_plans_on_two_streams_at_once(wq):
    """The library keeps no state outside plans, blobs and workspaces: two layers enqueued on two
    streams at the same time, many times over, give the results of running them one by one."""
    cases = [workloads.small_layer(91, 2, 13, 11, 64, 48, 6, 32), workloads.small_layer(92, 1, 16, 16, 256, 64, 4, 64)]
    ctx = []
    for d in cases:
        lay = d.layer
        plan = wq.Plan(lay.N, lay.H, lay.W, lay.Cin, lay.Cout, lay.m, lay.group_size)
        blob, ws, y = plan.alloc_blob(), plan.alloc_workspace(), plan.alloc_output()
        x = torch.from_numpy(d.x).cuda()
        plan.weight_prepare(torch.from_numpy(d.w).cuda(), torch.from_numpy(d.bias).cuda(), blob)
        plan.forward(x, blob, ws, y)
        torch.cuda.synchronize()
        ctx.append(dict(plan=plan, blob=blob, ws=ws, y=y, x=x, want=y.clone(), stream=torch.cuda.Stream()))
    for rep in range(20):
        for c in ctx:
            c["y"].fill_(float("nan"))
        torch.cuda.synchronize()
        for c in ctx:
            with torch.cuda.stream(c["stream"]):
                c["plan"].forward(c["x"], c["blob"], c["ws"], c["y"])
        torch.cuda.synchronize()
        for c in ctx:
            assert torch.equal(c["y"], c["want"]), f"repetition {rep}"


# ---- every kernel instance of stages 2+3, forced through wq_plan_tune ----
VARIANT_SHAPES = [
    # seed N  H   W  Cin Cout m  g   scaled
    (201, 2, 20, 20, 128, 96, 4, 64, False),    # 50 tiles -> 64 padded, Cout padded
    (202, 1, 37, 23, 64, 80, 4, 32, True),      # ragged both ways, groups of 32 (K-step 32)
    (203, 2, 30, 30, 64, 64, 6, 32, False),     # F(6,3)
    (204, 1, 16, 16, 512, 40, 4, 128, False),   # several K-steps per group
    (205, 3, 10, 10, 640, 48, 4, 64, True),     # more than 8 groups: fp64 chunk totals
    (206, 2, 12, 12, 64, 32, 2, 32, False),     # F(2,3)
    (207, 1, 24, 24, 768, 70, 6, 32, True),     # F(6,3), 24 groups, odd channel count
]
ALL_VARIANTS = ["fused_16x16", "fused_ksplit", "fused_32x16", "fused_32x32", "gemm_64x64", "gemm_32x128",
                "gemm_128x128", "lds_full_64x64", "lds_full_32x64", "lds_full_32x32", "lds_row_64x64", "lds_row_32x64",
                "lds_tap_64x64", "lds_tap_128x128"]


@pytest.mark.parametrize("variant", ALL_VARIANTS)
def test_every_k2_variant(wq, variant):
    """Each kernel instance on every shape it applies to: int8 codes, scales and the int32 sums
    dumped by THAT instance bit-exact, outputs within the bound."""
    ran = 0
    for case in VARIANT_SHAPES:
        seed, N, H, W, Cin, Cout, m, g, scaled = case
        d = workloads.small_layer(seed, N, H, W, Cin, Cout, m, g, row_scales=scaled)
        try:
            check(wq, d, variant=variant)
            ran += 1
        except wq.WqError as e:
            assert e.status == 2, e      # WQ_ERR_UNSUPPORTED: the variant does not apply to this shape
    assert ran >= 1, f"{variant} applied to none of the shapes"
    assert variant in SEEN_VARIANTS


@pytest.mark.parametrize("rows", [1, 2, 3, 6])
def test_every_k1_row_split(wq, rows):
    d = workloads.small_layer(211, 2, 21, 17, 96, 48, 4, 32)
    check(wq, d, k1_rows=rows)


def test_debug_slab_equals_the_full_dump(wq):
    d = workloads.small_layer(221, 2, 19, 14, 128, 72, 4, 64)
    lay = d.layer
    for variant in ("fused_32x16", "gemm_64x64", "lds_full_64x64", "lds_row_64x64"):
        plan = wq.Plan(lay.N, lay.H, lay.W, lay.Cin, lay.Cout, lay.m, lay.group_size).tune(0, variant)
        blob, ws, y = plan.alloc_blob(), plan.alloc_workspace(), plan.alloc_output()
        x = torch.from_numpy(d.x).cuda()
        plan.weight_prepare(torch.from_numpy(d.w).cuda(), torch.from_numpy(d.bias).cuda(), blob)
        P = plan.alloc_debug_P()
        plan.forward_debug(x, blob, ws, y, P)
        full = P.cpu().numpy()
        L = plan.layout
        for tap0, ntaps, tile0, ntiles in ((0, 1, 0, 1), (5, 7, 13, 20), (35, 1, L.T - 1, 1), (0, 36, 0, L.T)):
            slab = plan.forward_debug_slab(x, blob, ws, y, tap0, ntaps, tile0, ntiles).cpu().numpy()
            assert np.array_equal(slab, full[tap0:tap0 + ntaps, tile0:tile0 + ntiles]), (variant, tap0, tile0)
        with pytest.raises(wq.WqError):
            plan.forward_debug_slab(x, blob, ws, y, 30, 7, 0, 1)          # taps past the end
        with pytest.raises(wq.WqError):
            plan.forward_debug_slab(x, blob, ws, y, 0, 1, L.T, 1)         # tiles past the end


def test_adversarially_rounded_column_scales_take_the_dense_output_transform(wq):
    """A^T whose paired columns agree only to several ulps (entries nudged after the scaling):
    the library must use every entry as given, like the oracle does."""
    d = workloads.small_layer(231, 1, 13, 13, 64, 32, 6, 32, row_scales=True)
    lay = d.layer
    AT, BT, G = (M.astype(np.float32) for M in ct.scaled_matrices(lay.m, d.u_B, d.u_G))
    AT = AT.copy()
    bits = AT.view(np.uint32)
    nudge = np.zeros(AT.shape, np.uint32)
    nudge[1::2, 2::2] = 3          # three ulps on every other entry of the even columns
    nudge[0::2, 1::2] = 2
    bits += nudge * (AT != 0)      # the exact zeros of the first and last columns stay
    ref = oracle.qwino_pipeline(d.x, d.w, d.bias, AT, BT, G, lay.m, lay.group_size, want_P=False)
    got = run_gpu(wq, d, (AT, BT, G), want_P=False)
    scale = np.abs(ref["y64"]).max()
    for key in ("y", "y_split"):
        err = np.abs(got[key].astype(np.float64) - ref["y64"]).max()
        assert err <= Y_TOL * scale, (key, err / scale)
