"""GPU parity of the fully-integer input and output transforms (first and third quantized-stage
equations of Section "Learnable Winograd transform scales") against oracle/fullint.py.

Stage by stage, so that every decision that turns a floating-point value into an integer code is
taken on identical inputs on both sides:
  * stage 1 (integer input transform + group quantizer): codes and scales bit for bit;
  * stage 2 (int8 contraction): the int32 sums bit for bit, the fp32 Winograd-domain result M to
    1e-5 of its largest magnitude (its summation order is free);
  * stage 3 (integer output transform): the oracle's third stage applied to the GPU's own M,
    rounded once to fp32, bit for bit;
  * end to end: within a few steps of the output quantizer of the oracle's pipeline (a code of
    Q(Y / s_Y) may differ where M differs in its last bits).
"""
import numpy as np
import pytest
import torch

import oracle
from oracle import cook_toom as ct
from oracle import fullint
from paper_2412_19867_amd import workloads

pytestmark = pytest.mark.gpu

CASES = [
    # seed N  H   W  Cin Cout m  g   scaled mode variant
    (301, 1, 8, 8, 32, 16, 4, 32, False, 1, None),
    (302, 2, 11, 9, 64, 40, 4, 32, True, 1, None),          # ragged tiles, padded Cout, row-scaled matrices
    (303, 1, 13, 14, 128, 33, 6, 64, True, 1, None),        # F(6,3), odd Cout
    (304, 3, 16, 16, 128, 64, 4, 64, False, 2, None),       # one scale per matrix row
    (305, 1, 12, 12, 256, 32, 6, 128, True, 2, "gemm_64x64"),
    (306, 2, 6, 6, 64, 32, 2, 32, False, 1, None),          # F(2,3): the int8 matrices are exact
    (307, 2, 20, 20, 192, 96, 4, 64, False, 1, "lds_tap_64x64"),
    (308, 2, 20, 20, 192, 96, 4, 64, True, 1, "gemm_32x128"),
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "i%d_F%d_g%d_mode%d" % (c[0], c[6], c[7], c[9]))
def test_integer_transforms_match_the_oracle(wq, case):
    seed, N, H, W, Cin, Cout, m, g, scaled, mode, variant = case
    d = workloads.small_layer(seed, N, H, W, Cin, Cout, m, g, row_scales=scaled)
    check_integer(wq, d, mode, variant)


@pytest.mark.parametrize("idx", [0, 1, 2])
def test_integer_transforms_on_the_headline_layers_at_full_size(wq, idx):
    """The three layer shapes of the SDXL-scale stack, in the variant the plan picks."""
    check_integer(wq, workloads.make_layer_data(workloads.CONFIGS[5][idx]), 1, None)


def check_integer(wq, d, mode, variant):
    lay = d.layer
    N, H, W, Cin, Cout, m, g = lay.N, lay.H, lay.W, lay.Cin, lay.Cout, lay.m, lay.group_size
    if d.u_B is not None:
        AT, BT, G = (M.astype(np.float32) for M in ct.scaled_matrices(m, d.u_B, d.u_G))
    else:
        AT, BT, G = (np.asarray(M, np.float32) for M in ct.standard_matrices(m))
    ms = "matrix" if mode == 1 else "row"
    ref = fullint.fullint_pipeline(d.x, d.w, d.bias, AT, BT, G, m, g, matrix_scales=ms)

    plan = wq.Plan(N, H, W, Cin, Cout, m, g, AT=AT, BT=BT, G=G)
    plan.set_integer_transforms(mode)
    assert plan.layout.k2_kernels == 2 and plan.layout.k1_rows == m + 2
    with pytest.raises(wq.WqError) as e:
        plan.tune(0, "fused_16x16")          # no Winograd-domain tile to quantize in the fused forms
    assert e.value.status == 2
    if variant is not None:
        plan.tune(0, variant)
    L = plan.layout
    blob, ws, y = plan.alloc_blob(), plan.alloc_workspace(), plan.alloc_output()
    y.fill_(float("nan"))
    x = torch.from_numpy(d.x).cuda()
    plan.weight_prepare(torch.from_numpy(d.w).cuda(), torch.from_numpy(d.bias).cuda(), blob)
    P = plan.alloc_debug_P()
    plan.forward_debug(x, blob, ws, y, P)
    torch.cuda.synchronize()
    Xq, sX = plan.workspace_views(ws)
    Xq, sX = Xq[:, :L.T].cpu().numpy(), sX[:, :L.T].cpu().numpy()
    # stage 1
    bad = np.count_nonzero(Xq != ref["Xq"])
    assert bad == 0, f"{bad} of {Xq.size} activation codes differ"
    assert np.array_equal(sX.view(np.uint32), ref["sX"].view(np.uint32))
    # stage 2
    _, Pref = oracle.contract(ref["Xq"], ref["sX"], ref["Wq"], ref["sW"], g, want_P=True)
    assert np.array_equal(P.cpu().numpy(), Pref)
    Mg = plan.product_view(ws).cpu().numpy()                       # [n*n][T][Cout] fp32
    assert np.abs(Mg.astype(np.float64) - ref["Yt"]).max() <= 1e-5 * np.abs(ref["Yt"]).max()
    # stage 3 on the GPU's own M
    st3 = fullint.output_transform_int(Mg.astype(np.float64), AT, d.bias, N, H, W, m, matrix_scales=ms)
    yg = y.cpu().numpy()
    assert np.isfinite(yg).all()
    assert np.array_equal(yg.view(np.uint32), st3["y"].astype(np.float32).view(np.uint32)), \
        f"max diff {np.abs(yg - st3['y']).max():.3e}"
    # end to end: a few output-quantizer steps
    sAA = np.outer(st3["s_qA"], st3["s_qA"])
    step = (np.abs(sAA).max() * st3["s_qY"].max() * np.abs(st3["QA"]).sum(axis=1).max() ** 2)
    assert np.abs(yg.astype(np.float64) - ref["y"]).max() <= 2.0 * step


def test_integer_transforms_switch_off_again(wq):
    """Mode 0 restores the fp32 transforms: same bits as a plan that never had the mode on."""
    d = workloads.small_layer(310, 2, 10, 10, 64, 32, 4, 32)
    lay = d.layer
    x, w, b = (torch.from_numpy(a).cuda() for a in (d.x, d.w, d.bias))
    outs = []
    for toggle in (False, True):
        plan = wq.Plan(lay.N, lay.H, lay.W, lay.Cin, lay.Cout, lay.m, lay.group_size)
        if toggle:
            plan.set_integer_transforms(1)
            plan.set_integer_transforms(0)
        blob, ws, y = plan.alloc_blob(), plan.alloc_workspace(), plan.alloc_output()
        plan.weight_prepare(w, b, blob)
        plan.forward(x, blob, ws, y)
        outs.append((y, plan.k2_variant_name, plan.layout.k1_rows))
    torch.cuda.synchronize()
    assert outs[0][1:] == outs[1][1:]
    assert torch.equal(outs[0][0], outs[1][0])
