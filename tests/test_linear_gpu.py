"""GPU parity of the group-wise quantized linear layer (the one-tap case of the quantized
implicit GEMM) against its oracle, with 8-bit and with 4-bit weight codes (W8A8, W4A8): codes
and fp32 scales bit-exact, fp32 output within 1e-5 of the largest output magnitude."""
import numpy as np
import pytest
import torch

import oracle

pytestmark = pytest.mark.gpu

Y_TOL = 1e-5

CASES = [
    # seed  R    Cin  Cout  g
    (1, 1, 32, 1, 32),
    (2, 37, 64, 19, 32),
    (3, 200, 256, 80, 64),
    (4, 65, 512, 33, 128),
    (5, 128, 512, 64, 256),
    (6, 9, 1024, 16, 512),
    (7, 1000, 320, 320, 32),
    (8, 4096, 1280, 640, 64),     # an attention-sized projection
    (9, 16, 2048, 256, 64),       # few rows: the reduction is split over 16 workgroups per tile
    (10, 77, 768, 768, 32),       # a text-encoder sized layer
]


@pytest.mark.parametrize("bits", [8, 4], ids=["w8", "w4"])
@pytest.mark.parametrize("case", CASES, ids=lambda c: "l%d_%dx%d-%d_g%d" % c)
def test_linear_layers(wq, case, bits):
    seed, R, Cin, Cout, g = case
    rng = np.random.default_rng(3000 + seed)
    x = rng.standard_normal((R, Cin)).astype(np.float32)
    x[:, rng.integers(0, Cin)] *= 20.0
    w = (rng.standard_normal((Cout, Cin)) * 0.05).astype(np.float32)
    b = rng.standard_normal(Cout).astype(np.float32) if seed % 2 else None
    ref = oracle.linear_pipeline(x, w, b, g, weight_bits=bits)

    plan = wq.DirectPlan(R, 1, 1, Cin, Cout, g, linear=True, weight_bits=bits)
    L = plan.layout
    assert L.taps == 1 and L.P == R and L.weight_bits == bits and (Cin // g) % L.splits == 0
    assert L.blob_sW_off >= L.Cout_pad * Cin * bits // 8 and L.blob_sW_off < L.Cout_pad * Cin * bits // 8 + 256
    blob, ws, y = plan.alloc_blob(), plan.alloc_workspace(), plan.alloc_output()
    y.fill_(float("nan"))
    plan.weight_prepare(torch.from_numpy(w).cuda(), None if b is None else torch.from_numpy(b).cuda(), blob)
    plan.forward(torch.from_numpy(x).cuda(), blob, ws, y)
    torch.cuda.synchronize()
    Wq, sW, bias = plan.blob_views(blob)
    xq, sx = plan.workspace_views(ws)
    assert np.array_equal(Wq[0, :Cout].cpu().numpy(), ref["wq"])
    assert np.array_equal(sW[0, :, :Cout].cpu().numpy().view(np.uint32), ref["sw"].view(np.uint32))
    assert bool((Wq[0, Cout:] == 0).all() and (sW[0, :, Cout:] == 0).all() and (bias[Cout:] == 0).all())
    assert np.array_equal(xq.cpu().numpy(), ref["xq"])
    assert np.array_equal(sx.cpu().numpy().view(np.uint32), ref["sx"].view(np.uint32))
    got = y.cpu().numpy().reshape(R, Cout)
    assert np.isfinite(got).all()
    scale = np.abs(ref["y64"]).max()
    err = np.abs(got.astype(np.float64) - ref["y64"]).max()
    assert err <= Y_TOL * scale, f"max|err| {err:.3e} > {Y_TOL * scale:.3e}"
    print(f"linear W{bits}A8 {R}x{Cin}->{Cout} g{g}: max|err|/max|y| = {err / scale:.2e}")
