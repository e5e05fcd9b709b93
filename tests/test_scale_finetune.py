"""The scale fine-tuning loop (the paper's algorithm box) on synthetic layers.

Its differentiable forward pass is checked against the fully-integer oracle; the loop itself
against what the paper fixes: the SQNR objective rises, the three diagonal scale matrices still
multiply to the identity, and the learned pattern has the shape of the tabulated one (the
columns of A^T that belong to the points +-2 get the smallest scales)."""
import numpy as np
import pytest
import torch

import oracle
from oracle import cook_toom as ct
from oracle import fullint
from paper_2412_19867_amd import scale_finetune as sf

from conftest import golden_path


@pytest.mark.parametrize("m", [2, 4, 6])
def test_vandermonde_factors_rebuild_the_standard_matrices(m):
    VA, VB, VG = sf.vandermonde_factors(m)
    AT, BT, G = sf.WinogradScales.standard(m).matrices((VA, VB, VG))
    AT0, BT0, G0 = ct.standard_matrices(m)
    np.testing.assert_allclose(AT.detach().numpy(), AT0, rtol=1e-14, atol=1e-15)
    np.testing.assert_allclose(BT.detach().numpy(), BT0, rtol=1e-14, atol=1e-15)
    np.testing.assert_allclose(G.detach().numpy(), G0, rtol=1e-14, atol=1e-15)


@pytest.mark.parametrize("m,matrix_scales", [(4, "matrix"), (6, "matrix"), (6, "row"), (2, "matrix")])
def test_forward_pass_equals_the_fully_integer_oracle(m, matrix_scales):
    gen = torch.Generator().manual_seed(m)
    x = torch.randn(2, 64, 13, 11, generator=gen, dtype=torch.float64)
    w = torch.randn(24, 64, 3, 3, generator=gen, dtype=torch.float64) * 0.06
    y = sf.quantized_winograd_conv(x, w, sf.WinogradScales.standard(m), sf.vandermonde_factors(m), 32,
                                   matrix_scales).detach().numpy().transpose(0, 2, 3, 1)
    ref = fullint.fullint_pipeline(x.permute(0, 2, 3, 1).numpy().astype(np.float32), w.numpy().astype(np.float32),
                                   None, *ct.standard_matrices(m), m, 32, matrix_scales)["y"]
    if m == 2:
        # every F(2,3) intermediate is a small integer times a scale: exact rounding ties are common
        # and fall differently in the oracle's fp32 quantizer and in fp64 here
        assert fullint.sqnr_db(ref, y) > 40.0
    else:
        assert np.abs(y - ref).max() <= 1e-6 * np.abs(ref).max()


def test_learned_scales_of_the_paper_score_the_same_in_both_implementations():
    rows = [[float(t) for t in l.split()] for l in open(golden_path("learned_scales_f63.txt")) if not l.startswith("#")]
    sc = sf.WinogradScales.standard(6)
    with torch.no_grad():
        sc.log_sb.copy_(torch.tensor([abs(r[1]) for r in rows], dtype=torch.float64).log())
        sc.log_sg.copy_(torch.tensor([abs(r[2]) for r in rows], dtype=torch.float64).log())
    sc.sign_sb = torch.tensor([np.sign(r[1]) for r in rows], dtype=torch.float64)
    sc.sign_sg = torch.tensor([np.sign(r[2]) for r in rows], dtype=torch.float64)
    gen = torch.Generator().manual_seed(3)
    x = torch.randn(1, 64, 24, 24, generator=gen, dtype=torch.float64)
    w = torch.randn(32, 64, 3, 3, generator=gen, dtype=torch.float64) * (2 / (9 * 64)) ** 0.5
    y = sf.quantized_winograd_conv(x, w, sc, sf.vandermonde_factors(6), 32).detach()
    y_ref = torch.nn.functional.conv2d(x, w, padding=1)
    mats = ct.matrices_from_scales(6, [r[1] for r in rows], [r[2] for r in rows])
    o = fullint.fullint_pipeline(x.permute(0, 2, 3, 1).numpy().astype(np.float32), w.numpy().astype(np.float32),
                                 None, *mats, 6, 32)["y"]
    s_t = float(sf.sqnr_db(y_ref, y))
    s_o = fullint.sqnr_db(y_ref.permute(0, 2, 3, 1).numpy(), o)
    assert abs(s_t - s_o) < 0.05 and s_t > 0.0


@pytest.mark.parametrize("m", [4, 6])
def test_finetuning_raises_the_sqnr_and_keeps_the_scaling_condition(m):
    gen = torch.Generator().manual_seed(0)
    layers = [torch.randn(co, ci, 3, 3, generator=gen, dtype=torch.float64) * (2 / (9 * ci)) ** 0.5
              for co, ci in ((32, 64), (64, 32), (48, 64))]
    log = []
    sc = sf.finetune_scales(layers, m, 32, epochs=2, batches=25, K=2, log=log, size=24, seed=1)
    first, last = float(np.mean(log[:5])), float(np.mean(log[-5:]))
    print(f"F({m},3): SQNR {first:.1f} dB -> {last:.1f} dB over {len(log)} steps")
    assert last > first + 8.0
    S_A, S_B, S_G = (t.detach() for t in sc.diagonals())
    np.testing.assert_allclose((S_A * S_B * S_G).numpy(), 1.0, rtol=1e-12)
    # a valid F(m,3) triple for the library: the exact 1-D identity holds for the learned scales
    AT, BT, G = (t.detach().numpy() for t in sc.matrices(sf.vandermonde_factors(m)))
    n = m + 2
    ident = np.einsum("ai,ik,il->akl", AT, G, BT)
    want = np.zeros((m, 3, n))
    for a in range(m):
        for k in range(3):
            want[a, k, a + k] = 1.0
    np.testing.assert_allclose(ident, want, atol=1e-9)
    # the learned pattern: the points +-2 (and only they) get a much smaller output scale
    sa = S_A.abs().numpy()
    assert sa[3] < 0.25 * np.median(sa) and sa[4] < 0.25 * np.median(sa)
    # held-out layer and noise: the gain carries over (one shared set of scales for all layers)
    w_new = torch.randn(40, 32, 3, 3, generator=gen, dtype=torch.float64) * (2 / (9 * 32)) ** 0.5
    x_new = torch.rand(1, 32, 18, 18, generator=gen, dtype=torch.float64) * 2 - 1          # uniform noise
    y_ref = torch.nn.functional.conv2d(x_new, w_new, padding=1)
    fac = sf.vandermonde_factors(m)
    before = float(sf.sqnr_db(y_ref, sf.quantized_winograd_conv(x_new, w_new, sf.WinogradScales.standard(m), fac, 32).detach()))
    after = float(sf.sqnr_db(y_ref, sf.quantized_winograd_conv(x_new, w_new, sc, fac, 32).detach()))
    assert after > before + 8.0
