"""Pins for the oracle's transform-matrix construction (CPU only).

The construction (Vandermonde matrix of the homogeneous points, diagonal
scales) is checked against every matrix the paper prints for F(4,3) and
F(6,3), against the exact 1-D minimal-filtering identity, and against the
scaling condition S_A S_B S_G = I.
"""
from fractions import Fraction as Fr

import numpy as np
import pytest

from oracle import cook_toom as ct
from conftest import golden_path


def parse_golden(name):
    out, cur = {}, None
    for line in open(golden_path(name)):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        if line.startswith("["):
            cur = line.strip("[]")
            out[cur] = []
        else:
            out[cur].append([Fr(tok) for tok in line.split()])
    return out


def built(m):
    st = ct.STANDARD[m]
    n = m + 2
    AT, BT, G = ct.standard_fractions(m)
    return {
        "V_nm": ct.vandermonde(st["points"], m),
        "VinvT": ct.transpose(ct.inverse(ct.vandermonde(st["points"], n))),
        "V_nr": ct.vandermonde(st["points"], 3),
        "AT": AT, "BT": BT, "G": G,
    }


def diff(printed, constructed):
    bad = {}
    for key, mat in printed.items():
        ref = constructed[key]
        assert len(mat) == len(ref) and all(len(a) == len(b) for a, b in zip(mat, ref)), key
        for i, row in enumerate(mat):
            for j, v in enumerate(row):
                if v != ref[i][j]:
                    bad[(key, i, j)] = (v, ref[i][j])
    return bad


def test_f43_matches_every_printed_matrix():
    assert diff(parse_golden("f43_printed.txt"), built(4)) == {}


def test_f63_matches_print_except_known_slips():
    # The print's slips, found by rebuilding from the printed points: each is
    # contradicted by another printed matrix (B^T = S_B V^{-T} and the last
    # Vandermonde row (0,...,0,1) of the point at infinity).
    known = {
        ("V_nm", 1, 5): (Fr(0), Fr(1)),
        ("VinvT", 2, 4): (Fr(-17, 18), Fr(17, 18)),
        ("VinvT", 7, 1): (Fr(-1, 4), Fr(-1)),
        ("AT", 5, 7): (Fr(0), Fr(1)),
    }
    assert diff(parse_golden("f63_printed.txt"), built(6)) == known


@pytest.mark.parametrize("m", [2, 4, 6])
def test_identity_and_scaling_condition_exact(m):
    st = ct.STANDARD[m]
    AT, BT, G = ct.standard_fractions(m)
    assert ct.identity_defect(AT, BT, G) == 0
    for a, b, g in zip(st["S_A"], st["S_B"], st["S_G"]):
        assert Fr(a) * Fr(b) * Fr(g) == 1


def test_f23_is_the_familiar_small_integer_form():
    AT, BT, G = ct.standard_fractions(2)
    assert BT == [[1, 0, -1, 0], [0, 1, 1, 0], [0, -1, 1, 0], [0, 1, 0, -1]]
    assert AT == [[1, 1, 1, 0], [0, 1, -1, -1]]
    assert G == [[1, 0, 0], [Fr(1, 2)] * 3, [Fr(1, 2), Fr(-1, 2), Fr(1, 2)], [0, 0, 1]]


def test_printed_f63_BT_and_G_satisfy_identity_with_corrected_AT():
    pr = parse_golden("f63_printed.txt")
    AT = [list(r) for r in pr["AT"]]
    assert ct.identity_defect(AT, pr["BT"], pr["G"]) != 0      # the slip is visible
    AT[5][7] = Fr(1)
    assert ct.identity_defect(AT, pr["BT"], pr["G"]) == 0


def test_identity_detects_a_wrong_matrix():
    AT, BT, G = ct.standard_fractions(4)
    BT2 = [list(r) for r in BT]
    BT2[1][2], BT2[2][1] = BT2[2][1], BT2[1][2]     # a transposed pair
    assert ct.identity_defect(AT, BT2, G) != 0
    G2 = [list(r) for r in G]
    G2[3][1] = -G2[3][1]                             # a wrong sign
    assert ct.identity_defect(AT, BT, G2) != 0


def test_learned_scales_rows_multiply_to_one_and_build_valid_matrices():
    rows = [[float(t) for t in l.split()] for l in open(golden_path("learned_scales_f63.txt"))
            if l.strip() and not l.startswith("#")]
    S_A, S_B, S_G = (np.array(c) for c in zip(*rows))
    assert len(rows) == 8
    # three printed digits => product within a percent of one
    assert np.all(np.abs(S_A * S_B * S_G - 1.0) < 1e-2)
    AT, BT, G = ct.matrices_from_scales(6, S_B, S_G)
    # float64-rounded matrices satisfy the identity to rounding
    n, m = 8, 6
    worst = 0.0
    for a in range(m):
        for k in range(3):
            for l in range(n):
                s = sum(AT[a, i] * G[i, k] * BT[i, l] for i in range(n))
                worst = max(worst, abs(s - (1.0 if l == a + k else 0.0)))
    assert worst < 1e-12
    # recomputed S_A agrees with the printed S_A column to its digits
    S_A_re = 1.0 / (S_B * S_G)
    assert np.all(np.abs(S_A_re - S_A) <= 0.012 * np.abs(S_A))


def test_scaled_matrices_are_row_and_column_scalings_of_standard():
    rng = np.random.default_rng(7)
    for m in (4, 6):
        n = m + 2
        u_B, u_G = rng.uniform(0.5, 2, n), rng.uniform(0.5, 2, n)
        AT0, BT0, G0 = ct.standard_matrices(m)
        AT, BT, G = ct.scaled_matrices(m, u_B, u_G)
        np.testing.assert_allclose(BT, u_B[:, None] * BT0, rtol=1e-15)
        np.testing.assert_allclose(G, u_G[:, None] * G0, rtol=1e-15)
        np.testing.assert_allclose(AT, AT0 / (u_B * u_G)[None, :], rtol=1e-15)
