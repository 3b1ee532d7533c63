"""Pins for the step-by-step RNS-Winograd reference.

Every check compares against something other than the code under test: the
matrices and worked numbers the paper prints (tests/golden/paper_matrices.txt
and the values quoted inline below, each with its place in the paper), exact
identities that hold for all inputs, and the direct-convolution definition.
"""
from fractions import Fraction
from math import gcd

import numpy as np
import pytest

import synth_inputs as si
from oracle import rnswino as rw
from oracle import direct_conv2d


# ---- section 3: residue number system -----------------------------------

def test_rns_worked_example_48():
    assert rw.to_rns(48, (7, 9)) == [6, 3]                       # section 3, RNS(7,9)
    assert rw.mrc([6, 3], [7, 9], signed=False) == 48            # x = 6 + 7*[((3-6)/7) mod 9]
    assert ((3 - 6) * rw.modinv(7, 9)) % 9 == 6


def test_rns_arithmetic_example():
    x, y, mod = [6, 3], [5, 10], (7, 9)                           # section 3; the operand 10 is unreduced mod 9
    assert [(a + b) % p for a, b, p in zip(x, y, mod)] == [4, 4]
    assert [(a - b) % p for a, b, p in zip(x, y, mod)] == [1, 2]
    assert [(a * b) % p for a, b, p in zip(x, y, mod)] == [2, 3]
    # and they are the residues of the integer results (48 and 19 -> 67=4 mod 63, 29, 912)
    for op in (lambda a, b: a + b, lambda a, b: a - b, lambda a, b: a * b):
        v = op(48, rw.mrc(y, list(mod), signed=False))
        got = [op(a, b) % p for a, b, p in zip(x, y, mod)]
        assert got == rw.to_rns(v, mod)


@pytest.mark.parametrize("moduli,rng", [((253, 251, 247), 7842620), ((251, 241, 239), 7228674),
                                        ((4001, 4331), 8664165)])
def test_dynamic_ranges_quoted_in_the_paper(moduli, rng):
    assert rw.dynamic_range(moduli) == rng                        # sections 5 and 8


@pytest.mark.parametrize("moduli", [(251, 241, 239), (251, 241, 239, 233), (65521, 65519), (253, 251, 247), (7, 9)])
def test_mrc_round_trip_signed(moduli):
    R = rw.dynamic_range(moduli)
    vals = np.array([0, 1, -1, R, -R, R - 1, -(R - 1), 12345 % R, -(54321 % R)], dtype=np.int64)
    rnd = (si.splitmix64(77, 500).astype(np.int64)) % (2 * R + 1) - R
    vals = np.concatenate([vals, rnd])
    back = rw.mrc([vals % p for p in moduli], list(moduli), signed=True)
    assert np.array_equal(back, vals)
    # residues need not be canonical
    back2 = rw.mrc([rw.sym(vals, p) for p in moduli], list(moduli), signed=True)
    assert np.array_equal(back2, vals)


def test_mrc_wraps_outside_the_dynamic_range():
    y = 7372800                                                   # all -128, C=50, 3x3: above 7228674
    assert rw.mrc(rw.to_rns(y, (251, 241, 239)), [251, 241, 239]) == y - 251 * 241 * 239 == -7084549


# ---- sections 4-5: transform matrices ------------------------------------

@pytest.mark.parametrize("algo,m,r", [("F2_3", 2, 3), ("F4_3", 4, 3), ("F10_3", 10, 3)])
def test_rational_matrices_equal_the_printed_ones(paper_matrices, algo, m, r):
    AT, G, BT = rw.matrices_Q(m, r)
    assert AT == paper_matrices[(algo, "AT", "Q")]
    assert G == paper_matrices[(algo, "G", "Q")]
    assert BT == paper_matrices[(algo, "BT", "Q")]


def test_g_prime_scalings(paper_matrices):
    _, G4, _ = rw.matrices_Q(4, 3)
    _, G10, _ = rw.matrices_Q(10, 3)
    assert [[v * 24 for v in row] for row in G4] == paper_matrices[("F4_3", "Gprime", "Q")]
    assert [[v * 3628800 for v in row] for row in G10] == paper_matrices[("F10_3", "Gprime", "Q")]
    assert 3628800 == 2**8 * 3**4 * 5**2 * 7                       # section 5


@pytest.mark.parametrize("p", [253, 251, 247, 4001, 4331])
def test_modular_matrices_equal_the_printed_ones(paper_matrices, p):
    AT, G, BT = rw.matrices_mod(10, 3, p)
    for got, which in ((AT, "AT"), (G, "G"), (BT, "BT")):
        want = np.array([[int(v) for v in row] for row in paper_matrices[("F10_3", which, str(p))]])
        assert np.array_equal(got, want), (which, p)
        assert np.abs(got).max() <= (p - 1) // 2


def test_inverse_of_14400():
    assert [rw.sym(rw.modinv(14400, p), p) for p in (253, 251, 247)] == [12, 27, -10]   # section 5


def test_magnifications_quoted_in_section_4():
    def mag(Mx):
        return float(sum(v * v for row in Mx for v in row)) / len(Mx)
    _, G2, BT2 = rw.matrices_Q(2, 3)
    _, G4, BT4 = rw.matrices_Q(4, 3)
    G2p = [[v * 2 for v in row] for row in G2]
    G4p = [[v * 24 for v in row] for row in G4]
    assert mag(G2p) == 3.5 and mag(BT2) == 2.0
    assert mag(G4p) == 125.0 and round(mag(BT4), 1) == 28.7


@pytest.mark.parametrize("m,r", [(2, 3), (4, 3), (6, 3), (8, 3), (10, 3), (14, 3), (8, 5), (12, 5), (3, 2)])
def test_bilinear_tensor_identity_over_Q(m, r):
    # sum_j A^T[i][j] G[j][k] B^T[j][l] = [l == i + k]  <=>  y_i = sum_k d_{i+k} g_k for ALL d, g
    AT, G, BT = rw.matrices_Q(m, r)
    t = m + r - 1
    for i in range(m):
        for k in range(r):
            for l in range(t):
                s = sum(AT[i][j] * G[j][k] * BT[j][l] for j in range(t))
                assert s == (1 if l == i + k else 0)


ALL_MODULI = (251, 241, 239, 233, 65521, 65519)


@pytest.mark.parametrize("m,r", [(8, 3), (14, 3), (12, 5)])
@pytest.mark.parametrize("p", ALL_MODULI)
def test_bilinear_tensor_identity_mod_p(m, r, p):
    AT, G, BT = rw.matrices_mod(m, r, p)
    t = m + r - 1
    ten = np.einsum("ij,jk,jl->ikl", AT % p, G % p, BT % p) % p
    want = np.zeros((m, r, t), dtype=np.int64)
    for i in range(m):
        for k in range(r):
            want[i, k, i + k] = 1
    assert np.array_equal(ten, want)


@pytest.mark.parametrize("m,r", [(2, 3), (4, 3), (8, 3), (10, 3), (14, 3), (12, 5)])
def test_2d_winograd_identity_mod_p_on_random_tiles(m, r):
    t = m + r - 1
    d = si.int8_tensor(41 + m, (t, t)).astype(np.int64)
    g = si.int8_tensor(43 + m, (r, r)).astype(np.int64)
    direct = np.array([[sum(d[u + i, v + j] * g[i, j] for i in range(r) for j in range(r))
                        for v in range(m)] for u in range(m)])
    for p in ALL_MODULI:
        AT, G, BT = rw.matrices_mod(m, r, p)
        y = (AT @ (((G @ g @ G.T) % p) * ((BT @ d @ BT.T) % p) % p) @ AT.T) % p
        assert np.array_equal(y, direct % p), (m, r, p)


def test_invertibility_rule():
    rw.check_moduli(10, 3, (253, 251, 247))                       # the paper's running example is valid
    rw.check_moduli(14, 3, (251, 241, 239))
    rw.check_moduli(12, 5, (251, 241, 239, 233))
    rw.check_moduli(14, 3, (65521, 65519))
    rw.check_moduli(10, 3, (4001, 4331))                          # 4331 = 61*71: composite but fine
    with pytest.raises(ValueError):
        rw.check_moduli(14, 3, (253, 251, 247))                   # 16 points: differences 11 and 13 appear
    with pytest.raises(ValueError):
        rw.check_moduli(12, 5, (251, 247))
    with pytest.raises(ValueError):
        rw.check_moduli(8, 3, (251, 241, 241))
    with pytest.raises(ValueError):
        rw.check_moduli(8, 3, (249, 243))                         # share the factor 3


def test_points_pattern():
    assert rw.interpolation_points(4) == [0, 1, -1, rw.INF]
    assert rw.interpolation_points(6) == [0, 1, -1, 2, -2, rw.INF]
    assert rw.interpolation_points(12)[:-1] == [0, 1, -1, 2, -2, 3, -3, 4, -4, 5, -5]
    assert rw.interpolation_points(16)[-3:] == [7, -7, rw.INF]


TABLE2 = {  # section 7, table "Complexity reduction": (m, r) -> (2 moduli, 3 moduli)
    (2, 3): (1.125, 0.75), (4, 3): (2.00, 1.33), (6, 3): (2.53, 1.69), (8, 3): (2.88, 1.92), (8, 5): (5.56, 3.70),
    (9, 3): (3.01, 2.01), (9, 5): (5.99, 3.99), (10, 3): (3.13, 2.08), (10, 5): (6.38, 4.25), (11, 3): (3.22, 2.14),
    (11, 5): (6.72, 4.48), (12, 3): (3.31, 2.20), (12, 5): (7.03, 4.69), (14, 3): (3.45, 2.30)}


def test_arithmetic_reduction_table():
    # the table prints two decimals, some rounded and some truncated (2.1479 appears as 2.14)
    for (m, r), (two, three) in TABLE2.items():
        assert abs(rw.arithmetic_reduction(m, r, 2) - two) < 0.01
        assert abs(rw.arithmetic_reduction(m, r, 3) - three) < 0.01


# ---- section 6: the layer algorithm equals the definition ---------------------

LAYER_CASES = [
    # N, C, K, H, W, r, m, pad, moduli
    (1, 3, 2, 8, 8, 3, 2, 1, (251, 241, 239)),
    (1, 4, 3, 16, 16, 3, 8, 1, (251, 241, 239)),
    (2, 5, 4, 13, 17, 3, 8, 1, (251, 241, 239, 233)),        # ragged tiles, batch
    (1, 6, 5, 12, 12, 5, 12, 2, (251, 241, 239, 233)),
    (1, 3, 2, 30, 30, 5, 12, 2, (251, 241, 239, 233)),       # ragged 5x5
    (1, 7, 3, 28, 14, 3, 14, 1, (65521, 65519)),
    (1, 4, 4, 12, 12, 3, 10, 1, (253, 251, 247)),            # the paper's running example set
    (1, 4, 4, 10, 10, 3, 8, 0, (251, 241, 239)),             # no padding
    (1, 5, 3, 12, 12, 3, 10, 1, (4001, 4331)),
]


@pytest.mark.parametrize("case", LAYER_CASES)
def test_pipeline_equals_direct_convolution(case):
    N, C, K, H, W, r, m, pad, moduli = case
    x = si.int8_tensor(51, (N, C, H, W))
    w = si.int8_tensor(52, (K, C, r, r))
    y, st = rw.conv2d(x, w, m, pad, moduli, return_stages=True)
    assert np.array_equal(y, direct_conv2d(x, w, pad).astype(np.int64))
    for i, p in enumerate(moduli):
        for name in ("U", "V", "O", "Y"):
            assert np.abs(st[name][i]).max() <= (p - 1) // 2


def test_extreme_values_within_range():
    # all -128 against all -128 / +127: largest magnitudes the bound 2^14 r^2 C allows
    C, moduli = 40, (251, 241, 239)                               # 2^14*9*40 = 5 898 240 <= 7 228 674
    x = np.full((1, C, 8, 8), -128, dtype=np.int8)
    for wv in (-128, 127):
        w = np.full((2, C, 3, 3), wv, dtype=np.int8)
        assert np.array_equal(rw.conv2d(x, w, 8, 1, moduli), direct_conv2d(x, w, 1).astype(np.int64))


def test_out_of_range_result_is_the_residue_of_the_true_one():
    C, moduli = 50, (251, 241, 239)                               # 2^14*9*50 = 7 372 800 > 7 228 674
    x = np.full((1, C, 8, 8), -128, dtype=np.int8)
    w = np.full((1, C, 3, 3), -128, dtype=np.int8)
    y = rw.conv2d(x, w, 8, 1, moduli)
    P = 251 * 241 * 239
    ref = direct_conv2d(x, w, 1).astype(np.int64)
    assert np.array_equal(y, rw.sym(ref, P))
    assert y[0, 0, 3, 3] == -7084549


def test_input_tiles_overlap_and_zero_extension():
    x = np.arange(1, 1 + 36, dtype=np.int8).reshape(1, 1, 6, 6)
    d = rw.input_tiles(x, r=3, m=4, pad=1)                        # t = 6, tiles 2x2, stride 4
    assert d.shape == (4, 1, 6, 6)
    assert (d[0, 0, 0, :] == 0).all() and (d[0, 0, :, 0] == 0).all()
    assert d[0, 0, 1, 1] == 1 and d[0, 0, 5, 5] == x[0, 0, 4, 4]
    assert d[1, 0, 1, 0] == x[0, 0, 0, 3]                          # tile (0,1) starts at column 4-1
    assert (d[1, 0, :, 3:] == 0).all()                            # overhang beyond the plane
    assert d[3, 0, 0, 0] == x[0, 0, 3, 3]


def test_planted_mistakes_are_caught():
    # a transposed operand or a wrong sign in the transforms must break the identity
    m, r, p = 8, 3, 251
    t = m + r - 1
    AT, G, BT = rw.matrices_mod(m, r, p)
    d = si.int8_tensor(61, (t, t)).astype(np.int64)
    g = si.int8_tensor(62, (r, r)).astype(np.int64)
    direct = np.array([[sum(d[u + i, v + j] * g[i, j] for i in range(r) for j in range(r))
                        for v in range(m)] for u in range(m)]) % p
    good = (AT @ (((G @ g @ G.T) % p) * ((BT @ d @ BT.T) % p) % p) @ AT.T) % p
    bad_t = (AT @ (((G @ g @ G.T) % p) * ((BT.T @ d @ BT) % p) % p) @ AT.T) % p
    bad_f = (AT @ (((G @ g[::-1, ::-1] @ G.T) % p) * ((BT @ d @ BT.T) % p) % p) @ AT.T) % p
    assert np.array_equal(good, direct)
    assert not np.array_equal(bad_t, direct) and not np.array_equal(bad_f, direct)
