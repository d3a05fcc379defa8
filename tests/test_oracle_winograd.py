"""Pins for the oracle's Winograd building blocks and its kernel splitting.

None of these re-type the oracle's own formulas: the F(2,l) matrices are checked
against the paper's printed F(2,3) (golden file), against exact rational arithmetic on
basis vectors (a bilinear identity that any wrong sign, index or 1/2 breaks), and the
splitting is checked against what the paper prints: the 5x5 examples of Sec. 4.1 and
every DWM row of Table 3.
"""
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle


def _read_matrices(path):
    mats, cur, rows_left = {}, None, 0
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        tok = line.split()
        if rows_left == 0:
            cur, rows_left = tok[0], int(tok[1])
            mats[cur] = []
        else:
            mats[cur].append([Fraction(t) for t in tok])
            rows_left -= 1
    return mats


def test_f23_matrices_are_the_printed_ones(golden_dir):
    """Sec. 3.2: B^T, G, A^T of F(2,3), entry by entry."""
    gold = _read_matrices(os.path.join(golden_dir, "f23_matrices.txt"))
    BT, G, AT = oracle.winograd_matrices(3)
    for name, got in (("BT", BT), ("G", G), ("AT", AT)):
        want = np.array([[float(v) for v in row] for row in gold[name]])
        assert got.shape == want.shape
        assert np.array_equal(got, want), name


@pytest.fixture
def f22_form(request):
    """Select one of the oracle's two F(2,2) forms for a test, restoring the default after."""
    oracle.set_f22_form(request.param)
    yield request.param
    oracle.set_f22_form(0)


@pytest.mark.parametrize("f22_form", [0, 1], indirect=True)
@pytest.mark.parametrize("l", [1, 2, 3])
def test_f2l_matrices_reproduce_correlation_exactly(l, f22_form):
    """A^T[(G g) .* (B^T d)] == [sum_k d[k] g[k], sum_k d[k+1] g[k]] as an identity
    over the rationals (Sec. 3.1 formula; correlation form of the printed matrices).
    The map is bilinear in (g, d), so exactness on all basis pairs proves it.
    Both F(2,2) forms (the paper prints neither) must pass."""
    BT, G, AT = oracle.winograd_matrices(l)
    fr = lambda M: [[Fraction(v).limit_denominator(8) for v in row] for row in M]
    BTf, Gf, ATf = fr(BT), fr(G), fr(AT)
    # entries must be representable exactly (0, +-1, +-1/2): no silent rounding above
    assert np.array_equal(np.array(BTf, float), BT) and np.array_equal(np.array(Gf, float), G)
    t = l + 1
    for a, b in itertools.product(range(l), range(t)):
        g = [Fraction(int(i == a)) for i in range(l)]
        d = [Fraction(int(i == b)) for i in range(t)]
        u = [sum(Gf[i][j] * g[j] for j in range(l)) for i in range(t)]
        v = [sum(BTf[i][j] * d[j] for j in range(t)) for i in range(t)]
        y = [sum(ATf[o][i] * u[i] * v[i] for i in range(t)) for o in range(2)]
        want = [sum(d[o + k] * g[k] for k in range(l)) for o in range(2)]
        assert y == want, (l, a, b)


@pytest.mark.parametrize("l", [1, 2, 3])
def test_multiplication_count_of_f2l(l):
    """F(m,r) needs m+r-1 multiplications (Sec. 3.1): tile length l+1 for m=2."""
    BT, G, AT = oracle.winograd_matrices(l)
    assert BT.shape == (l + 1, l + 1) and G.shape == (l + 1, l) and AT.shape == (2, l + 1)


def test_second_f22_form_is_the_printed_f23_without_its_last_point(golden_dir):
    """Form 1 of F(2,2): rows/columns 0..2 of the printed F(2,3) matrices (Sec. 3.2), i.e. a
    3-tap piece whose third tap is zero with the vanishing fourth product dropped."""
    gold = _read_matrices(os.path.join(golden_dir, "f23_matrices.txt"))
    want = {k: np.array([[float(v) for v in row] for row in gold[k]]) for k in ("BT", "G", "AT")}
    oracle.set_f22_form(1)
    try:
        BT, G, AT = oracle.winograd_matrices(2)
    finally:
        oracle.set_f22_form(0)
    assert np.array_equal(BT, want["BT"][:3, :3])
    assert np.array_equal(G, want["G"][:3, :2])
    assert np.array_equal(AT, want["AT"][:, :3])
    # the dropped parts really vanish or are unused: G's last row only sees the third tap,
    # B^T's first three rows do not read the fourth sample
    assert np.all(want["G"][3, :2] == 0) and np.all(want["BT"][:3, 3] == 0)
    BT0, G0, AT0 = oracle.winograd_matrices(2)
    assert not np.array_equal(G0, G)  # the default form is a different algorithm


@pytest.mark.parametrize("f22_form", [0, 1], indirect=True)
@pytest.mark.parametrize("l", [1, 2, 3])
def test_winograd_1d_function_matches_numpy_correlate(l, f22_form):
    rng = np.random.default_rng(7 + l)
    for _ in range(20):
        g, d = rng.standard_normal(l), rng.standard_normal(l + 1)
        want = np.correlate(d, g, mode="valid")
        got = oracle.winograd_1d(g, d)
        assert np.allclose(got, want, rtol=0, atol=1e-14)


def test_1d_split_examples_from_the_paper():
    # Sec. 4.1, the r=5 example: F(2,3) on taps 0-2, F(2,2) on taps 3-4.
    assert oracle.split_1d(5, 1) == [(0, 0, 3), (0, 3, 2)]
    # Sec. 4.1 stride-2 grouping (eq. 13): even taps {0,2,4}, odd taps {1,3}.
    assert oracle.split_1d(5, 2) == [(0, 0, 3), (1, 0, 2)]
    # 3 | r: ceil(r/3) pieces, not floor(r/3)+1 (Table 3's 9x9 row fixes this).
    assert oracle.split_1d(9, 1) == [(0, 0, 3), (0, 3, 3), (0, 6, 3)]
    # stride larger than the kernel: only phases that hold a tap exist.
    assert oracle.split_1d(1, 2) == [(0, 0, 1)]
    assert oracle.split_1d(3, 2) == [(0, 0, 2), (1, 0, 1)]
    assert oracle.split_1d(11, 4) == [(0, 0, 3), (1, 0, 3), (2, 0, 3), (3, 0, 2)]
    assert oracle.split_1d(7, 2) == [(0, 0, 3), (0, 3, 1), (1, 0, 3)]


@pytest.mark.parametrize("stride", [1, 2])
def test_5x5_splits_into_3x3_3x2_2x3_2x2(stride):
    """Sec. 4.1 / Fig. 2: a 5x5 kernel (stride 1, and stride 2) gives four stride-1
    convolutions of sizes 3x3, 3x2, 2x3, 2x2."""
    parts = oracle.split_2d(5, 5, stride)
    assert sorted((p[2], p[5]) for p in parts) == [(2, 2), (2, 3), (3, 2), (3, 3)]


@pytest.mark.parametrize("R,S,s", [(r, q, s) for r in range(1, 13) for q in (1, 3, 5, 8, 11)
                                   for s in (1, 2, 3, 4, 5)])
def test_every_tap_belongs_to_exactly_one_part(R, S, s):
    cover = np.zeros((R, S), int)
    for ph, jh, lh, pw, jw, lw in oracle.split_2d(R, S, s):
        assert 1 <= lh <= 3 and 1 <= lw <= 3
        for a in range(lh):
            for b in range(lw):
                cover[s * (jh + a) + ph, s * (jw + b) + pw] += 1
    assert np.all(cover == 1)


def _sig3(v):
    return float("%.2E" % v)


def test_table3_multiplication_counts(golden_dir):
    """Every DWM row and the Direct column of Table 3: 14x14 outputs = 49 tiles of 2x2."""
    rows = [l.split() for l in open(os.path.join(golden_dir, "table3_mults.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 10
    for k, s, direct_p, dwm_p, speed_p in rows:
        k, s = int(k), int(s)
        dwm = 49 * oracle.mults_per_tile(k, k, s)
        direct = 196 * k * k
        # printed with three significant digits: allow half a unit in the last place
        assert abs(direct - float(direct_p)) <= 0.5 * 10 ** (len(str(direct)) - 3), (k, s, direct)
        assert abs(dwm - float(dwm_p)) <= 0.5 * 10 ** max(len(str(dwm)) - 3, 0), (k, s, dwm)
        assert abs(direct / dwm - float(speed_p)) <= 0.005 + 1e-9, (k, s, direct / dwm)
    # exact values that the count model must give (3+1)^2*49, (4+3)^2*49, (4+4+2)^2*49 ...
    assert [49 * oracle.mults_per_tile(k, k, 1) for k in (3, 5, 7, 9, 11)] == [784, 2401, 4900, 7056, 11025]
    assert [49 * oracle.mults_per_tile(k, k, 2) for k in (3, 5, 7, 9, 11)] == [1225, 2401, 4900, 8281, 11025]
