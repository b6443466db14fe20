"""Pins for the CPU oracle: everything here checks oracle/ against something
other than itself -- hand-worked rows, exact rational arithmetic, closed forms,
library routines for the pieces that have one, invariants the paper claims,
and brute force against the independent big-integer Python version."""
import itertools
from fractions import Fraction

import numpy as np
import pytest

from conftest import golden_files, read_golden
from oracle import hccs_ref
from paper_2604_02292_amd import synth

MODES = {"u8": 0, "i16": 1, "clb_u8": 2, "clb_i16": 3}
PY_ROW = {0: hccs_ref.row_u8, 1: hccs_ref.row_i16, 2: hccs_ref.row_clb_u8, 3: hccs_ref.row_clb_i16}
N_U8 = 255 * 2 ** 15


# ---------------------------------------------------------------- hand-worked rows
@pytest.mark.parametrize("name", golden_files())
def test_golden_rows(oracle, name):
    g = read_golden(name)
    mode = MODES[g["mode"]]
    B, S, D = g["params"]
    p, Z, rho, rc = oracle.row(g["x"], B, S, D, mode)
    assert rc == 0
    assert Z == g["Z"][0]
    assert rho == g["rho"][0]
    assert p.tolist() == g["p"]
    assert PY_ROW[mode](g["x"], B, S, D) == g["p"]
    # the fixture's own intermediate lines are consistent with each other
    assert sum(g["s"]) == g["Z"][0]
    assert [B - S * d for d in g["delta"]] == g["s"]


# ---------------------------------------------------------------- admissibility (Sec. IV-C)
@pytest.mark.parametrize("B,S,D,n,band,ok", [
    (511, 0, 1, 64, 1, True),      # n*B = 32704 <= 32767
    (512, 0, 1, 64, 1, False),     # n*B = 32768
    (512, 0, 1, 64, 0, True),      # 8-bit band has the wider ceiling
    (130560, 0, 1, 64, 0, False),  # B > 32767
    (32767, 0, 1, 255, 0, True),   # 255*32767 = 8355585 <= 8355840
    (32767, 0, 1, 256, 0, False),  # 256*32767 > 8355840
    (100, 1, 96, 64, 1, True),     # floor 4 -> 64*4 = 256
    (100, 1, 97, 64, 1, False),    # floor 3 -> 192 < 256
    (100, 1, 101, 64, 1, False),   # B - S*D < 0
    (100, 1, 128, 64, 1, False),   # D > 127
    (100, 128, 0, 64, 1, False),   # S > 127
    (0, 0, 0, 64, 1, False),       # B < 1
    (7, 0, 127, 4096, 1, True),
    (8, 0, 127, 4096, 1, False),
    (2040, 15, 127, 4096, 0, True),
    (2041, 15, 127, 4096, 0, False),
])
def test_admissibility_boundaries(oracle, B, S, D, n, band, ok):
    assert (oracle.check_params(B, S, D, n, band) == 0) == ok
    assert hccs_ref.admissible(B, S, D, n, band) == ok


def test_admissibility_error_kinds(oracle):
    assert oracle.check_params(100, 1, 101, 64, 1) == -5
    assert oracle.check_params(100, 1, 97, 64, 1) == -6
    assert oracle.check_params(512, 0, 1, 64, 1) == -7


# ---------------------------------------------------------------- the pieces against library routines
def _rows(seed, count, n, sigma=30.0):
    g = np.random.default_rng(seed)
    return np.clip(np.rint(g.normal(0, sigma, size=(count, n))), -128, 127).astype(np.int8)


@pytest.mark.parametrize("n,params", [(16, (900, 9, 77)), (64, (511, 3, 120)), (128, (255, 2, 100)),
                                      (48, (600, 5, 60))])
def test_scores_are_the_clipped_linear_interpolant(oracle, n, params):
    """Eq. (2)+(3): s as a function of (max - x) is the piecewise-linear curve through
    (0,B), (D,B-S*D), flat beyond -- numpy.interp states that curve independently.
    The scores are recovered from the 16-bit output (p = s*rho, Eq. (7))."""
    B, S, D = params
    if not hccs_ref.admissible(B, S, D, n, 1):
        pytest.skip("not in the strict band")
    for x in _rows(n, 40, n):
        p, Z, rho, rc = oracle.row(x, B, S, D, 1)
        assert rc == 0
        dist = (int(x.max()) - x.astype(np.int64)).astype(np.float64)
        s_lib = np.interp(dist, [0.0, float(D), 255.0], [float(B), float(B - S * D), float(B - S * D)])
        assert np.array_equal(p.astype(np.int64), np.rint(s_lib).astype(np.int64) * rho)
        assert Z == int(np.rint(s_lib).sum())
        assert rho == 32767 // Z


@pytest.mark.parametrize("n,params,band", [(4, (200, 10, 12), 1), (64, (511, 3, 120), 1),
                                           (128, (255, 2, 100), 1), (512, (63, 1, 40), 1),
                                           (512, (16000, 120, 127), 0), (4096, (2040, 15, 127), 0)])
def test_sandwich_against_exact_rationals(oracle, n, params, band):
    """Eq. (8): rho/2^15 lies in (255/Z - 2^-15, 255/Z] and s < 2^15, so the two-floor
    result is floor(255*s/Z) or one less, never anything else, and never above it."""
    B, S, D = params
    assert hccs_ref.admissible(B, S, D, n, band)
    for x in _rows(7 * n, 12, n):
        p, Z, rho, rc = oracle.row(x, B, S, D, 0)
        assert rc == 0
        assert rho * Z <= N_U8 < (rho + 1) * Z
        m = int(x.max())
        for xi, pi in zip(x.tolist(), p.tolist()):
            s = B - S * min(m - xi, D)
            exact = Fraction(255 * s, Z)
            assert pi <= exact and pi in (int(exact), int(exact) - 1)


def test_u8_close_to_float_normalisation(oracle):
    """Eq. (5): p/255 is s/Z up to the truncations; compare with a float64 normalise."""
    B, S, D = 255, 2, 100
    for x in _rows(3, 50, 128):
        p, Z, rho, rc = oracle.row(x, B, S, D, 0)
        s = B - S * np.minimum(int(x.max()) - x.astype(np.int64), D)
        ideal = 255.0 * s / s.sum()
        assert np.all(p <= ideal + 1e-9) and np.all(p > ideal - 2.0)


# ---------------------------------------------------------------- invariants the paper claims
@pytest.mark.parametrize("n,band", [(32, 1), (64, 1), (128, 1), (256, 1), (80, 1), (1024, 0)])
def test_invariants_random_rows_and_params(oracle, n, band):
    table = synth.head_params(24, n, band, seed=n)
    rows = np.concatenate([_rows(n, 30, n, 12.0), _rows(n + 1, 30, n, 60.0)])
    for (B, S, D), x in zip(itertools.cycle(table.tolist()), rows):
        p, Z, rho, rc = oracle.row(x, B, S, D, 0)
        assert rc == 0
        p = p.astype(np.int64)
        assert p.min() >= 0 and p.max() <= 255                      # bounded, non-negative
        order = np.argsort(x, kind="stable")
        assert np.all(np.diff(p[order]) >= 0)                       # order preserved (weakly)
        for v in np.unique(x):                                      # ties stay ties
            assert np.unique(p[x == v]).size == 1
        assert p[np.argmax(x)] == p.max()
        assert Z >= 256 and 1 <= rho <= 32767
        assert p.sum() <= 255
        if band == 1:
            assert Z <= 32767 and rho >= 255
            assert p.sum() >= max(0, 255 - n)                        # sum ~ T up to truncation
        assert p.tolist() == hccs_ref.row_u8(x.tolist(), B, S, D)


def test_i16_invariants(oracle):
    for n in (32, 64, 128):
        table = synth.head_params(12, n, 1, seed=100 + n)
        for (B, S, D), x in zip(itertools.cycle(table.tolist()), _rows(n, 24, n)):
            p, Z, rho, rc = oracle.row(x, B, S, D, 1)
            assert rc == 0
            p = p.astype(np.int64)
            assert p.sum() == rho * Z and 32767 - Z < p.sum() <= 32767
            assert p.tolist() == hccs_ref.row_i16(x.tolist(), B, S, D)


def test_clb_over_estimates_by_less_than_two(oracle):
    """Eq. (9): 2^k <= Z < 2^(k+1), so the approximate reciprocal is in [exact, 2*exact+1]."""
    for n in (32, 64, 128):
        table = synth.head_params(12, n, 1, seed=200 + n)
        for (B, S, D), x in zip(itertools.cycle(table.tolist()), _rows(n, 24, n)):
            _, Z, rho_exact, _ = oracle.row(x, B, S, D, 0)
            pc, Zc, rho_clb, rc = oracle.row(x, B, S, D, 2)
            assert rc == 0 and Zc == Z
            assert rho_clb == N_U8 >> (Z.bit_length() - 1)
            assert rho_exact <= rho_clb <= 2 * rho_exact + 1
            pe = oracle.row(x, B, S, D, 0)[0].astype(np.int64)
            assert np.all(pc.astype(np.int64) >= pe)
            assert pc.tolist() == hccs_ref.row_clb_u8(x.tolist(), B, S, D)
            p16, _, rho16, rc = oracle.row(x, B, S, D, 3)
            assert rc == 0 and rho16 == 32767 >> (Z.bit_length() - 1)
            assert p16.tolist() == hccs_ref.row_clb_i16(x.tolist(), B, S, D)


# ---------------------------------------------------------------- closed forms
def test_flat_rows_and_zero_slope(oracle):
    """All logits equal, or S = 0, or D = 0: every score is B, Z = n*B,
    p = (B*floor(N/(n*B))) >> 15 for every element."""
    for n, B in [(64, 511), (64, 4), (128, 255), (32, 1000), (256, 127), (4096, 2040)]:
        band = 1 if n * B <= 32767 else 0
        want = (B * (N_U8 // (n * B))) >> 15
        flat = np.full(n, -7, dtype=np.int8)
        rnd = _rows(n, 1, n)[0]
        for x, (S, D) in [(flat, (0, 127)), (flat, (min(127, (B - -(-256 // n)) // 5), 5)),
                          (rnd, (0, 127)), (rnd, (127, 0))]:
            if not hccs_ref.admissible(B, S, D, n, band):
                continue
            p, Z, rho, rc = oracle.row(x, B, S, D, 0)
            assert rc == 0 and Z == n * B
            assert np.all(p == want)
    # the n = 64, B = 511 value, worked by hand: rho = floor(8355840/32704) = 255, 511*255 >> 15 = 3
    assert oracle.row(np.zeros(64, np.int8), 511, 0, 1, 0)[0].tolist() == [3] * 64


def test_one_hot_like_row(oracle):
    """One maximum, every other logit at least D below it: Z = B + (n-1)(B - S*D)."""
    n, (B, S, D) = 64, (500, 4, 120)
    x = np.full(n, -128, dtype=np.int8)
    x[17] = 5
    p, Z, rho, rc = oracle.row(x, B, S, D, 0)
    assert rc == 0 and Z == B + (n - 1) * (B - S * D) == 1760
    assert rho == 8355840 // 1760 == 4747
    assert p[17] == (500 * 4747) >> 15 == 72 and np.all(np.delete(p, 17) == (20 * 4747) >> 15)


def test_shift_invariance_and_permutation_equivariance(oracle):
    B, S, D = 255, 2, 100
    g = np.random.default_rng(5)
    for x in _rows(11, 20, 128, 20.0):
        x = np.clip(x, -100, 100).astype(np.int8)
        base = oracle.row(x, B, S, D, 0)[0]
        for c in (-28, 13, 27):
            assert np.array_equal(oracle.row((x + c).astype(np.int8), B, S, D, 0)[0], base)
        perm = g.permutation(128)
        assert np.array_equal(oracle.row(x[perm], B, S, D, 0)[0], base[perm])


# ---------------------------------------------------------------- brute force
def test_brute_force_all_rows_of_length_two(oracle):
    """Every one of the 65,536 int8 rows of length 2, C oracle vs the big-integer Python
    version vs the definition's invariants, for several admissible parameter sets."""
    vals = np.arange(-128, 128, dtype=np.int8)
    grid = np.stack(np.meshgrid(vals, vals, indexing="ij"), -1).reshape(1, 1, 65536, 2)
    for B, S, D in [(1100, 7, 127), (16383, 127, 127), (128, 0, 1), (5000, 50, 90), (300, 1, 127)]:
        assert hccs_ref.admissible(B, S, D, 2, 1)
        out, rc = oracle.softmax(grid, np.array([[B, S, D]], np.int32), 1, 0)
        assert rc == 0
        out = out.reshape(65536, 2)
        x = grid.reshape(65536, 2).astype(np.int64)
        # closed form for n = 2: the larger logit has s = B, the other B - S*min(|x0-x1|, D)
        gap = np.minimum(np.abs(x[:, 0] - x[:, 1]), D)
        s_hi, s_lo = np.full(65536, B), B - S * gap
        Z = s_hi + s_lo
        rho = N_U8 // Z
        hi_is_0 = x[:, 0] >= x[:, 1]
        want0 = np.where(hi_is_0, s_hi, s_lo) * rho >> 15
        want1 = np.where(hi_is_0, s_lo, s_hi) * rho >> 15
        assert np.array_equal(out[:, 0], want0) and np.array_equal(out[:, 1], want1)
        for idx in range(0, 65536, 97):
            assert out[idx].tolist() == hccs_ref.row_u8(x[idx].tolist(), B, S, D)


def test_brute_force_length_three_sampled_grid(oracle):
    vals = np.array([-128, -127, -64, -3, -1, 0, 1, 2, 50, 126, 127], dtype=np.int8)
    rows = np.array(list(itertools.product(vals, repeat=3)), dtype=np.int8).reshape(1, 1, -1, 3)
    for B, S, D in [(10922, 85, 127), (86, 0, 0), (900, 7, 100)]:
        assert hccs_ref.admissible(B, S, D, 3, 1)
        for mode in range(4):
            out, rc = oracle.softmax(rows, np.array([[B, S, D]], np.int32), 1, mode)
            assert rc == 0
            for x, p in zip(rows.reshape(-1, 3).tolist(), out.reshape(-1, 3).tolist()):
                assert p == PY_ROW[mode](x, B, S, D)


def test_exhaustive_reciprocal(oracle):
    """Every row sum the 8-bit band admits: rho*Z <= 255*2^15 < (rho+1)*Z, rho in [1, 32640]."""
    Z = np.arange(256, N_U8 + 1, dtype=np.int64)
    rho, rc = oracle.reciprocal_u8(Z)
    assert rc == 0
    assert np.all(rho * Z <= N_U8) and np.all((rho + 1) * Z > N_U8)
    assert rho.max() == 32640 and rho.min() == 1
    assert np.all(rho[Z <= 32767] >= 255)


# ---------------------------------------------------------------- tensor layout: head of a row
def test_head_lookup_and_row_independence(oracle):
    """Row r uses head (r // Lq) % H; rows are independent, so any split of the
    batch axis concatenates to the whole (Sec. IV-D)."""
    w = synth.make_workload("edge_encoder", shape=(3, 8, 5, 128))
    out, rc = oracle.softmax(w["logits"], w["table"], w["band"])
    assert rc == 0
    for b, h, q in [(0, 0, 0), (1, 3, 4), (2, 7, 2)]:
        B, S, D = w["table"][h].tolist()
        assert out[b, h, q].tolist() == hccs_ref.row_u8(w["logits"][b, h, q].tolist(), B, S, D)
    parts = [oracle.softmax(w["logits"][b:b + 1], w["table"], w["band"])[0] for b in range(3)]
    assert np.array_equal(np.concatenate(parts), out)
    out_mt, rc = oracle.softmax(w["logits"], w["table"], w["band"], threads=4)
    assert rc == 0 and np.array_equal(out_mt, out)


def test_rejects_inadmissible_table(oracle):
    x = np.zeros((1, 2, 4, 64), np.int8)
    bad = np.array([[511, 0, 1], [512, 0, 1]], np.int32)
    assert oracle.softmax(x, bad, 1)[1] == -7
    assert oracle.softmax(x, bad, 0)[1] == 0


# ---------------------------------------------------------------- strict band at n = 4096 is vacuous
def test_strict_band_long_rows_give_all_zero_output(oracle):
    """With n = 4096 the band of Eq. (11) caps B at 7, so p <= floor(255*7/4096) = 0."""
    x = _rows(1, 4, 4096)
    for B in range(1, 8):
        for S, D in [(0, 127), (1, B - 1), (B - 1, 1)]:
            if hccs_ref.admissible(B, S, D, 4096, 1):
                for row in x:
                    assert not oracle.row(row, B, S, D, 0)[0].any()
