"""Pins for the oracle's calibration objective (Sec. III-C, Eq. (10)): the divergence
against scipy's routines, non-negativity, cases where HCCS reproduces softmax exactly,
a closed form at n = 2 rows, and the arg-min rule."""
import math

import numpy as np
import pytest
from scipy.special import softmax as sp_softmax
from scipy.stats import entropy as sp_kl

from oracle import hccs_ref


def _logits(seed, shape, sigma=20.0):
    g = np.random.default_rng(seed)
    return np.clip(np.rint(g.normal(0, sigma, size=shape)), -128, 127).astype(np.int8)


def test_objective_matches_scipy_on_each_row(oracle):
    x = _logits(1, (3, 2, 5, 64))
    alpha = np.array([0.11, 0.05])
    cand = np.array([[511, 3, 120], [300, 2, 100], [64, 0, 0], [512, 0, 1], [100, 1, 97]], np.int32)
    obj, best, rc = oracle.calibrate(x, alpha, cand)
    assert rc == 0
    assert np.isinf(obj[:, 3]).all() and np.isinf(obj[:, 4]).all()      # inadmissible under the strict band
    for h in range(2):
        for c in range(3):
            B, S, D = cand[c].tolist()
            kls = []
            for b in range(3):
                for q in range(5):
                    row = x[b, h, q]
                    P = sp_softmax(alpha[h] * row.astype(np.float64))           # library softmax
                    ph = np.array(hccs_ref.row_i16(row.tolist(), B, S, D), dtype=np.float64)
                    kls.append(sp_kl(P, ph / ph.sum()))                         # library KL divergence
            assert obj[h, c] == pytest.approx(np.mean(kls), rel=1e-12, abs=1e-15)
    assert obj[np.isfinite(obj)].min() >= 0.0                                   # Gibbs' inequality
    assert best.tolist() == [int(np.argmin(obj[0])), int(np.argmin(obj[1]))]


def test_exact_reproduction_gives_zero_divergence(oracle):
    """x = [0,-1,0,-1] with alpha = ln 2: softmax = [1/3,1/6,1/3,1/6]; (254,127,1) scores [254,127,254,127],
    the same distribution.  A flat row is reproduced by any candidate."""
    x = np.array([0, -1, 0, -1], np.int8).reshape(1, 1, 1, 4)
    cand = np.array([[254, 127, 1], [254, 100, 1], [200, 10, 12]], np.int32)
    obj, best, rc = oracle.calibrate(x, np.array([math.log(2.0)]), cand)
    assert rc == 0
    assert obj[0, 0] == pytest.approx(0.0, abs=1e-15) and best[0] == 0
    assert obj[0, 1] > 1e-4 and obj[0, 2] > 1e-4
    flat = np.full((2, 1, 3, 16), 9, np.int8)
    obj, best, rc = oracle.calibrate(flat, np.array([0.3]), np.array([[100, 1, 50], [2047, 0, 0]], np.int32))
    assert rc == 0 and np.allclose(obj, 0.0, atol=1e-15) and best[0] == 0      # first index wins ties


def test_closed_form_two_element_rows(oracle):
    """n = 2, rows [0,-d]: P = [1/(1+e^-ad), e^-ad/(1+e^-ad)], q = [B, B-S*min(d,D)]/Z."""
    ds = [0, 1, 3, 10, 40]
    x = np.array([[0, -d] for d in ds], np.int8).reshape(1, 1, len(ds), 2)
    a = 0.07
    B, S, D = 1100, 7, 30
    obj, _, rc = oracle.calibrate(x, np.array([a]), np.array([[B, S, D]], np.int32))
    assert rc == 0
    want = 0.0
    for d in ds:
        e = math.exp(-a * d)
        P = [1 / (1 + e), e / (1 + e)]
        s = [B, B - S * min(d, D)]
        want += sum(p * math.log(p / (si / sum(s))) for p, si in zip(P, s))
    assert obj[0, 0] == pytest.approx(want / len(ds), rel=1e-12)


def test_argmin_prefers_the_better_slope(oracle):
    """Logits within 6 of the maximum and alpha = 0.1: softmax falls to e^-0.6 = 0.55 at distance 6, which a
    line from B = 600 reaches with S = 45.  Among candidates that differ only in slope the objective must be
    unimodal with its minimum next to that slope."""
    g = np.random.default_rng(3)
    x = g.integers(-6, 1, size=(4, 1, 16, 32)).astype(np.int8)
    x[..., 0] = 0
    slopes = [0, 15, 30, 45, 60, 75, 90]
    cand = np.array([[600, s, 6] for s in slopes], np.int32)
    assert all(hccs_ref.admissible(600, s, 6, 32, 1) for s in slopes)
    obj, best, rc = oracle.calibrate(x, np.array([0.1]), cand, threads=2)
    assert rc == 0
    j = obj[0]
    assert slopes[best[0]] in (30, 45, 60)
    assert np.all(np.diff(j[:best[0] + 1]) < 0) and np.all(np.diff(j[best[0]:]) > 0)


def test_threads_do_not_change_the_result(oracle):
    x = _logits(5, (2, 3, 8, 48))
    cand = np.array([[600, 5, 60], [682, 0, 1], [300, 2, 100], [100, 1, 90]], np.int32)
    a = np.array([0.1, 0.2, 0.05])
    o1, b1, _ = oracle.calibrate(x, a, cand, threads=1)
    o4, b4, _ = oracle.calibrate(x, a, cand, threads=4)
    assert np.array_equal(o1, o4) and np.array_equal(b1, b4)
