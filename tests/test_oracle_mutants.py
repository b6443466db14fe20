"""The pins must be able to fail: each plausible mistake, planted in a copy of the
row function on the CPU, has to trip at least one check of the battery that the real
oracle passes."""
from fractions import Fraction

import numpy as np
import pytest

from conftest import golden_files, read_golden
from oracle import hccs_ref

N = 255 << 15


def battery(row_fn):
    """Returns the names of the pins that `row_fn(x, B, S, D) -> list` violates."""
    failed = []
    for name in golden_files():
        g = read_golden(name)
        if g["mode"] == "u8" and row_fn(g["x"], *g["params"]) != g["p"]:
            failed.append("golden:" + name)
    rng = np.random.default_rng(1)
    for n, (B, S, D) in [(64, (511, 3, 120)), (128, (255, 2, 100)), (16, (900, 9, 77))]:
        for _ in range(6):
            x = np.clip(np.rint(rng.normal(0, 30, n)), -128, 127).astype(int).tolist()
            p = row_fn(x, B, S, D)
            m = max(x)
            s = np.interp([m - v for v in x], [0, D, 255], [B, B - S * D, B - S * D])
            Z = int(round(s.sum()))
            for si, pi in zip(s, p):
                e = Fraction(255 * int(round(si)), Z)
                if not (pi <= e and pi in (int(e), int(e) - 1)):
                    failed.append("sandwich")
                    break
            order = np.argsort(x, kind="stable")
            if np.any(np.diff(np.array(p)[order]) < 0):
                failed.append("monotone")
            if not (255 - n <= sum(p) <= 255):
                failed.append("sum")
    x = [-128] * 64
    x[17] = 5
    p = row_fn(x, 500, 4, 120)
    if p[17] != 72 or any(v != 2 for i, v in enumerate(p) if i != 17):
        failed.append("one_hot")
    if row_fn([0] * 64, 511, 0, 1) != [3] * 64:
        failed.append("flat")
    return failed


def _mutant(no_clamp=False, wrong_dir=False, plus=False, z_plus=0, shift=15, one_div=False,
            first_as_max=False, drop_last=False, round_rho=False, d_off=0, num=N):
    def fn(x, B, S, D):
        m = x[0] if first_as_max else max(x)
        if wrong_dir:
            lo = min(x)
            delta = [min(v - lo, D) for v in x]
        elif no_clamp:
            delta = [m - v for v in x]
        else:
            delta = [min(max(m - v, 0), D + d_off) for v in x]
        s = [max(B + S * d, 0) if plus else max(B - S * d, 0) for d in delta]
        Z = sum(s[:-1]) if drop_last else sum(s)
        Z += z_plus
        if one_div:
            return [(255 * v) // Z for v in s]
        rho = (num + Z // 2) // Z if round_rho else num // Z
        return [min((v * rho) >> shift, 255) for v in s]
    return fn


MUTANTS = {
    "no_clamp": dict(no_clamp=True),
    "distance_from_min": dict(wrong_dir=True),
    "slope_sign": dict(plus=True),
    "sum_off_by_one": dict(z_plus=1),
    "shift_16": dict(shift=16),
    "shift_14": dict(shift=14),
    "single_division": dict(one_div=True),
    "first_element_as_max": dict(first_as_max=True),
    "dropped_last_term": dict(drop_last=True),
    "rounded_reciprocal": dict(round_rho=True),
    "clamp_at_D_plus_1": dict(d_off=1),
    "clamp_at_D_minus_1": dict(d_off=-1),
    "numerator_256": dict(num=256 << 15),
}


def test_unmutated_functions_pass_the_battery(oracle):
    assert battery(hccs_ref.row_u8) == []
    assert battery(_mutant()) == []
    assert battery(lambda x, B, S, D: oracle.row(x, B, S, D, 0)[0].tolist()) == []


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_each_planted_mistake_is_caught(name):
    assert battery(_mutant(**MUTANTS[name])) != [], name
