"""Pins for the oracle's fused block (Q.K^T -> requantise -> HCCS -> P.V).
The paper defines no such block; these pin this repository's definition: a
hand-worked case, each stage against a library routine or exact rationals,
and the composition against the separately pinned row function."""
from fractions import Fraction
import math

import numpy as np
import pytest

from conftest import read_golden
from oracle import hccs_ref
from paper_2604_02292_amd import synth


def _qkv(seed, shape, lo=-64, hi=63):
    g = np.random.default_rng(seed)
    return tuple(g.integers(lo, hi + 1, size=shape, dtype=np.int8) for _ in range(3))


def test_hand_worked_block(oracle):
    g = read_golden("a1_attention_tiny.txt")
    q = np.array(g["q"], np.int8).reshape(1, 1, 2, 1)
    k = np.array(g["k"], np.int8).reshape(1, 1, 2, 1)
    v = np.array(g["v"], np.int8).reshape(1, 1, 2, 1)
    table = np.array([g["params"]], np.int32)
    rq = np.array([g["requant"]], np.int32)
    x, rc = oracle.requant_logits(q, k, rq)
    assert rc == 0 and x.reshape(-1).tolist() == g["x"]
    p, rc = oracle.softmax(x, table, 1)
    assert rc == 0 and p.reshape(-1).tolist() == g["p"]
    o, rc = oracle.attention(q, k, v, table, rq, 1)
    assert rc == 0 and o.reshape(-1).tolist() == g["o"]
    B, S, D = g["params"]
    o_py = hccs_ref.attention([[3], [-2]], [[5], [4]], [[7], [-1]], B, S, D, 1, 1)
    assert [r[0] for r in o_py] == g["o"]


@pytest.mark.parametrize("mult,shift", [(1, 1), (97, 16), (256, 16), (4096, 12), (4096, 23), (4096, 24), (1, 24), (3, 2)])
def test_requant_is_round_half_up_of_the_exact_ratio(oracle, mult, shift):
    q, k, _ = _qkv(shift * 7 + mult, (1, 2, 24, 64), -128, 127)
    rq = np.array([[mult, shift]] * 2, np.int32)
    x, rc = oracle.requant_logits(q, k, rq)
    assert rc == 0
    acc = np.matmul(q.astype(np.int64), np.swapaxes(k.astype(np.int64), -1, -2))   # library product
    for a, got in zip(acc.reshape(-1).tolist()[::7], x.reshape(-1).tolist()[::7]):
        want = math.floor(Fraction(a * mult, 2 ** shift) + Fraction(1, 2))
        assert got == max(-128, min(127, want))
        assert got == hccs_ref.requant(a, mult, shift)


def test_identity_requant_and_sign_handling(oracle):
    # mult = 2^12, shift = 12 is the identity on the accumulator
    q, k, _ = _qkv(3, (1, 1, 8, 4), -5, 5)
    x, rc = oracle.requant_logits(q, k, np.array([[4096, 12]], np.int32))
    acc = np.matmul(q.astype(np.int64), np.swapaxes(k.astype(np.int64), -1, -2))
    assert rc == 0 and np.array_equal(x.astype(np.int64), np.clip(acc, -128, 127))
    # halves round up: -3/2 -> -1, -1/2 -> 0, 1/2 -> 1, 3/2 -> 2
    assert [hccs_ref.requant(a, 1, 1) for a in (-3, -1, 1, 3)] == [-1, 0, 1, 2]


def test_composition_reduces_to_the_row_function(oracle):
    """K = I and V = I with the identity rescale make the block the row-wise HCCS of Q,
    which has its own pins."""
    L = 32
    g = np.random.default_rng(11)
    q = g.integers(-128, 128, size=(2, 3, L, L), dtype=np.int8)
    eye = np.broadcast_to(np.eye(L, dtype=np.int8), q.shape).copy()
    table = synth.head_params(3, L, 1, seed=5)
    rq = np.array([[4096, 12]] * 3, np.int32)
    o, rc = oracle.attention(q, eye, eye, table, rq, 1)
    p, rc2 = oracle.softmax(q, table, 1)
    assert rc == 0 and rc2 == 0
    assert np.array_equal(o, p.astype(np.int32))


def test_all_ones_values_give_row_sums(oracle):
    L, d = 48, 8
    q, k, _ = _qkv(2, (1, 2, L, d))
    v = np.ones((1, 2, L, d), np.int8)
    table = synth.head_params(2, L, 1, seed=8)
    rq = synth.requant_params(2, seed=8, shift=10)
    o, rc = oracle.attention(q, k, v, table, rq, 1)
    assert rc == 0
    assert np.all(o <= 255) and np.all(o >= 255 - L)
    assert np.all(o == o[..., :1])


@pytest.mark.parametrize("shape,band", [((2, 3, 16, 8), 1), ((1, 2, 64, 64), 1), ((1, 1, 40, 24), 0)])
def test_stages_against_library_matmul(oracle, shape, band):
    q, k, v = _qkv(sum(shape), shape)
    H, L = shape[1], shape[2]
    table = synth.head_params(H, L, band, seed=L)
    rq = synth.requant_params(H, seed=L, shift=12, mult_lo=20, mult_hi=60)
    o, rc = oracle.attention(q, k, v, table, rq, band, threads=2)
    assert rc == 0
    x, _ = oracle.requant_logits(q, k, rq)
    p, _ = oracle.softmax(x, table, band)
    want = np.matmul(p.astype(np.int64), v.astype(np.int64))
    assert np.array_equal(o.astype(np.int64), want)
    # and the big-integer version on one block
    b, h = shape[0] - 1, H - 1
    B, S, D = table[h].tolist()
    o_py = hccs_ref.attention(q[b, h].tolist(), k[b, h].tolist(), v[b, h].tolist(), B, S, D,
                              int(rq[h, 0]), int(rq[h, 1]))
    assert o[b, h].tolist() == o_py


def test_offset_identity_for_unsigned_probabilities(oracle):
    """P.V = (P-128).V + 128*colsum(V): the identity a signed-int8 matrix unit needs."""
    shape = (3, 1, 4, 16)
    q, k, v = _qkv(21, shape)
    table = np.array([[8000, 60, 127]], np.int32)         # strict band at n = 4, p can exceed 127
    rq = np.array([[40, 12]], np.int32)
    o, rc = oracle.attention(q, k, v, table, rq, 1)
    x, _ = oracle.requant_logits(q, k, rq)
    p, _ = oracle.softmax(x, table, 1)
    assert rc == 0 and p.max() > 127
    signed = p.astype(np.int64) - 128
    want = np.matmul(signed, v.astype(np.int64)) + 128 * v.astype(np.int64).sum(axis=-2, keepdims=True)
    assert np.array_equal(o.astype(np.int64), want)


def test_rectangular_blocks_against_library_matmul(oracle):
    """Lq != Lk: n = Lk for the row function and the band; each query row is independent."""
    g = np.random.default_rng(8)
    Bt, H, Lq, Lk, d = 2, 2, 5, 48, 16
    q = g.integers(-64, 64, size=(Bt, H, Lq, d), dtype=np.int8)
    k = g.integers(-64, 64, size=(Bt, H, Lk, d), dtype=np.int8)
    v = g.integers(-64, 64, size=(Bt, H, Lk, d), dtype=np.int8)
    table = synth.head_params(H, Lk, 1, seed=1)
    rq = synth.requant_params(H, seed=1, shift=11, mult_lo=20, mult_hi=60)
    o, rc = oracle.attention(q, k, v, table, rq, 1)
    x, rc2 = oracle.requant_logits(q, k, rq)
    assert rc == 0 and rc2 == 0 and x.shape == (Bt, H, Lq, Lk)
    p, _ = oracle.softmax(x, table, 1)
    assert np.array_equal(o.astype(np.int64), np.matmul(p.astype(np.int64), v.astype(np.int64)))
    # dropping query rows does not change the others
    o2, _ = oracle.attention(q[:, :, :2], k, v, table, rq, 1)
    assert np.array_equal(o2, o[:, :, :2])
