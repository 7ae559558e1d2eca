"""Pins for the oracle's dyadic requantiser (Section 3.1, requantisation equation and DN)."""
import math
import random
from fractions import Fraction

import numpy as np
import pytest

import oracle
from helpers import rq_exact, dyadic_from_real
from conftest import read_golden


def test_rq_matches_exact_rationals_random():
    rnd = random.Random(11)
    ts, bs, cs = [], [], []
    for _ in range(20000):
        c = rnd.randint(1, 62)
        b = rnd.choice([rnd.randint(0, (1 << 31) - 1), rnd.randint(1 << 14, (1 << 15) - 1), 1, 0])
        t = rnd.choice([rnd.randint(-(1 << 31), (1 << 31) - 1), rnd.randint(-300, 300)])
        ts.append(t); bs.append(b); cs.append(c)
    got = oracle.rq(np.array(ts), np.array(bs), np.array(cs))
    for t, b, c, g in zip(ts, bs, cs, got):
        assert int(g) == rq_exact(t, b, c), (t, b, c)


def test_rq_adversarial_ties_and_extremes():
    cases = []
    for c in (1, 2, 7, 15, 20, 30, 31, 32, 33, 47, 62):
        for b in (1, 3, (1 << 14), (1 << 15) - 1, (1 << 31) - 1):
            for t in (0, 1, -1, (1 << 31) - 1, -(1 << 31), 12345, -12345):
                cases.append((t, b, c))
        # exact ties: t*b == (2j+1) * 2^(c-1)  -> choose b = 2^(c-1) when it fits, t odd
        if c - 1 <= 30:
            b = 1 << (c - 1)
            for t in (1, -1, 3, -3, 101, -101, (1 << 31) - 1, -(1 << 31) + 1):
                cases.append((t, b, c))
    t, b, c = (np.array(v) for v in zip(*cases))
    got = oracle.rq(t, b, c)
    for (ti, bi, ci), g in zip(cases, got):
        assert int(g) == rq_exact(ti, bi, ci), (ti, bi, ci)
    # ties go toward +infinity: 0.5 -> 1, -0.5 -> 0, -1.5 -> -1
    assert list(oracle.rq(np.array([1, -1, -3, 3]), 1, 1)) == [1, 0, -1, 2]


def test_rq_equals_rounding_of_dyadic_product():
    # invariant: rq(x) == round(x * b / 2^c) with half-up rounding, checked in float64 where exact
    g = np.random.default_rng(5)
    t = g.integers(-(1 << 27), 1 << 27, size=5000)
    b = g.integers(1 << 14, 1 << 15, size=5000)
    c = g.integers(20, 31, size=5000)
    got = oracle.rq(t, b, c)
    want = np.floor(t.astype(np.float64) * b / np.exp2(c) + 0.5)  # products < 2^42: exact in float64
    assert np.array_equal(got, want.astype(np.int64))


def test_dn_helper_error_bound_and_requant_within_one():
    rnd = random.Random(3)
    for _ in range(2000):
        s = math.exp(rnd.uniform(math.log(2.0 ** -16), math.log(2.0 ** -5)))
        b, c = dyadic_from_real(s)
        assert (1 << 14) <= b < (1 << 15)
        assert abs(Fraction(b, 2 ** c) - Fraction(s)) <= Fraction(s) / (1 << 15)
        t = rnd.randint(-(1 << 20), 1 << 20)
        exact = math.floor(Fraction(t) * Fraction(s) + Fraction(1, 2))  # Int(t*s)
        got = int(oracle.rq(np.array([t]), b, c)[0])
        assert abs(got - exact) <= 1
        # they can differ only when t*s is within |t| s 2^-15 of a rounding boundary
        if got != exact:
            frac = (Fraction(t) * Fraction(s)) % 1
            assert abs(frac - Fraction(1, 2)) <= abs(t) * Fraction(s) / (1 << 15)


def test_residual_rounding_example_from_paper(golden_dir):
    """Appendix G: rounding each branch and then adding gives 6 where FP accumulation gives 7."""
    gold = read_golden(golden_dir + "/residual_rounding_example.txt")
    m, r, S_a = gold["m"], gold["r"], gold["S_a"]
    assert math.floor((m + r) / S_a + 0.5) == gold["fake_quant_result"]
    # integer-only: the two branches arrive as integers Int(m/S_a), Int(r/S_a); unit dyadic multipliers
    qm, qr = math.floor(m / S_a + 0.5), math.floor(r / S_a + 0.5)
    b, c = dyadic_from_real(1.0)
    y = oracle.residual_add_dyadic(np.array([qm], dtype=np.int32), [b], [c], np.array([qr], dtype=np.uint8), [b], [c],
                                   n_pixels=1, K=1, m_dt=oracle.S32, r_dt=oracle.U8, y_dt=oracle.U8,
                                   relu=1, y_lo=0, y_hi=127)
    assert int(y[0, 0]) == gold["integer_only_result"]
    # and with real scales: branches at scale 0.1 hold 44 and 24; DN(0.1/1) applied to each, separately rounded
    b2, c2 = dyadic_from_real(0.1)
    y = oracle.residual_add_dyadic(np.array([44], dtype=np.int32), [b2], [c2], np.array([24], dtype=np.uint8), [b2], [c2],
                                   n_pixels=1, K=1, m_dt=oracle.S32, r_dt=oracle.U8, y_dt=oracle.U8,
                                   relu=1, y_lo=0, y_hi=127)
    assert int(y[0, 0]) == gold["integer_only_result"]
