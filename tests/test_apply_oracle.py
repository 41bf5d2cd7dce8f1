"""Pins of the per-element oracle (Sec. 3.3 experiment): hand-worked values that
need both roundings, identities, and exactness on dyadic inputs against rational
arithmetic."""
import os
from fractions import Fraction

import numpy as np

import oracle
from paper_1606_04884_amd import synth

HERE = os.path.dirname(os.path.abspath(__file__))


def test_hand_worked_values():
    rows = [l.split() for l in open(os.path.join(HERE, "golden", "apply_mul_add.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 4
    for a, b, x, y in rows:
        got = oracle.apply_mul_add(np.array([float(x)], dtype=np.float32), float(a), float(b))
        assert got.dtype == np.float32 and got[0] == np.float32(float(y)), (a, b, x, y, got)


def test_identities():
    x = synth.normal((1000,), 11)
    assert np.array_equal(oracle.apply_mul_add(x, 1.0, 0.0), x)
    assert np.array_equal(oracle.apply_mul_add(x, 0.0, 2.5), np.full_like(x, 2.5))
    assert np.array_equal(oracle.apply_mul_add(x, -1.0, 0.0), -x)
    assert np.array_equal(oracle.apply_mul_add(x, 2.0, 0.0), x + x)


def test_exact_on_dyadic_inputs():
    # small dyadic values: a*x + b is exactly representable, so the result must equal
    # the rational value whatever the rounding order
    x = synth.dyadic((257,), 5)
    a, b = 0.375, -1.25
    got = oracle.apply_mul_add(x, a, b)
    for xi, yi in zip(x, got):
        assert Fraction(float(yi)) == Fraction(a) * Fraction(float(xi)) + Fraction(b)


def test_empty():
    assert oracle.apply_mul_add(np.zeros((0,), dtype=np.float32), 2.0, 1.0).shape == (0,)
