"""Pins for the oracle's gate and threshold calibration (not gpu): the integer form of the
vote-fraction test against exact rational arithmetic, set/ordering invariants, the least-
confidence closed form of Section 3.2, and Algorithm 1's quantile index rule on lists small
enough to index by hand."""
from fractions import Fraction
from math import ceil

import numpy as np
import pytest

import oracle


def test_vmin_is_exact_ceiling():
    # theta*T integer: 0.75*16 = 12 -> a flow with exactly 12 votes is kept, 11 escalates
    assert oracle.vmin_from_theta(0.75, 16) == 12
    top = np.array([11, 12, 13, 0, 16], np.uint16)
    esc = oracle.route(top, np.zeros(5, np.uint16), 12)
    assert esc.tolist() == [0, 3]
    # theta's binary32 value decides, not the decimal literal: float32(0.3) > 3/10, so with T=100
    # thirty votes are a fraction *below* theta and the flow escalates (vmin = 31)
    th = Fraction(float(np.float32(0.3)))
    assert th > Fraction(3, 10)
    assert oracle.vmin_from_theta(0.3, 100) == 31
    # float32(0.7) < 7/10: seventy votes of 100 are kept
    assert Fraction(float(np.float32(0.7))) < Fraction(7, 10)
    assert oracle.vmin_from_theta(0.7, 100) == 70
    for theta in (0.0, 0.1, 0.25, 1 / 3, 0.5, 0.62, 0.75, 0.9, 1.0):
        for T in (1, 7, 16, 100, 200, 500, 65535):
            exact = ceil(Fraction(float(np.float32(theta))) * T)
            assert oracle.vmin_from_theta(theta, T) == exact, (theta, T)


@pytest.mark.parametrize("T,C", [(16, 4), (100, 10)])
def test_gate_equals_rational_fraction_test(T, C):
    """escalated set = exactly the flows whose vote fraction top/T is below theta, the fraction
    taken as a rational number (never a rounded float)."""
    rng = np.random.default_rng(5)
    top = rng.integers(0, T + 1, size=5000).astype(np.uint16)
    pred = rng.integers(0, C, size=5000).astype(np.uint16)
    for theta in (0.1, 0.3, 0.5, 0.75, 0.9):
        thf = Fraction(float(np.float32(theta)))
        want = [i for i in range(5000) if Fraction(int(top[i]), T) < thf]
        got = oracle.route(top, pred, oracle.vmin_from_theta(theta, T))
        assert got.tolist() == want
        # least confidence LC = 1 - max P(y|x) with P = votes/T: escalate <=> LC > 1 - theta
        lc = [1 - Fraction(int(v), T) for v in top]
        assert got.tolist() == [i for i in range(5000) if lc[i] > 1 - thf]


def test_gate_extremes_order_and_partition():
    rng = np.random.default_rng(6)
    T = 50
    top = rng.integers(0, T + 1, size=3000).astype(np.uint16)
    pred = rng.integers(0, 8, size=3000).astype(np.uint16)
    assert oracle.route(top, pred, 0).size == 0
    assert oracle.route(top, pred, T + 1).tolist() == list(range(3000))
    esc = oracle.route(top, pred, 20)
    assert np.all(np.diff(esc.astype(np.int64)) > 0)
    kept = np.setdiff1d(np.arange(3000), esc)
    assert esc.size + kept.size == 3000
    assert np.all(top[esc] < 20) and np.all(top[kept] >= 20)
    assert oracle.route(np.zeros(0, np.uint16), np.zeros(0, np.uint16), 5).size == 0


def test_per_class_gate():
    top = np.array([5, 5, 5, 9, 9, 2], np.uint16)
    pred = np.array([0, 1, 2, 0, 2, 1], np.uint16)
    vmin = np.array([6, 5, 10], np.uint16)      # class 0: <6, class 1: <5, class 2: <10
    assert oracle.route(top, pred, vmin).tolist() == [0, 2, 4, 5]
    # equal per-class thresholds reduce to the universal gate
    rng = np.random.default_rng(7)
    t = rng.integers(0, 30, size=500).astype(np.uint16)
    p = rng.integers(0, 4, size=500).astype(np.uint16)
    assert np.array_equal(oracle.route(t, p, np.full(4, 11, np.uint16)), oracle.route(t, p, 11))


def test_universal_thresholds_index_rule():
    """Algorithm 1: thresholds are the sorted scores at position ceil(q*|U|), counted from one."""
    scores = [0.9, 0.1, 0.5, 0.3, 0.7, 0.2, 0.8, 0.4, 0.6, 1.0]      # sorted: 0.1 .. 1.0
    q = [0.01, 0.1, 0.11, 0.25, 0.5, 0.95, 0.99, 1.0]
    # |U| = 10: positions 1,1,2,3,5,10,10,10
    want = [0.1, 0.1, 0.2, 0.3, 0.5, 1.0, 1.0, 1.0]
    assert oracle.universal_thresholds(scores, q).tolist() == want
    # a threshold read at quantile q assigns at least a fraction 1-q... checked on ties too
    rng = np.random.default_rng(8)
    top = rng.integers(0, 17, size=1000)
    lc = 1.0 - top / 16.0                           # exact in binary64 (sixteenths)
    qs = np.linspace(0.01, 0.99, 99)
    th = oracle.universal_thresholds(lc, qs)
    srt = np.sort(lc)
    for qq, tt in zip(qs, th):
        assert tt == srt[ceil(Fraction(float(qq)) * 1000) - 1]
        assert (lc <= tt).mean() >= qq - 1e-12      # at least a fraction q scores at or below it
    with pytest.raises(ValueError):
        oracle.universal_thresholds([], [0.5])
