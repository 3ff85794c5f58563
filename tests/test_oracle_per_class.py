"""Pins for the oracle's slope-based per-class thresholds (Algorithm 2 of the paper) and, on the host,
the library's version of it on a histogram (not gpu)."""
import ctypes
from fractions import Fraction

import numpy as np
import pytest

import oracle
import synth


def _hand_case():
    # (class, top_votes, correct); n_trees = 4
    rows = [(0, 1, 0), (0, 1, 0), (0, 2, 1), (0, 2, 0), (0, 3, 1),
            (1, 1, 1), (1, 1, 0), (1, 2, 1), (1, 2, 1), (1, 3, 0)]
    a = np.array(rows)
    return a[:, 0].astype(np.uint16), a[:, 1].astype(np.uint16), a[:, 2].astype(bool)


def test_hand_worked_sequence():
    """class 0 candidates (v: correct, incorrect): 1: 0,2 (slope 1)   2: 1,1 (1/2)   3: 1,0 (0)
       class 1 candidates:                          1: 1,1 (1/2)      2: 2,0 (0)     3: 0,1 (1)
    10 flows.  target 0.3: class 0 v=1 (2 assigned), then 1/2 against 1/2 -> the lower class, class 0 v=2
    (4 assigned >= 3, stop).  target 0.5: next 0 against 1/2 -> class 1 v=1 (6 >= 5).  target 1: 0 against 0
    -> class 0 v=3, then class 1 v=2, v=3.  The slope-1 candidate of class 1 sits behind a slope-0 one and is
    reached last: a class's threshold only moves one way."""
    pred, top, corr = _hand_case()
    vmin, frac, taken = oracle.per_class_thresholds(pred, top, corr, 4, 2, 0.3)
    assert vmin.tolist() == [3, 0] and frac == 0.4 and taken == [(0, 1, 0, 2), (0, 2, 1, 1)]
    vmin, frac, taken = oracle.per_class_thresholds(pred, top, corr, 4, 2, 0.5)
    assert vmin.tolist() == [3, 2] and frac == 0.6 and taken[-1] == (1, 1, 1, 1)
    vmin, frac, taken = oracle.per_class_thresholds(pred, top, corr, 4, 2, 1.0)
    assert vmin.tolist() == [4, 4] and frac == 1.0
    assert [t[:2] for t in taken] == [(0, 1), (0, 2), (1, 1), (0, 3), (1, 2), (1, 3)]
    vmin, frac, taken = oracle.per_class_thresholds(pred, top, corr, 4, 2, 0.0)
    assert vmin.tolist() == [0, 0] and frac == 0.0 and taken == []


def _workload(n=30000, cfg_id=2):
    cfg = synth.get_config(cfg_id).scaled(n)
    pk = synth.make_packets(cfg)
    feat, _ = oracle.featurize(pk.flow_off, pk.pkt_size, pk.pkt_iat, pk.pkt_dir, cfg.depths, n_threads=8)
    _, pred, top, _ = oracle.fast_infer(feat, synth.make_forest(cfg, feat[:4096]), want_votes=False, n_threads=8)
    truth = synth.make_truth(cfg, pred, top)
    return cfg, pred, top, truth


def test_single_class_reduces_to_most_uncertain_first():
    """with one class the rule is the universal one: the smallest vote threshold that assigns the target"""
    cfg, pred, top, truth = _workload(8000)
    one = np.zeros_like(pred)
    corr = truth == pred
    for target in (0.05, 0.2, 0.5, 0.9):
        vmin, frac, _ = oracle.per_class_thresholds(one, top, corr, cfg.n_trees, 1, target)
        below = np.array([(top < v).sum() for v in range(cfg.n_trees + 2)])
        want = int(np.argmax(below >= target * top.size))
        assert int(vmin[0]) == want and frac == below[want] / top.size
        # and it is where Algorithm 1 puts the threshold: the element at quantile 1 - target of the ascending
        # uncertainty LC = 1 - top/T has LC >= 1 - (vmin - 1)/T
        lc = 1.0 - top / cfg.n_trees
        thr = oracle.universal_thresholds(lc, [1.0 - target])[0]
        assert thr >= 1.0 - (want - 1) / cfg.n_trees - 1e-12


def test_every_increment_takes_the_steepest_candidate():
    cfg, pred, top, truth = _workload()
    corr = truth == pred
    C, T, n = cfg.n_classes, cfg.n_trees, pred.size
    vmin, frac, taken = oracle.per_class_thresholds(pred, top, corr, T, C, 0.3)
    # replay with an independent table: H[c][v] = (correct, incorrect)
    H = np.zeros((C, T + 1, 2), np.int64)
    np.add.at(H, (pred.astype(int), top.astype(int), (~corr).astype(int)), 1)
    cur = [0] * C
    total = 0
    for (c, v, dc, di) in taken:
        assert total < 0.3 * n
        assert (H[c, v, 0], H[c, v, 1]) == (dc, di) and dc + di > 0
        assert H[c, cur[c]:v].sum() == 0                     # nothing skipped but empty vote counts
        mine = Fraction(di, dc + di)
        for o in range(C):                                  # no other class offers a steeper next candidate
            nz = np.flatnonzero(H[o, cur[o]:].sum(axis=1))
            if nz.size:
                w = cur[o] + nz[0]
                other = Fraction(int(H[o, w, 1]), int(H[o, w].sum()))
                assert other < mine or (other == mine and o >= c), (c, v, o, w)
        cur[c] = v + 1
        total += dc + di
    assert total >= 0.3 * n and cur == vmin.tolist() and frac == total / n
    # the gate with these thresholds assigns exactly those flows
    esc = oracle.route(top, pred, vmin)
    assert esc.size == total
    # and it collects more of the mistakes than the universal threshold that assigns at least as much
    uni = next(v for v in range(T + 2) if (top < v).sum() >= total)
    assert (~corr[esc]).sum() > (~corr[top < uni]).sum() * total / (top < uni).sum()


def test_monotone_in_the_target():
    cfg, pred, top, truth = _workload(12000)
    corr = truth == pred
    last, last_frac = np.zeros(cfg.n_classes, np.uint16), 0.0
    for target in (0.01, 0.05, 0.1, 0.3, 0.6, 1.0):
        vmin, frac, _ = oracle.per_class_thresholds(pred, top, corr, cfg.n_trees, cfg.n_classes, target)
        assert np.all(vmin >= last) and frac >= last_frac and frac >= min(target, 1.0) - 1e-12
        last, last_frac = vmin, frac
    assert last_frac == 1.0


# ---- the library's host function on a histogram -------------------------------------------------

@pytest.fixture(scope="module")
def lib():
    from paper_2402_03694_amd import binding, build
    if build.is_stale():
        build.build()
    return binding.load_library()


def _lib_thresholds(lib, hist, T, C, target):
    h = np.ascontiguousarray(hist, np.uint32)
    out = (ctypes.c_uint16 * C)()
    reached = ctypes.c_double()
    rc = lib.sf_per_class_thresholds(h.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32)), T, C, ctypes.c_double(target),
                                     out, ctypes.byref(reached))
    assert rc == 0
    return list(out), reached.value


def test_library_matches_oracle_on_histograms(lib):
    pred, top, corr = _hand_case()
    H = np.zeros((2, 5, 2), np.uint32)
    np.add.at(H, (pred.astype(int), top.astype(int), (~corr).astype(int)), 1)
    for target in (0.0, 0.3, 0.5, 1.0):
        want, frac, _ = oracle.per_class_thresholds(pred, top, corr, 4, 2, target)
        got, reached = _lib_thresholds(lib, H, 4, 2, target)
        assert got == want.tolist() and reached == frac
    for cfg_id, n in ((2, 20000), (4, 9000), (1, 4096)):
        cfg, pred, top, truth = _workload(n, cfg_id)
        corr = truth == pred
        C, T = cfg.n_classes, cfg.n_trees
        H = np.zeros((C, T + 1, 2), np.uint32)
        np.add.at(H, (pred.astype(int), top.astype(int), (~corr).astype(int)), 1)
        for target in (0.02, 0.1, 0.25, 0.5, 0.97):
            want, frac, _ = oracle.per_class_thresholds(pred, top, corr, T, C, target)
            got, reached = _lib_thresholds(lib, H, T, C, target)
            assert got == want.tolist() and abs(reached - frac) < 1e-15, (cfg_id, target)


def test_library_stops_exactly_at_the_target(lib):
    """target * n is compared without rounding: binary64(0.1) is a little above 1/10, so 3 of 30 assigned flows
    are not yet 0.1 of them, while 0.5 and 0.25 are exact"""
    H = np.zeros((1, 11, 2), np.uint32)
    H[0, 1:11, 0] = 3                                        # 30 flows, three per vote count
    pred = np.zeros(30, np.uint16)
    top = np.repeat(np.arange(1, 11), 3).astype(np.uint16)
    corr = np.ones(30, bool)
    for target in (0.1, 0.2, 0.3, 0.5, 0.25, 0.7, 0.9999999999999999, 1.0, 1e-300, 5e-324, 2.0):
        want, frac, _ = oracle.per_class_thresholds(pred, top, corr, 10, 1, target)
        got, reached = _lib_thresholds(lib, H, 10, 1, target)
        assert got == want.tolist() and reached == frac, target
    assert _lib_thresholds(lib, H, 10, 1, 0.1)[0] == [3]     # 3/30 < binary64(0.1): one more step
    assert _lib_thresholds(lib, H, 10, 1, 0.5)[0] == [6]


def test_library_rejects_bad_arguments(lib):
    out = (ctypes.c_uint16 * 2)()
    assert lib.sf_per_class_thresholds(None, 4, 2, ctypes.c_double(0.5), out, None) == -1
    h = (ctypes.c_uint32 * 20)()
    assert lib.sf_per_class_thresholds(h, 0, 2, ctypes.c_double(0.5), out, None) == -1
    assert lib.sf_per_class_thresholds(h, 4, 2, ctypes.c_double(0.5), out, None) == 0 and list(out) == [0, 0]
