"""Threshold calibration of the library (Algorithm 1 on the score histogram, target-portion rule)
against the oracle and brute force.  The host parts need no GPU; the device histogram does."""
from fractions import Fraction
from math import ceil

import numpy as np
import pytest

import oracle


@pytest.fixture(scope="module")
def sf():
    from paper_2402_03694_amd import build
    if build.is_stale():
        build.build()
    import paper_2402_03694_amd as m
    return m


@pytest.mark.parametrize("T,n,seed", [(16, 1000, 0), (100, 5000, 1), (500, 777, 2), (7, 13, 3)])
def test_universal_thresholds_match_oracle(sf, T, n, seed):
    """Algorithm 1 on LC = 1 - top/T: the oracle sorts the scores, the library walks the histogram."""
    rng = np.random.default_rng(seed)
    top = rng.binomial(T, 0.3, size=n).astype(np.uint16)
    hist = np.bincount(top, minlength=T + 1)
    qs = np.concatenate([np.linspace(0.01, 0.99, 99), [1e-9, 1.0, 0.5 + 1e-12]])
    got = sf.sf_universal_thresholds(hist, T, qs)
    lc = 1.0 - top.astype(np.float64) / T
    want = oracle.universal_thresholds(lc, qs)
    assert np.array_equal(1.0 - np.array(got, np.float64) / T, want)
    # the gate vmin = that vote count assigns at most a fraction 1 - q
    for q, v in zip(qs, got):
        assert (top < v).mean() <= 1 - q + 1e-12


def test_universal_thresholds_index_rule_by_hand(sf):
    # scores sorted ascending = votes descending 9 9 8 5 5 5 2 0 (|U| = 8); position ceil(q*8)
    hist = [1, 0, 1, 0, 0, 3, 0, 0, 1, 2]
    assert sf.sf_universal_thresholds(hist, 9, [0.01, 0.25, 0.26, 0.5, 0.75, 0.76, 0.99]) == [9, 9, 8, 5, 5, 2, 0]
    with pytest.raises(sf.ServeFlowError):
        sf.sf_universal_thresholds([0] * 10, 9, [0.5])


@pytest.mark.parametrize("T,seed", [(16, 0), (100, 1), (200, 2)])
def test_vmin_for_target_bruteforce(sf, T, seed):
    rng = np.random.default_rng(seed)
    top = rng.binomial(T, 0.2, size=4000).astype(np.uint16)
    hist = np.bincount(top, minlength=T + 1)
    n = top.size
    for target in (0.0, 0.05, 0.2, 0.25, 0.5, 0.9, 1.0):
        fr = [Fraction(int((top < v).sum()), n) for v in range(T + 2)]
        tf = Fraction(target)
        best = min(range(T + 2), key=lambda v: (abs(fr[v] - tf), fr[v], v))
        got, reached = sf.sf_vmin_for_target(hist, T, target)
        assert fr[got] == fr[best], (target, got, best)          # same escalated set (equal fractions)
        assert abs(reached - float(fr[best])) < 1e-12


def test_vmin_for_target_tie_takes_smaller_fraction(sf):
    # fractions reachable: 0, 0.25, 0.75, 1.0; target 0.5 is equally far from 0.25 and 0.75
    got, reached = sf.sf_vmin_for_target([1, 2, 1], 2, 0.5)
    assert got == 1 and reached == 0.25


@pytest.mark.gpu
@pytest.mark.parametrize("T,n", [(16, 1), (100, 100003), (500, 1 << 20), (10000, 50000), (65535, 70000)])
def test_score_histogram_on_device(sf, T, n):
    import torch
    rng = np.random.default_rng(T + n)
    top = rng.integers(0, T + 1, size=n).astype(np.uint16)
    ctx = sf.ServeFlow(sf.sf_workspace_bytes(n, 100, 10) + 4 * (T + 1))
    d_top = torch.from_numpy(top.view(np.int16)).cuda()
    hist = ctx.sf_score_histogram(d_top, T)
    assert hist == np.bincount(top, minlength=T + 1).tolist()
    assert ctx.sf_score_histogram(d_top[:0], T, n_flows=0) == [0] * (T + 1)


@pytest.mark.gpu
def test_per_class_thresholds_end_to_end(sf):
    """Algorithm 2: class-by-score histogram on the device, slope search on the host, then the per-class
    gate; every stage against the oracle on the same validation flows."""
    import torch
    import synth
    cfg = synth.get_config(2).scaled(40000 + 9)
    pk = synth.make_packets(cfg)
    feat, _ = oracle.featurize(pk.flow_off, pk.pkt_size, pk.pkt_iat, pk.pkt_dir, cfg.depths, n_threads=8)
    forest = synth.make_forest(cfg, feat[:4096])
    _, pred, top, _ = oracle.fast_infer(feat, forest, want_votes=False, n_threads=8)
    truth = synth.make_truth(cfg, pred, top)
    n, C, T = pred.size, cfg.n_classes, cfg.n_trees
    ctx = sf.ServeFlow(sf.sf_workspace_bytes(n))
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to("cuda:0")
    d_top, d_pred, d_truth = dev(top), dev(pred), dev(truth)
    hist = ctx.sf_class_score_histogram(d_top, d_pred, d_truth, T, C)
    want_h = np.zeros((C, T + 1, 2), np.int64)
    np.add.at(want_h, (pred.astype(int), top.astype(int), (pred != truth).astype(int)), 1)
    assert np.array_equal(np.array(hist, np.int64).reshape(C, T + 1, 2), want_h)
    esc = torch.full((n,), -1, dtype=torch.int32, device="cuda:0")
    cnt = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    for target in (0.05, 0.25, 0.5):
        vmin, reached = sf.sf_per_class_thresholds(hist, T, C, target)
        o_vmin, o_frac, _ = oracle.per_class_thresholds(pred, top, truth == pred, T, C, target)
        assert vmin == o_vmin.tolist() and reached == o_frac
        ctx.sf_route(d_top, d_pred, vmin, esc, cnt)
        torch.cuda.synchronize()
        want = oracle.route(top, pred, o_vmin)
        k = int(cnt.cpu().numpy().view(np.uint32)[0])
        assert k == want.size == round(reached * n)
        assert np.array_equal(esc.cpu().numpy().view(np.uint32)[:k], want)
    # an empty batch gives an all-zero histogram without touching the device
    assert sum(ctx.sf_class_score_histogram(d_top, d_pred, d_truth, T, C, n_flows=0)) == 0
