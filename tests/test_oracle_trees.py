"""Pins for the oracle's tree ensemble and vote scoring (not gpu)."""
import os
from fractions import Fraction
from math import factorial
from types import SimpleNamespace

import numpy as np
import pytest

import oracle
import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "trees_handtraced.txt")
FLT_MAX = np.finfo(np.float32).max


def _forest(trees, n_classes, n_features):
    d = trees[0][0]
    return SimpleNamespace(
        n_trees=len(trees), depth=d, n_classes=n_classes, n_features=n_features,
        node_feat=np.array([t[1] for t in trees], np.uint16),
        node_thr=np.array([t[2] for t in trees], np.float32),
        leaf_label=np.array([t[3] for t in trees], np.uint8))


def test_handtraced_trees():
    trees, samples, C = [], [], None
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        if line.startswith("classes"):
            C = int(line.split()[1])
        elif line.startswith("tree"):
            d, f, th, lab = [p.split() for p in line[4:].split("|")]
            trees.append((int(d[0]), [int(v) for v in f], [float(v) for v in th], [int(v) for v in lab]))
        elif line.startswith("x"):
            xs, rest = line[1:].split("->")
            leaves, votes, pt = [p.split() for p in rest.split("|")]
            samples.append(([float(v) for v in xs.split()], [int(v) for v in leaves],
                            [int(v) for v in votes], int(pt[0]), int(pt[1])))
    forest = _forest(trees, C, 2)
    feat = np.array([s[0] for s in samples], np.float32)
    votes, pred, top, leaves = oracle.fast_infer(feat, forest, want_leaves=True)
    assert leaves.tolist() == [s[1] for s in samples]
    assert votes.tolist() == [s[2] for s in samples]
    assert pred.tolist() == [s[3] for s in samples]
    assert top.tolist() == [s[4] for s in samples]


@pytest.mark.parametrize("d", [1, 3, 8, 12])
def test_extreme_thresholds_and_equality(d):
    n_int = (1 << d) - 1
    x = np.array([[0.0, 1.5], [-3.0, 2.0]], np.float32)
    labels = list(np.arange(1 << d) % 5)
    left = _forest([(d, [0] * n_int, [FLT_MAX] * n_int, labels)], 5, 2)
    right = _forest([(d, [1] * n_int, [-FLT_MAX] * n_int, labels)], 5, 2)
    assert oracle.fast_infer(x, left, want_leaves=True)[3].ravel().tolist() == [0, 0]
    assert oracle.fast_infer(x, right, want_leaves=True)[3].ravel().tolist() == [(1 << d) - 1] * 2
    # a value exactly equal to the threshold goes left, the next float up goes right
    eq = _forest([(d, [1] * n_int, [1.5] * n_int, labels)], 5, 2)
    up = np.array([[0.0, np.nextafter(np.float32(1.5), np.float32(2))]], np.float32)
    assert oracle.fast_infer(x[:1], eq, want_leaves=True)[3][0, 0] == 0
    assert oracle.fast_infer(up, eq, want_leaves=True)[3][0, 0] == (1 << d) - 1


def _walk_recursive(x, nf, nt, k, n_int):
    """Brute force: explicit recursion over child links instead of the heap-index update."""
    if k >= n_int:
        return k - n_int
    child = 2 * k + 1 if x[nf[k]] <= nt[k] else 2 * k + 2
    return _walk_recursive(x, nf, nt, child, n_int)


def test_recursive_walk_on_random_forest():
    cfg = synth.get_config(1)
    pk = synth.make_packets(cfg, n_flows=64)
    feat, _ = oracle.featurize(pk.flow_off, pk.pkt_size, pk.pkt_iat, pk.pkt_dir, cfg.depths)
    forest = synth.make_forest(cfg, feat)
    votes, pred, top, leaves = oracle.fast_infer(feat, forest, want_leaves=True)
    n_int = (1 << forest.depth) - 1
    for i in range(64):
        exp_votes = np.zeros(cfg.n_classes, int)
        for t in range(forest.n_trees):
            leaf = _walk_recursive(feat[i], forest.node_feat[t], forest.node_thr[t], 0, n_int)
            assert leaves[i, t] == leaf
            exp_votes[forest.leaf_label[t, leaf]] += 1
        assert votes[i].tolist() == exp_votes.tolist()
        assert top[i] == exp_votes.max() and pred[i] == int(np.argmax(exp_votes))
    assert np.all(votes.sum(axis=1) == forest.n_trees)


def test_constant_leaf_labels():
    cfg = synth.get_config(1)
    pk = synth.make_packets(cfg, n_flows=32)
    feat, _ = oracle.featurize(pk.flow_off, pk.pkt_size, pk.pkt_iat, pk.pkt_dir, cfg.depths)
    forest = synth.make_forest(cfg, feat)
    forest.leaf_label[:] = 3
    votes, pred, top, _ = oracle.fast_infer(feat, forest)
    assert np.all(pred == 3) and np.all(top == 16) and np.all(votes[:, 3] == 16)
    assert np.all(votes.sum(axis=1) == 16)


def test_rejects_out_of_range_model():
    f = _forest([(1, [2], [0.0], [0, 1])], 2, 2)
    with pytest.raises(ValueError):
        oracle.fast_infer(np.zeros((1, 2), np.float32), f)
    f = _forest([(1, [0], [0.0], [0, 2])], 2, 2)
    with pytest.raises(ValueError):
        oracle.fast_infer(np.zeros((1, 2), np.float32), f)


def _multinomial_max_cdf(T, C):
    """P(max vote <= m) for T independent uniform votes over C classes, exactly:
    T!/C^T * [x^T] (sum_{j<=m} x^j/j!)^C."""
    out = []
    for m in range(T + 1):
        base = [Fraction(1, factorial(j)) for j in range(m + 1)]
        poly = [Fraction(1)]
        for _ in range(C):
            new = [Fraction(0)] * min(T + 1, len(poly) + m)
            for a, pa in enumerate(poly):
                if pa == 0:
                    continue
                for b, pb in enumerate(base):
                    if a + b <= T and a + b < len(new):
                        new[a + b] += pa * pb
            poly = new
        coef = poly[T] if T < len(poly) else Fraction(0)
        out.append(float(coef * factorial(T) / Fraction(C) ** T))
    return np.array(out)


def test_top_vote_histogram_matches_multinomial():
    """Leaf labels are independent uniform draws, so a flow's votes are Multinomial(T; 1/C...)
    whatever its features; the top-vote histogram must follow the closed form."""
    cfg = synth.get_config(1)
    n = 4096
    pk = synth.make_packets(cfg, n_flows=n)
    feat, _ = oracle.featurize(pk.flow_off, pk.pkt_size, pk.pkt_iat, pk.pkt_dir, cfg.depths)
    forest = synth.make_forest(cfg, feat)
    _, _, top, _ = oracle.fast_infer(feat, forest)
    cdf = _multinomial_max_cdf(16, 4)
    pmf = np.diff(np.concatenate([[0.0], cdf]))
    hist = np.bincount(top, minlength=17) / n
    # flows share trees, so counts are correlated; allow 5 binomial standard errors + slack
    tol = 5 * np.sqrt(pmf * (1 - pmf) / n) + 0.02
    assert np.all(np.abs(hist - pmf) <= tol), (hist, pmf)
    assert abs(float((top * 1.0).mean()) - float((np.arange(17) * pmf).sum())) < 0.25
