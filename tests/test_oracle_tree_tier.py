"""Pins for the oracle's first tier: a single decision tree with class counts at the leaves
and the least-confidence gate on the leaf distribution (not gpu)."""
import os
from fractions import Fraction
from types import SimpleNamespace

import numpy as np
import pytest

import oracle
import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "tree_tier_handtraced.txt")


def _tree(depth, feat, thr, counts, n_features):
    counts = np.asarray(counts, np.uint16)
    return SimpleNamespace(depth=depth, n_classes=counts.shape[1], n_features=n_features,
                           node_feat=np.asarray(feat, np.uint16), node_thr=np.asarray(thr, np.float32),
                           leaf_count=counts)


def test_handtraced_tree_and_gate():
    tree, xs, want, gates = None, [], [], []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#") or line.startswith("classes"):
            continue
        if line.startswith("tree"):
            d, f, th, cnt = line[4:].split("|")
            counts = [[int(v) for v in leaf.split()] for leaf in cnt.split(",")]
            tree = _tree(int(d), [int(v) for v in f.split()], [float(v) for v in th.split()], counts, 2)
        elif line.startswith("x"):
            a, b = line[1:].split("->")
            xs.append([float(v) for v in a.split()])
            want.append([int(v) for v in b.split()])
        elif line.startswith("theta"):
            a, b = line[5:].split("->")
            gates.append((float(a), [int(v) for v in b.split()]))
    pred, top, tot, leaf = oracle.tree_infer(np.array(xs, np.float32), tree, want_leaves=True)
    got = np.stack([leaf, pred, top, tot], axis=1).tolist()
    assert got == want
    assert len(gates) == 7
    for theta, esc in gates:
        assert float(np.float32(theta)) == theta          # the fixture spells binary32 values out
        assert oracle.route_ratio(top, tot, theta).tolist() == esc, theta


def _floor_f32(t64):
    """largest binary32 <= t64: for a binary32 x, x <= t64 iff x <= that value"""
    t = np.float32(t64)
    return np.nextafter(t, np.float32(-np.inf)) if float(t) > t64 else t


def _perfect_from_sklearn(sk, depth, n_classes):
    """Re-express a fitted scikit-learn tree as a perfect heap-ordered tree of the given depth:
    below a leaf that sits higher up, every split sends everything left (threshold +inf) and
    every leaf of the padding carries the leaf's counts."""
    n_int, n_leaf = (1 << depth) - 1, 1 << depth
    feat = np.zeros(n_int, np.uint16)
    thr = np.full(n_int, np.inf, np.float32)
    counts = np.zeros((n_leaf, n_classes), np.uint16)
    node_counts = np.rint(sk.value[:, 0, :] * sk.weighted_n_node_samples[:, None]).astype(np.int64)

    def place(node, k, level):
        if level == depth:
            assert sk.children_left[node] == -1
            counts[k - n_int] = node_counts[node]
            return
        if sk.children_left[node] == -1:
            place(node, 2 * k + 1, level + 1)      # padding: thr = +inf, always left
            place(node, 2 * k + 2, level + 1)
            return
        feat[k] = sk.feature[node]
        thr[k] = _floor_f32(sk.threshold[node])
        place(sk.children_left[node], 2 * k + 1, level + 1)
        place(sk.children_right[node], 2 * k + 2, level + 1)

    place(0, 0, 0)
    return feat, thr, counts


@pytest.mark.parametrize("depth,n_classes,seed", [(3, 2, 0), (6, 5, 1), (9, 12, 2)])
def test_matches_scikit_learn_decision_tree(depth, n_classes, seed):
    """A decision tree fitted by scikit-learn, whose leaves keep at least 15 training samples
    (Section 4.1): its predict_proba is the class share of the leaf's samples and its predict the
    first arg-max.  The oracle on the same tree must give the same leaf distribution and label."""
    from sklearn.tree import DecisionTreeClassifier
    rng = np.random.default_rng(seed)
    X = rng.normal(size=(6000, 7)).astype(np.float32)
    y = (np.floor(np.abs(X[:, 0] * 2 + X[:, 3] - X[:, 5] * X[:, 1]) * 1.7) % n_classes).astype(np.int64)
    noisy = rng.random(6000) < 0.2
    y[noisy] = rng.integers(0, n_classes, size=int(noisy.sum()))
    clf = DecisionTreeClassifier(max_depth=depth, min_samples_leaf=15, random_state=seed).fit(X, y)
    assert clf.n_classes_ == n_classes
    feat, thr, counts = _perfect_from_sklearn(clf.tree_, depth, n_classes)
    tree = _tree(depth, feat, thr, counts, 7)
    Xt = rng.normal(size=(4000, 7)).astype(np.float32)
    Xt[:200] = X[:200]
    # put some test values exactly on thresholds (the <= side must agree)
    for j in range(min(64, feat.size)):
        if np.isfinite(thr[j]):
            Xt[200 + j, feat[j]] = thr[j]
    pred, top, tot, _ = oracle.tree_infer(Xt, tree)
    proba = clf.predict_proba(Xt)
    assert np.array_equal(pred, clf.predict(Xt).astype(np.uint16))
    assert np.all(tot >= 15)
    assert np.allclose(top / tot, proba.max(axis=1), rtol=0, atol=1e-12)
    # the whole distribution, through the leaf index
    _, _, _, leaf = oracle.tree_infer(Xt, tree, want_leaves=True)
    assert np.allclose(counts[leaf] / tot[:, None], proba, rtol=0, atol=1e-12)


def test_ratio_gate_is_exact_rational_arithmetic():
    rng = np.random.default_rng(7)
    tot = rng.integers(1, 65536, size=4000).astype(np.uint16)
    top = (rng.random(4000) * (tot.astype(np.float64) + 1)).astype(np.uint16)
    top = np.minimum(top, tot)
    thetas = [0.5, 0.3, 0.1, 1 / 3, 2 / 3, 0.999999, 1.0, 1e-30, 3e-39, 1e30, 0.0, -0.25, 6e-8, 65535.0, 1.5e-5]
    # ratios that sit exactly on, just below and just above representable thresholds
    for theta in thetas:
        t32 = np.float32(theta)
        exact = Fraction(float(t32))
        want = [i for i in range(tot.size) if t32 > 0 and Fraction(int(top[i]), int(tot[i])) < exact]
        assert oracle.route_ratio(top, tot, t32).tolist() == want, theta
    # knife edges: top/total equal to theta exactly must not escalate, one ulp more must
    for num, den in [(1, 2), (3, 4), (5, 8), (1, 1), (12345, 32768)]:
        t = np.float32(num / den)
        assert float(t) == num / den
        a = np.array([num], np.uint16), np.array([den], np.uint16)
        assert oracle.route_ratio(*a, t).size == 0
        assert oracle.route_ratio(*a, np.nextafter(t, np.float32(2))).size == 1
        assert oracle.route_ratio(*a, np.nextafter(t, np.float32(0))).size == 0


def test_leaf_without_samples_escalates():
    top, tot = np.array([0, 0, 3], np.uint16), np.array([0, 5, 5], np.uint16)
    assert oracle.route_ratio(top, tot, 0.5).tolist() == [0, 1]
    assert oracle.route_ratio(top, tot, 1e-20).tolist() == [0, 1]
    assert oracle.route_ratio(top, tot, 0.0).tolist() == []


def test_one_hot_leaves_reduce_to_the_forest_with_one_tree():
    cfg = synth.get_config(1)
    pk = synth.make_packets(cfg, n_flows=512)
    feat, _ = oracle.featurize(pk.flow_off, pk.pkt_size, pk.pkt_iat, pk.pkt_dir, cfg.depths)
    forest = synth.make_forest(cfg, feat)
    for t in range(3):
        one = SimpleNamespace(n_trees=1, depth=forest.depth, n_classes=forest.n_classes, n_features=forest.n_features,
                              node_feat=forest.node_feat[t:t + 1], node_thr=forest.node_thr[t:t + 1],
                              leaf_label=forest.leaf_label[t:t + 1])
        _, f_pred, f_top, f_leaf = oracle.fast_infer(feat, one, want_leaves=True)
        counts = np.zeros((1 << forest.depth, forest.n_classes), np.uint16)
        counts[np.arange(1 << forest.depth), forest.leaf_label[t]] = 23
        tree = _tree(forest.depth, forest.node_feat[t], forest.node_thr[t], counts, forest.n_features)
        pred, top, tot, leaf = oracle.tree_infer(feat, tree, want_leaves=True)
        assert np.array_equal(pred, f_pred) and np.array_equal(leaf, f_leaf[:, 0])
        assert np.all(top == 23) and np.all(tot == 23) and np.all(f_top == 1)


def test_rejects_bad_trees():
    counts = np.full((4, 2), 40000, np.uint16)      # a leaf total that does not fit 16 bits
    with pytest.raises(ValueError):
        oracle.tree_infer(np.zeros((1, 2), np.float32), _tree(2, [0, 0, 0], [0, 0, 0], counts, 2))
    with pytest.raises(ValueError):                  # split feature outside the row
        oracle.tree_infer(np.zeros((1, 2), np.float32), _tree(2, [0, 2, 0], [0, 0, 0], counts // 4, 2))


def test_cascade_composition():
    """Three tiers (Section 3.1): every flow ends with the label of the last tier that saw it."""
    cfg = synth.get_config(6).scaled(3000)
    pk = synth.make_packets(cfg)
    feat, _ = oracle.featurize(pk.flow_off, pk.pkt_size, pk.pkt_iat, pk.pkt_dir, cfg.depths)
    tree, forest, mlp = synth.make_tree(cfg, feat), synth.make_forest(cfg, feat), synth.make_mlp(cfg, feat)
    assert tree.leaf_count.sum(axis=1).min() >= 15
    assert int(forest.node_feat.max()) < cfg.tree0_features and int(tree.node_feat.max()) < cfg.tree0_features
    r = oracle.classify3(pk, cfg.depths, tree, cfg.theta0, forest, cfg.vmin, mlp)
    n = cfg.n_flows
    e1, e2 = r["esc1"], r["esc2"]
    assert 0.2 < e1.size / n < 0.8 and 0 < e2.size < e1.size
    assert np.all(np.diff(e1.astype(np.int64)) > 0) and np.all(np.diff(e2.astype(np.int64)) > 0)
    assert np.all(np.isin(e2, e1))
    # the gate of tier 1 restated per flow in floating point on values where rounding cannot matter
    frac = r["top0"] / r["total0"]
    far = np.abs(frac - cfg.theta0) > 1e-6
    assert np.array_equal(np.isin(np.arange(n), e1)[far], (frac < cfg.theta0)[far])
    only0 = np.setdiff1d(np.arange(n), e1)
    only1 = np.setdiff1d(e1, e2)
    assert np.array_equal(r["labels"][only0], r["pred0"][only0])
    pos = np.searchsorted(e1, only1)
    assert np.array_equal(r["labels"][only1], r["pred1"][pos])
    assert np.array_equal(r["labels"][e2], r["logits"].argmax(axis=1).astype(np.uint16))
    # the forest tier on the subset is the forest on those rows, nothing else
    _, p_all, t_all, _ = oracle.fast_infer(feat, forest)
    assert np.array_equal(r["pred1"], p_all[e1]) and np.array_equal(r["top1"], t_all[e1])
