"""Pins for the oracle's boosted-tree fast model and its uncertainty scores (not gpu)."""
import math
from types import SimpleNamespace

import numpy as np
import pytest

import oracle
import synth


def _model(depth, n_classes, n_features, feat, thr, leaf_value, base):
    feat, thr, leaf_value = np.asarray(feat, np.uint16), np.asarray(thr, np.float32), np.asarray(leaf_value, np.float32)
    return SimpleNamespace(n_trees=feat.shape[0], depth=depth, n_classes=n_classes, n_features=n_features,
                           node_feat=feat, node_thr=thr, leaf_value=leaf_value,
                           base=None if base is None else np.asarray(base, np.float32))


def test_hand_worked_two_class_model():
    """depth-1 trees, 2 classes: tree 0 (class 0) x0 <= 0 -> +1 else -1; tree 1 (class 1) x1 <= 0 -> +0.25 else +2;
    initial margins (0.5, -0.5).  A 2-class softmax is the logistic function of the margin difference."""
    m = _model(1, 2, 2, [[0], [1]], [[0.0], [0.0]], [[1.0, -1.0], [0.25, 2.0]], [0.5, -0.5])
    x = np.array([[-1, 1], [1, -1], [0, 0]], np.float32)
    margins, pred, lc, ent = oracle.gbdt_infer(x, m)
    # flow 0: m = (0.5 + 1, -0.5 + 2) = (1.5, 1.5): a tie -> class 0, P = (1/2, 1/2)
    # flow 1: m = (0.5 - 1, -0.5 + 0.25) = (-0.5, -0.25) -> class 1
    # flow 2: both tests hold with equality -> left leaves: m = (1.5, -0.25) -> class 0
    assert margins.tolist() == [[1.5, 1.5], [-0.5, -0.25], [1.5, -0.25]]
    assert pred.tolist() == [0, 1, 0]
    assert lc[0] == 0.5 and abs(ent[0] - math.log(2.0)) < 1e-15
    for i, d in ((1, 0.25), (2, 1.75)):
        p = 1.0 / (1.0 + math.exp(-d))               # probability of the winning class
        assert abs(lc[i] - (1.0 - p)) < 1e-15
        assert abs(ent[i] + p * math.log(p) + (1 - p) * math.log(1 - p)) < 1e-15


def test_margin_sum_is_sequential_binary32():
    """1e8 + 1 - 1e8 is 0 when added left to right in binary32 and 1 in any wider or reordered sum:
    rounds 0, 1, 2 of class 0 contribute 1e8, 1, -1e8; class 1 gets them in the order 1e8, -1e8, 1."""
    vals0, vals1 = [1e8, 1.0, -1e8], [1e8, -1e8, 1.0]
    leaf = np.zeros((6, 2), np.float32)
    for r in range(3):
        leaf[2 * r] = vals0[r]
        leaf[2 * r + 1] = vals1[r]
    m = _model(1, 2, 1, [[0]] * 6, [[0.0]] * 6, leaf, None)
    margins, pred, _, _ = oracle.gbdt_infer(np.zeros((1, 1), np.float32), m)
    assert margins.tolist() == [[0.0, 1.0]] and pred.tolist() == [1]
    # and the initial margin comes first: 1e8 (base) + 1 - 1e8 = 0, not 1
    m2 = _model(1, 2, 1, [[0]] * 4, [[0.0]] * 4, [[1, 1], [0, 0], [-1e8, -1e8], [0, 0]], [1e8, 0.0])
    assert oracle.gbdt_infer(np.zeros((1, 1), np.float32), m2)[0].tolist() == [[0.0, 0.0]]


def test_scores_match_scipy_softmax_and_entropy():
    from scipy.special import softmax
    from scipy.stats import entropy
    cfg = synth.get_config(7).scaled(2000)
    pk = synth.make_packets(cfg)
    feat, _ = oracle.featurize(pk.flow_off, pk.pkt_size, pk.pkt_iat, pk.pkt_dir, cfg.depths)
    model = synth.make_gbdt(cfg, feat)
    margins, pred, lc, ent = oracle.gbdt_infer(feat, model)
    p = softmax(margins.astype(np.float64), axis=1)
    assert np.allclose(lc, 1.0 - p.max(axis=1), rtol=0, atol=1e-14)
    assert np.allclose(ent, entropy(p, axis=1), rtol=0, atol=1e-13)
    assert np.array_equal(pred, margins.argmax(axis=1).astype(np.uint16))
    # the workload's softmax is neither flat nor saturated
    assert 0.2 < np.median(lc) < 0.8 and ent.max() <= math.log(cfg.n_classes) + 1e-12 and ent.min() >= 0
    # margins: a plain float64 sum of the same leaf values agrees to binary32 rounding
    n_int = (1 << model.depth) - 1
    for i in (0, 17, 1999):
        want = model.base.astype(np.float64).copy()
        for t in range(model.n_trees):
            k = 0
            for _ in range(model.depth):
                k = 2 * k + 1 + (0 if feat[i, model.node_feat[t, k]] <= model.node_thr[t, k] else 1)
            want[t % model.n_classes] += float(model.leaf_value[t, k - n_int])
        assert np.allclose(margins[i], want, rtol=0, atol=2e-5)


def test_degenerate_distributions():
    """one class far ahead: LC and entropy go to 0 without NaN; C = 1: both exactly 0"""
    m = _model(1, 3, 1, [[0]] * 3, [[0.0]] * 3, [[1000.0, 0], [0, 0], [0, 0]], None)
    _, pred, lc, ent = oracle.gbdt_infer(np.array([[-1.0], [1.0]], np.float32), m)
    assert pred.tolist() == [0, 0] and lc[0] == 0.0 and ent[0] == 0.0
    assert abs(lc[1] - 2 / 3) < 1e-15 and abs(ent[1] - math.log(3)) < 1e-15
    m1 = _model(2, 1, 1, [[0, 0, 0]], [[0.0, 0.0, 0.0]], [[1, 2, 3, 4]], [0.5])
    _, pred, lc, ent = oracle.gbdt_infer(np.array([[5.0]], np.float32), m1)
    assert pred.tolist() == [0] and lc[0] == 0.0 and ent[0] == 0.0


def _floor_f32(t64):
    t = np.float32(t64)
    return np.nextafter(t, np.float32(-np.inf)) if float(t) > t64 else t


def _perfect_regression_tree(sk, depth, scale):
    n_int, n_leaf = (1 << depth) - 1, 1 << depth
    feat, thr = np.zeros(n_int, np.uint16), np.full(n_int, np.inf, np.float32)
    val = np.zeros(n_leaf, np.float32)

    def place(node, k, level):
        if level == depth:
            val[k - n_int] = np.float32(scale * sk.value[node, 0, 0])
            return
        if sk.children_left[node] == -1:
            place(node, 2 * k + 1, level + 1)
            place(node, 2 * k + 2, level + 1)
            return
        feat[k], thr[k] = sk.feature[node], _floor_f32(sk.threshold[node])
        place(sk.children_left[node], 2 * k + 1, level + 1)
        place(sk.children_right[node], 2 * k + 2, level + 1)

    place(0, 0, 0)
    return feat, thr, val


def test_matches_scikit_learn_gradient_boosting():
    """A multiclass gradient-boosting classifier fitted by scikit-learn (one regression tree per class and
    round, margins = initial log-odds + learning rate * sum of leaf values, softmax on top).  Re-expressed
    as perfect trees it must give the same margins (to binary32 rounding), labels and probabilities."""
    from sklearn.ensemble import GradientBoostingClassifier
    rng = np.random.default_rng(3)
    C, depth, rounds = 4, 3, 12
    X = rng.normal(size=(1500, 6)).astype(np.float32)
    y = ((X[:, 0] > 0).astype(int) + 2 * (X[:, 2] * X[:, 4] > 0.1).astype(int))
    flip = rng.random(1500) < 0.15
    y[flip] = rng.integers(0, C, size=int(flip.sum()))
    clf = GradientBoostingClassifier(n_estimators=rounds, max_depth=depth, learning_rate=0.3, random_state=0).fit(X, y)
    feats, thrs, vals = [], [], []
    for r in range(rounds):
        for c in range(C):
            f, t, v = _perfect_regression_tree(clf.estimators_[r, c].tree_, depth, clf.learning_rate)
            feats.append(f), thrs.append(t), vals.append(v)
    Xt = rng.normal(size=(800, 6)).astype(np.float32)
    base = clf._raw_predict_init(Xt[:1])[0]
    model = _model(depth, C, 6, feats, thrs, vals, base)
    margins, pred, lc, ent = oracle.gbdt_infer(Xt, model)
    want = clf.decision_function(Xt)
    assert np.allclose(margins, want, rtol=0, atol=5e-5)
    proba = clf.predict_proba(Xt)
    assert np.allclose(lc, 1.0 - proba.max(axis=1), rtol=0, atol=5e-5)
    clear = np.sort(want, axis=1)[:, -1] - np.sort(want, axis=1)[:, -2] > 1e-3
    assert clear.mean() > 0.9 and np.array_equal(pred[clear], clf.predict(Xt)[clear].astype(np.uint16))
    assert np.allclose(ent, -(proba * np.log(proba)).sum(axis=1), rtol=0, atol=2e-4)


def test_score_gate_is_strictly_above():
    s = np.array([0.1, 0.5, 0.5000001, 0.9, 0.0, 0.5], np.float32)
    assert oracle.route_score(s, 0.5).tolist() == [2, 3]
    assert oracle.route_score(s, -1.0).tolist() == [0, 1, 2, 3, 4, 5]
    assert oracle.route_score(s, 0.9).tolist() == []
    rng = np.random.default_rng(1)
    s = rng.random(5000).astype(np.float32)
    for thr in (0.25, 0.75, float(s[77])):
        assert np.array_equal(oracle.route_score(s, thr), np.flatnonzero(s > np.float32(thr)).astype(np.uint32))


def test_quantile_threshold_reaches_the_target_portion():
    """Algorithm 1 on a real-valued score: the threshold at quantile 1 - p sends at most a share p on"""
    cfg = synth.get_config(7).scaled(20000)
    pk = synth.make_packets(cfg)
    feat, _ = oracle.featurize(pk.flow_off, pk.pkt_size, pk.pkt_iat, pk.pkt_dir, cfg.depths, n_threads=8)
    _, _, lc, ent = oracle.gbdt_infer(feat, synth.make_gbdt(cfg, feat[:4096]), want_margins=False, n_threads=8)
    for score in (lc.astype(np.float32), ent.astype(np.float32)):
        thr = oracle.universal_thresholds(score.astype(np.float64), [0.75])[0]
        frac = oracle.route_score(score, thr).size / score.size
        assert 0.249 <= frac <= 0.25
