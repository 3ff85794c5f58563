"""Seeded model parameters: a random-split forest and an Xavier-initialised MLP.

Trained models need the paper's datasets (Section 5.1); these random ones have
the same shapes and exercise the same code paths.  Both generators take a
feature sample as an argument and never compute features themselves.
"""
from dataclasses import dataclass
from typing import Optional

import numpy as np

from .configs import WorkloadConfig


@dataclass
class Forest:
    n_trees: int
    depth: int
    n_classes: int
    n_features: int
    node_feat: np.ndarray    # uint16 [T, 2^d - 1], heap order (children of k: 2k+1, 2k+2)
    node_thr: np.ndarray     # float32 [T, 2^d - 1]
    leaf_label: np.ndarray   # uint8 [T, 2^d]


@dataclass
class Tree:
    depth: int
    n_classes: int
    n_features: int
    node_feat: np.ndarray    # uint16 [2^d - 1], heap order
    node_thr: np.ndarray     # float32 [2^d - 1]
    leaf_count: np.ndarray   # uint16 [2^d, C]: training samples of each class at the leaf


@dataclass
class Gbdt:
    n_trees: int             # rounds * n_classes; tree t belongs to class t % n_classes
    depth: int
    n_classes: int
    n_features: int
    node_feat: np.ndarray    # uint16 [T, 2^d - 1], heap order
    node_thr: np.ndarray     # float32 [T, 2^d - 1]
    leaf_value: np.ndarray   # float32 [T, 2^d]: the margin a leaf adds to its tree's class
    base: np.ndarray         # float32 [C]: initial margins


@dataclass
class Mlp:
    dims: tuple              # (n_in, n_h1, n_h2, n_classes)
    dtype: str               # "f32" | "bf16" (weights are bf16-representable float32 when "bf16")
    w1: np.ndarray           # float32 [n_h1, n_in], row-major [out][in]
    b1: np.ndarray           # float32 [n_h1]
    w2: np.ndarray
    b2: np.ndarray
    w3: np.ndarray
    b3: np.ndarray
    mu: Optional[np.ndarray]         # float32 [n_in] or None (identity input map)
    inv_sigma: Optional[np.ndarray]  # float32 [n_in] or None
    clamp: float = 8.0


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """float32 -> nearest bfloat16 (ties to even), returned widened back to float32.
    bfloat16 is the upper 16 bits of an IEEE-754 binary32 value."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(np.shape(x))


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """The uint16 bit patterns of bf16-representable float32 values."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    assert not np.any(u & 0xFFFF), "values are not bf16-representable"
    return (u >> 16).astype(np.uint16).reshape(np.shape(x))


def make_forest(cfg: WorkloadConfig, feat_sample: np.ndarray, seed: Optional[int] = None) -> Forest:
    """Perfect binary trees of depth d.  Split feature uniform over the columns; split
    threshold = that feature's value in a uniformly drawn sample flow (a draw from
    the empirical quantiles); leaf labels uniform over the classes."""
    seed = cfg.model_seed if seed is None else seed
    rng = np.random.Generator(np.random.PCG64(seed * 1000 + 1))
    T, d, C = cfg.n_trees, cfg.tree_depth, cfg.n_classes
    F = feat_sample.shape[1]
    n_int = (1 << d) - 1
    F = cfg.tree0_features or F           # a cascade's forest splits on the same columns as its tree
    node_feat = rng.integers(0, F, size=(T, n_int), dtype=np.uint16)
    pick = rng.integers(0, feat_sample.shape[0], size=(T, n_int))
    node_thr = np.ascontiguousarray(feat_sample[pick, node_feat.astype(np.int64)], dtype=np.float32)
    leaf_label = rng.integers(0, C, size=(T, 1 << d), dtype=np.uint8)
    return Forest(T, d, C, F, node_feat, node_thr, leaf_label)


def make_tree(cfg: WorkloadConfig, feat_sample: np.ndarray, seed: Optional[int] = None) -> Tree:
    """The single decision tree of the first tier.  Splits as in make_forest, on the first
    cfg.tree0_features columns.  Leaf class counts: the leaf holds 15 + Poisson(45) samples
    (the paper keeps at least 15 per leaf), a uniformly drawn majority class with share
    p ~ U(0.15, 1) and the rest spread evenly, drawn as one multinomial."""
    seed = cfg.model_seed if seed is None else seed
    rng = np.random.Generator(np.random.PCG64(seed * 1000 + 3))
    d, C = cfg.tree0_depth, cfg.n_classes
    F = cfg.tree0_features or feat_sample.shape[1]
    n_int, n_leaf = (1 << d) - 1, 1 << d
    node_feat = rng.integers(0, F, size=n_int, dtype=np.uint16)
    pick = rng.integers(0, feat_sample.shape[0], size=n_int)
    node_thr = np.ascontiguousarray(feat_sample[pick, node_feat.astype(np.int64)], dtype=np.float32)
    total = 15 + rng.poisson(45.0, size=n_leaf)
    major = rng.integers(0, C, size=n_leaf)
    share = rng.uniform(0.15, 1.0, size=n_leaf)
    leaf_count = np.zeros((n_leaf, C), dtype=np.uint16)
    for l in range(n_leaf):
        p = np.full(C, (1.0 - share[l]) / max(C - 1, 1))
        p[major[l]] = share[l] if C > 1 else 1.0
        leaf_count[l] = rng.multinomial(int(total[l]), p / p.sum())
    return Tree(d, C, F, node_feat, node_thr, leaf_count)


def make_gbdt(cfg: WorkloadConfig, feat_sample: np.ndarray, seed: Optional[int] = None) -> Gbdt:
    """Boosted-tree fast model: splits as in make_forest; leaf margins N(0, 0.5^2) rounded to
    binary32 (ten rounds then give class margins of spread ~1.6, a softmax that is neither flat
    nor saturated); initial margins U(-0.5, 0.5)."""
    seed = cfg.model_seed if seed is None else seed
    rng = np.random.Generator(np.random.PCG64(seed * 1000 + 4))
    T, d, C = cfg.n_trees, cfg.tree_depth, cfg.n_classes
    F = feat_sample.shape[1]
    n_int = (1 << d) - 1
    node_feat = rng.integers(0, F, size=(T, n_int), dtype=np.uint16)
    pick = rng.integers(0, feat_sample.shape[0], size=(T, n_int))
    node_thr = np.ascontiguousarray(feat_sample[pick, node_feat.astype(np.int64)], dtype=np.float32)
    leaf_value = rng.normal(0.0, 0.5, size=(T, 1 << d)).astype(np.float32)
    base = rng.uniform(-0.5, 0.5, size=C).astype(np.float32)
    return Gbdt(T, d, C, F, node_feat, node_thr, leaf_value, base)


def make_truth(cfg: WorkloadConfig, pred: np.ndarray, top_votes: np.ndarray, seed: Optional[int] = None) -> np.ndarray:
    """Synthetic ground truth for a validation set (the paper's come with its datasets): the fast
    model's label is right with a probability that rises with its confidence, at a class-dependent
    rate, so that classes differ in how informative their uncertainty is (the situation per-class
    thresholds are made for).  p(correct) = clip(a_c + b_c * top_votes / n_trees, 0.02, 0.98) with
    a_c ~ U(-0.6, 0.1), b_c ~ U(3, 7); a wrong label is uniform over the other classes.
    pred and top_votes are inputs: whoever calls this has computed them."""
    seed = cfg.model_seed if seed is None else seed
    rng = np.random.Generator(np.random.PCG64(seed * 1000 + 5))
    C, T = cfg.n_classes, cfg.n_trees
    a, b = rng.uniform(-0.6, 0.1, size=C), rng.uniform(3.0, 7.0, size=C)
    pred = np.asarray(pred).astype(np.int64)
    p = np.clip(a[pred] + b[pred] * np.asarray(top_votes, np.float64) / T, 0.02, 0.98)
    right = rng.random(pred.shape[0]) < p
    other = (pred + 1 + rng.integers(0, max(C - 1, 1), size=pred.shape[0])) % C
    return np.where(right, pred, other).astype(np.uint16)


def _xavier(rng, fan_out, fan_in):
    a = np.sqrt(6.0 / (fan_in + fan_out))
    return rng.uniform(-a, a, size=(fan_out, fan_in)).astype(np.float32)


def make_mlp(cfg: WorkloadConfig, feat_sample: Optional[np.ndarray], seed: Optional[int] = None) -> Mlp:
    """Glorot-uniform weights, U(-0.1, 0.1) biases (non-zero so a dropped bias shows).
    For a bf16 model the weights are rounded to bf16 once, here, so every consumer
    sees identical values.  ``feat_sample`` (stat-feature input) yields the per-column
    standardisation constants; pass None for {0,1} raw-bit inputs (identity map)."""
    seed = cfg.model_seed if seed is None else seed
    rng = np.random.Generator(np.random.PCG64(seed * 1000 + 2))
    n_in, h1, h2, C = cfg.mlp_dims
    w1, w2, w3 = _xavier(rng, h1, n_in), _xavier(rng, h2, h1), _xavier(rng, C, h2)
    b1, b2, b3 = (rng.uniform(-0.1, 0.1, size=n).astype(np.float32) for n in (h1, h2, C))
    if cfg.mlp_dtype == "bf16":
        w1, w2, w3 = round_to_bf16(w1), round_to_bf16(w2), round_to_bf16(w3)
    mu = inv_sigma = None
    if feat_sample is not None:
        assert feat_sample.shape[1] == n_in
        s64 = feat_sample.astype(np.float64)
        mu = s64.mean(axis=0).astype(np.float32)
        sd = s64.std(axis=0)
        inv_sigma = np.where(sd > 0, 1.0 / np.where(sd > 0, sd, 1.0), 1.0).astype(np.float32)
    return Mlp((n_in, h1, h2, C), cfg.mlp_dtype, w1, b1, w2, b2, w3, b3, mu, inv_sigma, 8.0)
