"""Python face of the CPU oracle (oracle/serveflow_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  The product package never imports this module and
this module never imports the product package.

Every function takes and returns numpy arrays; see the C file for what each step
computes and which passage of the paper it follows.
"""
import ctypes
import os
import subprocess
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "serveflow_oracle.c")
# SF_ORACLE_SANITIZE=1: a second build with AddressSanitizer and UndefinedBehaviorSanitizer (the process must
# have gcc's libasan preloaded); the arithmetic flags stay the same, so every pin must still hold
_SANITIZE = os.environ.get("SF_ORACLE_SANITIZE") == "1"
_LIB = os.path.join(_HERE, "libsf_oracle_san.so" if _SANITIZE else "libsf_oracle.so")

CFLAGS = ["-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
          "-fno-unsafe-math-optimizations", "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (one second); returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        extra = ["-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all"] if _SANITIZE else []
        subprocess.check_call(["gcc", *CFLAGS, *extra, _SRC, "-o", tmp, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_vmin_from_theta.restype = ctypes.c_uint32
        _lib.oracle_vmin_from_theta.argtypes = [ctypes.c_float, ctypes.c_uint32]
        _lib.oracle_route.restype = ctypes.c_uint32
        _lib.oracle_route_ratio.restype = ctypes.c_uint32
        _lib.oracle_tree_infer.restype = ctypes.c_int
        _lib.oracle_gbdt_infer.restype = ctypes.c_int
        _lib.oracle_route_score.restype = ctypes.c_uint32
        for name in ("oracle_featurize", "oracle_fast_infer", "oracle_slow_infer",
                     "oracle_universal_thresholds", "oracle_max_window"):
            getattr(_lib, name).restype = ctypes.c_int
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


def default_threads() -> int:
    return max(1, min(16, os.cpu_count() or 1))


def featurize(flow_off, pkt_size, pkt_iat, pkt_dir, depths: Sequence[int], pkt_hdr=None,
              raw_pkts: int = 0, raw_bits: int = 0, feat_ld: Optional[int] = None,
              want_raw: bool = False, n_threads: int = 1) -> Tuple[np.ndarray, Optional[np.ndarray]]:
    lib = _load()
    flow_off = _c(flow_off, np.uint32)
    pkt_size, pkt_iat, pkt_dir = _c(pkt_size, np.uint16), _c(pkt_iat, np.float32), _c(pkt_dir, np.uint8)
    n = flow_off.shape[0] - 1
    W = len(depths)
    ld = 32 * W if feat_ld is None else feat_ld
    feat = np.zeros((n, ld), dtype=np.float32)
    dep = np.asarray(list(depths), dtype=np.uint32)
    hdr_words = 0
    raw = None
    if pkt_hdr is not None:
        pkt_hdr = _c(pkt_hdr, np.uint32)
        hdr_words = pkt_hdr.shape[1]
    if want_raw:
        raw = np.zeros((n, raw_pkts * raw_bits), dtype=np.uint8)
    rc = lib.oracle_featurize(ctypes.c_uint32(n), _p(flow_off), _p(pkt_size), _p(pkt_iat), _p(pkt_dir),
                              _p(pkt_hdr), ctypes.c_uint32(hdr_words), ctypes.c_uint32(W), _p(dep),
                              ctypes.c_uint32(raw_pkts), ctypes.c_uint32(raw_bits), _p(feat),
                              ctypes.c_uint32(ld), _p(raw), ctypes.c_int(n_threads))
    if rc != 0:
        raise ValueError("oracle_featurize: invalid arguments")
    return feat, raw


def fast_infer(feat, forest, want_votes: bool = True, want_leaves: bool = False, n_threads: int = 1):
    """forest: any object with n_trees, depth, n_classes, n_features, node_feat, node_thr, leaf_label."""
    lib = _load()
    feat = _c(feat, np.float32)
    n, ld = feat.shape
    T, C = forest.n_trees, forest.n_classes
    nf, nt, ll = _c(forest.node_feat, np.uint16), _c(forest.node_thr, np.float32), _c(forest.leaf_label, np.uint8)
    votes = np.zeros((n, C), np.uint16) if want_votes else None
    leaves = np.zeros((n, T), np.uint16) if want_leaves else None
    pred = np.zeros(n, np.uint16)
    top = np.zeros(n, np.uint16)
    rc = lib.oracle_fast_infer(ctypes.c_uint32(n), _p(feat), ctypes.c_uint32(ld), ctypes.c_uint32(T),
                               ctypes.c_uint32(forest.depth), ctypes.c_uint32(C),
                               ctypes.c_uint32(forest.n_features), _p(nf), _p(nt), _p(ll),
                               _p(votes), _p(pred), _p(top), _p(leaves), ctypes.c_int(n_threads))
    if rc != 0:
        raise ValueError("oracle_fast_infer: invalid arguments")
    return votes, pred, top, leaves


def vmin_from_theta(theta: float, n_trees: int) -> int:
    return int(_load().oracle_vmin_from_theta(ctypes.c_float(np.float32(theta)), ctypes.c_uint32(n_trees)))


def route(top_votes, pred, vmin) -> np.ndarray:
    lib = _load()
    top_votes, pred = _c(top_votes, np.uint16), _c(pred, np.uint16)
    vm = _c(np.atleast_1d(vmin), np.uint16)
    n = top_votes.shape[0]
    esc = np.zeros(max(n, 1), np.uint32)
    cnt = lib.oracle_route(ctypes.c_uint32(n), _p(top_votes), _p(pred), _p(vm),
                           ctypes.c_uint32(vm.shape[0]), _p(esc))
    return esc[:cnt].copy()


def tree_infer(feat, tree, want_leaves: bool = False, n_threads: int = 1):
    """tree: any object with depth, n_classes, n_features, node_feat, node_thr, leaf_count.
    Returns (pred, top_count, leaf_total, leaf_idx or None)."""
    lib = _load()
    feat = _c(feat, np.float32)
    n, ld = feat.shape
    nf, nt, lc = _c(tree.node_feat, np.uint16), _c(tree.node_thr, np.float32), _c(tree.leaf_count, np.uint16)
    assert nf.shape == ((1 << tree.depth) - 1,) and lc.shape == (1 << tree.depth, tree.n_classes)
    pred, top, tot = (np.zeros(n, np.uint16) for _ in range(3))
    leaves = np.zeros(n, np.uint16) if want_leaves else None
    rc = lib.oracle_tree_infer(ctypes.c_uint32(n), _p(feat), ctypes.c_uint32(ld), ctypes.c_uint32(tree.depth),
                               ctypes.c_uint32(tree.n_classes), ctypes.c_uint32(tree.n_features), _p(nf),
                               _p(nt), _p(lc), _p(pred), _p(top), _p(tot), _p(leaves), ctypes.c_int(n_threads))
    if rc != 0:
        raise ValueError("oracle_tree_infer: invalid arguments")
    return pred, top, tot, leaves


def route_ratio(top_count, leaf_total, theta) -> np.ndarray:
    lib = _load()
    top_count, leaf_total = _c(top_count, np.uint16), _c(leaf_total, np.uint16)
    n = top_count.shape[0]
    esc = np.zeros(max(n, 1), np.uint32)
    cnt = lib.oracle_route_ratio(ctypes.c_uint32(n), _p(top_count), _p(leaf_total),
                                 ctypes.c_float(np.float32(theta)), _p(esc))
    return esc[:cnt].copy()


def gbdt_infer(feat, model, want_margins: bool = True, n_threads: int = 1):
    """model: any object with n_trees, depth, n_classes, n_features, node_feat, node_thr, leaf_value, base.
    Returns (margins float32 [n, C] or None, pred, lc float64, entropy float64)."""
    lib = _load()
    feat = _c(feat, np.float32)
    n, ld = feat.shape
    T, C = model.n_trees, model.n_classes
    nf, nt, lv = _c(model.node_feat, np.uint16), _c(model.node_thr, np.float32), _c(model.leaf_value, np.float32)
    assert nf.shape == (T, (1 << model.depth) - 1) and lv.shape == (T, 1 << model.depth)
    base = None if model.base is None else _c(model.base, np.float32)
    margins = np.zeros((n, C), np.float32) if want_margins else None
    pred = np.zeros(n, np.uint16)
    lc, ent = np.zeros(n, np.float64), np.zeros(n, np.float64)
    rc = lib.oracle_gbdt_infer(ctypes.c_uint32(n), _p(feat), ctypes.c_uint32(ld), ctypes.c_uint32(T),
                               ctypes.c_uint32(model.depth), ctypes.c_uint32(C), ctypes.c_uint32(model.n_features),
                               _p(nf), _p(nt), _p(lv), _p(base), _p(margins), _p(pred), _p(lc), _p(ent),
                               ctypes.c_int(n_threads))
    if rc != 0:
        raise ValueError("oracle_gbdt_infer: invalid arguments")
    return margins, pred, lc, ent


def route_score(score, threshold) -> np.ndarray:
    lib = _load()
    score = _c(score, np.float32)
    n = score.shape[0]
    esc = np.zeros(max(n, 1), np.uint32)
    cnt = lib.oracle_route_score(ctypes.c_uint32(n), _p(score), ctypes.c_float(np.float32(threshold)), _p(esc))
    return esc[:cnt].copy()


def universal_thresholds(scores, quantiles) -> np.ndarray:
    lib = _load()
    s, q = _c(scores, np.float64), _c(quantiles, np.float64)
    out = np.zeros(q.shape[0], np.float64)
    rc = lib.oracle_universal_thresholds(_p(s), ctypes.c_uint32(s.shape[0]), _p(q),
                                         ctypes.c_uint32(q.shape[0]), _p(out))
    if rc != 0:
        raise ValueError("oracle_universal_thresholds: empty score list")
    return out


def per_class_thresholds(pred, top_votes, correct, n_trees: int, n_classes: int, target_fraction: float):
    """Slope-based per-class uncertainty thresholds (Algorithm 2) on the integer score.

    Uncertainty is LC = 1 - top_votes / n_trees, so "most uncertain first" is "fewest votes first".
    Reading of the algorithm's steps:
      * per predicted class L the flows are split into correct and incorrect ones;
      * the class's candidate thresholds are the distinct score values it contains (the finest quantile
        grid); lowering the class's threshold by one candidate assigns the flows of the next vote count v:
        dC correct and dI incorrect ones, slope = dI / (dC + dI);
      * every class starts at its highest uncertainty (nothing assigned); each increment takes, among the
        classes' next candidates, the one with the largest slope (exact comparison of the fractions; the
        lowest class on ties), moves that class's threshold and adds dC + dI to the assigned total;
      * increments stop as soon as the assigned total reaches target_fraction * N (or nothing is left).
    Returns (vmin[C], assigned fraction, the list of (class, v, dC, dI) taken): class c escalates a flow
    iff top_votes < vmin[c]."""
    from fractions import Fraction
    pred, top, correct = np.asarray(pred), np.asarray(top_votes), np.asarray(correct).astype(bool)
    n = pred.shape[0]
    steps = []                       # per class: list of (v, dC, dI) in order of decreasing uncertainty
    for L in range(n_classes):
        mine = pred == L
        cand = []
        for v in sorted(set(top[mine].tolist())):
            sel = mine & (top == v)
            cand.append((int(v), int((sel & correct).sum()), int((sel & ~correct).sum())))
        steps.append(cand)
    nxt = [0] * n_classes
    vmin = [0] * n_classes
    assigned, taken = 0, []
    want = Fraction(float(target_fraction)) * n
    while assigned < want:
        best, best_slope = None, None
        for L in range(n_classes):
            if nxt[L] < len(steps[L]):
                v, dc, di = steps[L][nxt[L]]
                slope = Fraction(di, dc + di)
                if best is None or slope > best_slope:
                    best, best_slope = L, slope
        if best is None:
            break
        v, dc, di = steps[best][nxt[best]]
        nxt[best] += 1
        vmin[best] = v + 1
        assigned += dc + di
        taken.append((best, v, dc, di))
    return np.asarray(vmin, np.uint16), (assigned / n if n else 0.0), taken


class FlowJoin:
    """The two queues in front of the slow model (Section 3.1): queue 3 carries the flows the fast model
    hands on, queue 2 the features of their later packets, both keyed by flow ID; the slow model takes a
    flow when both are there; what finds no partner in the other queue is discarded after a timeout.

    Batched reading: one step = (1) discard every waiting record older than ``timeout`` ticks
    (``now - stamp > timeout``, 32-bit wrap-around arithmetic), (2) take the step's arrivals of both
    queues, stamped ``now``; a flow ID present on both sides (waiting or just arrived) is a match: it
    yields the pair (queue-3 value, queue-2 value) once and leaves both sides; the rest waits.  Within
    one side a flow ID may be waiting or arriving only once (a second record is invalid input).
    The result does not depend on the order in which records are looked at; pairs are returned sorted by
    flow ID here (the library returns them in no particular order)."""

    def __init__(self):
        self.wait3, self.wait2 = {}, {}          # flow id -> (value, stamp)

    def step(self, now, timeout, q3_id, q3_val, q2_id, q2_val):
        now, timeout = int(now) & 0xFFFFFFFF, int(timeout)
        expired = 0
        for side in (self.wait3, self.wait2):
            old = [k for k, (_, st) in side.items() if ((now - st) & 0xFFFFFFFF) > timeout]
            for k in old:
                del side[k]
            expired += len(old)
        for k, v in zip(np.asarray(q3_id, np.uint64).tolist(), np.asarray(q3_val, np.uint32).tolist()):
            if k in self.wait3:
                raise ValueError("flow %d twice in queue 3" % k)
            self.wait3[k] = (v, now)
        for k, v in zip(np.asarray(q2_id, np.uint64).tolist(), np.asarray(q2_val, np.uint32).tolist()):
            if k in self.wait2:
                raise ValueError("flow %d twice in queue 2" % k)
            self.wait2[k] = (v, now)
        both = sorted(set(self.wait3) & set(self.wait2))
        pairs = [(k, self.wait3.pop(k)[0], self.wait2.pop(k)[0]) for k in both]
        return pairs, expired

    def pending(self, side):
        """sorted (flow id, value, stamp) of one side (3 or 2)"""
        d = self.wait3 if side == 3 else self.wait2
        return sorted((k, v, st) for k, (v, st) in d.items())


def slow_infer(esc_idx, mlp, n_flows: int, feat=None, flow_off=None, pkt_hdr=None, raw_pkts: int = 0,
               raw_bits: int = 0, labels: Optional[np.ndarray] = None, n_threads: int = 1):
    """mlp: any object with dims, dtype, w1..b3, mu, inv_sigma, clamp.  Returns (logits, labels);
    ``labels`` (length n_flows) is updated at escalated positions only."""
    lib = _load()
    esc_idx = _c(esc_idx, np.uint32)
    E = esc_idx.shape[0]
    n_in, h1, h2, C = mlp.dims
    logits = np.zeros((E, C), np.float32)
    if labels is None:
        labels = np.zeros(n_flows, np.uint16)
    assert labels.dtype == np.uint16 and labels.flags.c_contiguous and labels.shape[0] == n_flows
    ld = hdr_words = 0
    if feat is not None:
        feat = _c(feat, np.float32)
        ld = feat.shape[1]
    else:
        flow_off, pkt_hdr = _c(flow_off, np.uint32), _c(pkt_hdr, np.uint32)
        hdr_words = pkt_hdr.shape[1]
    w = [_c(getattr(mlp, k), np.float32) for k in ("w1", "b1", "w2", "b2", "w3", "b3")]
    mu = None if mlp.mu is None else _c(mlp.mu, np.float32)
    isg = None if mlp.inv_sigma is None else _c(mlp.inv_sigma, np.float32)
    rc = lib.oracle_slow_infer(ctypes.c_uint32(E), _p(esc_idx), _p(feat), ctypes.c_uint32(ld),
                               _p(flow_off), _p(pkt_hdr), ctypes.c_uint32(hdr_words),
                               ctypes.c_uint32(raw_pkts), ctypes.c_uint32(raw_bits),
                               ctypes.c_uint32(n_in), ctypes.c_uint32(h1), ctypes.c_uint32(h2),
                               ctypes.c_uint32(C), ctypes.c_int(1 if mlp.dtype == "bf16" else 0),
                               _p(mu), _p(isg), ctypes.c_float(mlp.clamp),
                               *[_p(a) for a in w], _p(logits), _p(labels), ctypes.c_int(n_threads))
    if rc != 0:
        raise ValueError("oracle_slow_infer: invalid arguments")
    return logits, labels


def classify3(pk, depths, tree, theta0, forest, vmin, mlp, n_threads: int = 1):
    """The three-tier cascade of Section 3.1: the tree on every flow, the forest on the flows
    the tree is unsure of, the MLP on the flows the forest is unsure of; a later tier's label
    replaces the earlier one (Section 4.4).  Lists are in flow numbering, ascending."""
    feat, _ = featurize(pk.flow_off, pk.pkt_size, pk.pkt_iat, pk.pkt_dir, depths, n_threads=n_threads)
    pred0, top0, tot0, leaf0 = tree_infer(feat, tree, want_leaves=True, n_threads=n_threads)
    esc1 = route_ratio(top0, tot0, theta0)
    votes, pred1, top1, _ = fast_infer(feat[esc1], forest, n_threads=n_threads)   # rows follow esc1
    esc2 = esc1[route(top1, pred1, vmin)]
    labels = pred0.copy()
    labels[esc1] = pred1
    logits, labels = slow_infer(esc2, mlp, feat.shape[0], feat=feat, labels=labels, n_threads=n_threads)
    return dict(feat=feat, pred0=pred0, top0=top0, total0=tot0, leaf0=leaf0, esc1=esc1, votes1=votes,
                pred1=pred1, top1=top1, esc2=esc2, logits=logits, labels=labels)


def classify(pk, depths, forest, vmin, mlp, raw_pkts=0, raw_bits=0, n_threads: int = 1):
    """All five steps in order; returns a dict of every intermediate result."""
    feat, _ = featurize(pk.flow_off, pk.pkt_size, pk.pkt_iat, pk.pkt_dir, depths, n_threads=n_threads)
    votes, pred, top, leaves = fast_infer(feat, forest, want_leaves=True, n_threads=n_threads)
    esc = route(top, pred, vmin)
    labels = pred.copy()
    if raw_pkts:
        logits, labels = slow_infer(esc, mlp, feat.shape[0], flow_off=pk.flow_off, pkt_hdr=pk.pkt_hdr,
                                    raw_pkts=raw_pkts, raw_bits=raw_bits, labels=labels,
                                    n_threads=n_threads)
    else:
        logits, labels = slow_infer(esc, mlp, feat.shape[0], feat=feat, labels=labels,
                                    n_threads=n_threads)
    return dict(feat=feat, votes=votes, pred=pred, top_votes=top, leaf_idx=leaves, esc_idx=esc,
                logits=logits, labels=labels)
