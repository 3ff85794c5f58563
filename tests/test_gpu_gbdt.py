"""Parity of the boosted-tree fast model and the score gate against the CPU oracle, through the C ABI.
Bit-exact: leaf indices, binary32 margins (both sides add in tree order), pred, and the gate / the
quantile thresholds on given scores.  The score itself is a binary64 softmax rounded to binary32 on both
sides; the two exp/log implementations may differ in the last places of binary64 (1e-13 absolute is
allowed before the rounding), so in rare cases the binary32 results are neighbours instead of equal: the
routing of the whole path is compared on every flow on whose binary32 score both sides agree."""
from dataclasses import replace
from types import SimpleNamespace

import numpy as np
import pytest

import oracle
import synth

pytestmark = pytest.mark.gpu

KINDS = {"lc": 0, "entropy": 1}


def _u16(t):
    return t.cpu().numpy().view(np.uint16)


def _u32(t):
    return t.cpu().numpy().view(np.uint32)


def _ulp_close(got, want64):
    """got: binary32 from the GPU; want64: the oracle's binary64 score.  ok: got is a correct rounding of a
    binary64 value within 1e-13 of the oracle's (two exp/log routines, a sum of at most 64 terms);
    same: got equals the oracle's value rounded to binary32."""
    w = want64.astype(np.float32)
    half_ulp = 0.5 * np.spacing(np.abs(w)).astype(np.float64)
    ok = np.abs(got.astype(np.float64) - want64) <= half_ulp + 1e-13
    return ok, got == w


def _setup(n, **kw):
    cfg = synth.get_config(7)
    if kw:
        cfg = replace(cfg, **kw)
    pk = synth.make_packets(cfg, n_flows=n)
    feat, _ = oracle.featurize(pk.flow_off, pk.pkt_size, pk.pkt_iat, pk.pkt_dir, cfg.depths, n_threads=8)
    return cfg, pk, feat, synth.make_gbdt(cfg, feat[:4096]), synth.make_mlp(cfg, feat[:4096])


def _gpu_gbdt(feat, model, kind, want_leaf=True):
    import torch
    import paper_2402_03694_amd as sf
    n, C, T = feat.shape[0], model.n_classes, model.n_trees
    ctx = sf.ServeFlow(sf.sf_workspace_bytes(max(n, 1), T, model.depth))
    dev = "cuda:0"
    margins = torch.full((n, C), float("nan"), dtype=torch.float32, device=dev)
    pred = torch.full((n,), -1, dtype=torch.int16, device=dev)
    score = torch.full((n,), float("nan"), dtype=torch.float32, device=dev)
    leaf = torch.full((n, T), -1, dtype=torch.int16, device=dev) if want_leaf else None
    ctx.sf_gbdt_infer(torch.from_numpy(np.ascontiguousarray(feat)).to(dev), sf.gbdt_to_device(model, dev), KINDS[kind],
                      pred, score, margins=margins, leaf_idx=leaf)
    torch.cuda.synchronize()
    return margins.cpu().numpy(), _u16(pred), score.cpu().numpy(), (_u16(leaf) if want_leaf else None)


@pytest.mark.parametrize("kind", ["lc", "entropy"])
@pytest.mark.parametrize("n,kw", [(5000 + 17, {}), (700, dict(tree_depth=7, n_trees=33, n_classes=3)),
                                  (300, dict(tree_depth=1, n_trees=5, n_classes=5)),
                                  (1000, dict(tree_depth=12, n_trees=24, n_classes=4))])
def test_margins_pred_and_scores(kind, n, kw):
    cfg, pk, feat, model, _ = _setup(n, **kw)
    o_m, o_pred, o_lc, o_ent = oracle.gbdt_infer(feat, model, n_threads=8)
    g_m, g_pred, g_score, g_leaf = _gpu_gbdt(feat, model, kind)
    assert np.array_equal(g_m.view(np.uint32), o_m.view(np.uint32))
    assert np.array_equal(g_pred, o_pred)
    ok, same = _ulp_close(g_score, o_lc if kind == "lc" else o_ent)
    assert ok.all(), int((~ok).sum())
    assert same.mean() > 0.9999
    # leaves against a walk of the same trees by the forest oracle (labels are irrelevant here)
    as_forest = SimpleNamespace(n_trees=model.n_trees, depth=model.depth, n_classes=1, n_features=model.n_features,
                                node_feat=model.node_feat, node_thr=model.node_thr,
                                leaf_label=np.zeros((model.n_trees, 1 << model.depth), np.uint8))
    assert np.array_equal(g_leaf, oracle.fast_infer(feat, as_forest, want_votes=False, want_leaves=True, n_threads=8)[3])


def test_sum_order_and_missing_base():
    """1e8 + 1 - 1e8 = 0 left to right in binary32 (1 in any other order); base = NULL means zeros"""
    vals0, vals1 = [1e8, 1.0, -1e8], [1e8, -1e8, 1.0]
    leaf = np.zeros((6, 2), np.float32)
    for r in range(3):
        leaf[2 * r], leaf[2 * r + 1] = vals0[r], vals1[r]
    model = SimpleNamespace(n_trees=6, depth=1, n_classes=2, n_features=4, node_feat=np.zeros((6, 1), np.uint16),
                            node_thr=np.zeros((6, 1), np.float32), leaf_value=leaf, base=None)
    feat = np.zeros((130, 4), np.float32)
    g_m, g_pred, g_score, _ = _gpu_gbdt(feat, model, "lc")
    assert np.all(g_m == np.array([0.0, 1.0], np.float32)) and np.all(g_pred == 1)
    o_m, o_pred, o_lc, _ = oracle.gbdt_infer(feat, model)
    assert np.array_equal(g_m, o_m) and _ulp_close(g_score, o_lc)[0].all()


def test_gate_and_quantiles_on_given_scores():
    """scores from the oracle go in; the gate and Algorithm 1's thresholds must be exact"""
    import torch
    import paper_2402_03694_amd as sf
    cfg, pk, feat, model, _ = _setup(30000 + 5)
    _, _, lc, ent = oracle.gbdt_infer(feat, model, want_margins=False, n_threads=8)
    n = lc.size
    ctx = sf.ServeFlow(sf.sf_workspace_bytes(n))
    esc = torch.full((n,), -1, dtype=torch.int32, device="cuda:0")
    cnt = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    rng = np.random.default_rng(2)
    special = np.array([0.0, -0.0, 1e-45, -1e-45, -3.5, np.inf, -np.inf, 2.5, 2.5, 2.5], np.float32)
    for s64 in (lc, ent):
        s = s64.astype(np.float32)
        s[rng.integers(0, n, size=special.size)] = special      # signs, zeros, denormals, infinities, ties
        d_s = torch.from_numpy(s).to("cuda:0")
        qs = [0.0, 1e-9, 0.01, 0.25, 0.5, 0.75, 0.99, 1.0, 0.3333333]
        got = ctx.sf_score_quantiles(d_s, qs)
        want = oracle.universal_thresholds(s.astype(np.float64), qs)
        assert [np.float32(g) for g in got] == [np.float32(w) for w in want]
        for thr in [float(want[3]), float(want[5]), 0.0, -1.0, 2.5, float(s[17]), float(np.nextafter(s[17], np.float32(9)))]:
            ctx.sf_route_score(d_s, thr, esc, cnt)
            torch.cuda.synchronize()
            w = oracle.route_score(s, thr)
            assert int(_u32(cnt)[0]) == w.size and np.array_equal(_u32(esc)[:w.size], w), thr
    thr75 = oracle.universal_thresholds(lc.astype(np.float32).astype(np.float64), [0.75])[0]
    assert 0.24 < oracle.route_score(lc.astype(np.float32), thr75).size / n <= 0.25


def _whole_path(cfg, n, feat_np, model, mlp, kind, thr):
    import torch
    import paper_2402_03694_amd as sf
    dev = "cuda:0"
    ctx = sf.ServeFlow(sf.sf_workspace_bytes(n, model.n_trees, model.depth, *mlp.dims[:3]))
    feat = torch.from_numpy(np.ascontiguousarray(feat_np)).to(dev)
    d_model, d_mlp = sf.gbdt_to_device(model, dev), sf.mlp_to_device(mlp, dev)
    pred = torch.full((n,), -1, dtype=torch.int16, device=dev)
    score = torch.zeros(n, dtype=torch.float32, device=dev)
    esc = torch.full((n,), -1, dtype=torch.int32, device=dev)
    cnt = torch.zeros(1, dtype=torch.int32, device=dev)
    labels = torch.full((n,), -1, dtype=torch.int16, device=dev)
    logits = torch.full((n, mlp.dims[3]), float("nan"), dtype=torch.float32, device=dev)
    for _ in range(2):
        ctx.sf_gbdt_infer(feat, d_model, KINDS[kind], pred, score)
        ctx.sf_route_score(score, thr, esc, cnt)
        ctx.sf_slow_infer(d_mlp, esc, cnt, labels, feat=feat, logits=logits, pred=pred)
    torch.cuda.synchronize()
    k = int(_u32(cnt)[0])
    return _u16(pred), score.cpu().numpy(), _u32(esc)[:k].copy(), _u16(labels), logits.cpu().numpy()[:k]


def _check_whole_path(n, kind):
    cfg, pk, feat, model, mlp = _setup(n)
    thr_n = oracle.default_threads()
    _, o_pred, o_lc, o_ent = oracle.gbdt_infer(feat, model, want_margins=False, n_threads=thr_n)
    o64 = o_lc if kind == "lc" else o_ent
    o_score = o64.astype(np.float32)
    thr = float(np.float32(oracle.universal_thresholds(o_score.astype(np.float64), [0.75])[0]))
    o_esc = oracle.route_score(o_score, thr)
    g_pred, g_score, g_esc, g_lab, g_logits = _whole_path(cfg, n, feat, model, mlp, kind, thr)
    assert np.array_equal(g_pred, o_pred)
    ok, same = _ulp_close(g_score, o64)
    assert ok.all()
    # routing: identical on every flow whose score both sides agree on (all but a handful, if any)
    firm = np.flatnonzero(same)
    # how many flows sat on a binary32 rounding boundary (the two binary64 scores differ in their last
    # places and round to neighbouring binary32 values): reported, and bounded
    import sys
    print("[gbdt] %d flows, %s score: %d with neighbouring binary32 scores on the two sides"
          % (n, kind, n - firm.size), file=sys.__stderr__, flush=True)
    assert firm.size >= n - 8
    g_in, o_in = np.zeros(n, bool), np.zeros(n, bool)
    g_in[g_esc], o_in[o_esc] = True, True
    assert np.array_equal(g_in[firm], o_in[firm])
    assert np.all(np.diff(g_esc.astype(np.int64)) > 0)
    assert 0.2 < g_esc.size / n <= 0.2501
    # labels: the boosted model's where the flow stayed, the MLP's where it went on
    both = np.flatnonzero(g_in & o_in)
    rows = both[:: max(1, both.size // 16384)]
    o_logits, o_lab = oracle.slow_infer(rows.astype(np.uint32), mlp, n, feat=feat, n_threads=thr_n)
    pos = np.searchsorted(g_esc, rows)
    err = np.abs(g_logits[pos] - o_logits)
    assert err.max() <= 2e-2, err.max()
    srt = np.sort(o_logits, axis=1)
    clear = (srt[:, -1] - srt[:, -2]) > 5e-2
    assert np.array_equal(g_lab[rows][clear], o_lab[rows][clear])
    assert np.array_equal(g_lab[~g_in], o_pred[~g_in])


@pytest.mark.parametrize("kind", ["lc", "entropy"])
def test_whole_path_small(kind):
    _check_whole_path(20000 + 3, kind)


def test_whole_path_full_size():
    """1,048,576 flows, the launch configuration bench.py times for the boosted workload"""
    _check_whole_path(1 << 20, "entropy")


def test_gbdt_error_paths():
    import torch
    import paper_2402_03694_amd as sf
    cfg, pk, feat, model, _ = _setup(64)
    ctx = sf.ServeFlow(sf.sf_workspace_bytes(64, model.n_trees, model.depth))
    d_feat = torch.from_numpy(feat).to("cuda:0")
    pred = torch.zeros(64, dtype=torch.int16, device="cuda:0")
    score = torch.zeros(64, dtype=torch.float32, device="cuda:0")
    esc = torch.zeros(64, dtype=torch.int32, device="cuda:0")
    cnt = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    d_model = sf.gbdt_to_device(model)
    with pytest.raises(sf.ServeFlowError) as e:
        ctx.sf_gbdt_infer(d_feat, d_model, 7, pred, score)
    assert e.value.code == -1 and "score_kind" in str(e.value)
    d_model.depth = 15
    with pytest.raises(sf.ServeFlowError) as e:
        ctx.sf_gbdt_infer(d_feat, d_model, 0, pred, score)
    assert e.value.code == -1 and "depth" in str(e.value)
    with pytest.raises(sf.ServeFlowError) as e:
        ctx.sf_route_score(score, float("nan"), esc, cnt)
    assert e.value.code == -1
    ctx.sf_route_score(score, 0.5, esc, cnt, n_flows=0)
    torch.cuda.synchronize()
    assert int(_u32(cnt)[0]) == 0
    small = sf.ServeFlow(4096)
    with pytest.raises(sf.ServeFlowError) as e:
        small.sf_score_quantiles(score, [0.5])
    assert e.value.code == -2
