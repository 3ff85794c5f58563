"""Parity at the full size of the benchmark workload, in the launch configuration bench.py times:
1,048,576 flows x 16 packets, 64 features, 100 trees of depth 12, 10 classes, bf16 MLP 64-512-512-10.
Features, pred, top_votes and the escalation list are compared with the oracle on EVERY flow
(the oracle runs its outer parallel-for on the host cores); slow-model logits on a fixed-stride
sample of the escalated flows.  A second case runs one full streaming batch of ragged flows."""
import numpy as np
import pytest

import oracle
import synth

pytestmark = pytest.mark.gpu


def _full(cfg_id, n, vmin, logit_sample):
    import torch
    import paper_2402_03694_amd as sf
    cfg = synth.get_config(cfg_id)
    pk = synth.make_packets(cfg, n_flows=n)
    thr = oracle.default_threads()
    o_feat, _ = oracle.featurize(pk.flow_off, pk.pkt_size, pk.pkt_iat, pk.pkt_dir, cfg.depths, n_threads=thr)
    forest = synth.make_forest(cfg, o_feat[:cfg.calib_flows])
    mlp = synth.make_mlp(cfg, o_feat[:cfg.calib_flows])
    _, o_pred, o_top, _ = oracle.fast_infer(o_feat, forest, want_votes=False, n_threads=thr)
    o_esc = oracle.route(o_top, o_pred, vmin)

    dev = "cuda:0"
    ctx = sf.ServeFlow(sf.sf_workspace_bytes(n, cfg.n_trees, cfg.tree_depth, *mlp.dims[:3]))
    d_pk, d_forest, d_mlp = sf.packets_to_device(pk, dev), sf.forest_to_device(forest, dev), sf.mlp_to_device(mlp, dev)
    feat = torch.empty((n, cfg.n_features), dtype=torch.float32, device=dev)
    pred = torch.empty(n, dtype=torch.int16, device=dev)
    top = torch.empty(n, dtype=torch.int16, device=dev)
    esc_idx = torch.full((n,), -1, dtype=torch.int32, device=dev)
    esc_count = torch.zeros(1, dtype=torch.int32, device=dev)
    labels = torch.empty(n, dtype=torch.int16, device=dev)
    logits = torch.full((n, cfg.n_classes), float("nan"), dtype=torch.float32, device=dev)
    ctx.sf_forest_pack(d_forest)        # models laid out once, as in the benchmark
    ctx.sf_mlp_order(d_mlp)
    for _ in range(2):          # twice: the second pass runs on a warm workspace, as in the benchmark
        ctx.sf_featurize(d_pk, cfg.depths, feat)
        ctx.sf_fast_infer(feat, d_forest, pred, top)
        ctx.sf_route(top, pred, vmin, esc_idx, esc_count)
        ctx.sf_slow_infer(d_mlp, esc_idx, esc_count, labels, feat=feat, logits=logits, pred=pred)
    torch.cuda.synchronize()

    g_feat = feat.cpu().numpy()
    assert np.array_equal(g_feat.view(np.uint32), o_feat.view(np.uint32)), \
        "first differing flow %d" % int(np.argwhere(g_feat.view(np.uint32) != o_feat.view(np.uint32))[0, 0])
    del g_feat
    assert np.array_equal(pred.cpu().numpy().view(np.uint16), o_pred)
    assert np.array_equal(top.cpu().numpy().view(np.uint16), o_top)
    cnt = int(esc_count.cpu().numpy().view(np.uint32)[0])
    assert cnt == o_esc.size
    g_esc = esc_idx.cpu().numpy().view(np.uint32)[:cnt]
    assert np.array_equal(g_esc, o_esc)
    # properties that hold at any size: ascending, exactly the flows below the threshold
    assert np.all(np.diff(g_esc.astype(np.int64)) > 0)
    assert np.array_equal(g_esc, np.flatnonzero(o_top < vmin).astype(np.uint32))

    stride = max(1, cnt // logit_sample)
    rows = np.arange(0, cnt, stride)
    sub = o_esc[rows]
    o_logits, o_lab = oracle.slow_infer(sub, mlp, n, feat=o_feat, n_threads=thr)
    g_logits = logits.cpu().numpy()[rows]
    err = np.abs(g_logits - o_logits)
    assert np.all(np.isfinite(g_logits)) and err.max() <= 2e-2, err.max()
    srt = np.sort(o_logits, axis=1)
    clear = (srt[:, -1] - srt[:, -2]) > 5e-2
    g_lab = labels.cpu().numpy().view(np.uint16)
    assert clear.mean() > 0.5
    assert np.array_equal(g_lab[sub][clear], o_lab[sub][clear])
    kept = np.ones(n, bool)
    kept[o_esc] = False
    assert np.array_equal(g_lab[kept], o_pred[kept])
    return cnt / n, float(err.max())


def test_headline_workload_full_size():
    frac, err = _full(2, 1 << 20, 14, 32768)
    assert 0.15 < frac < 0.20          # the multinomial closed form gives 17.3 % below 14 of 100 votes


def test_streaming_batch_full_size():
    frac, err = _full(4, 65536, 18, 4096)
    assert 0.15 < frac < 0.27


def test_three_tier_full_size():
    """The cascade at 1,048,576 flows in the launch configuration bench.py times: the tree writes the label
    array directly, the forest's list form and the MLP overwrite their flows.  Every integer result is
    compared on every flow; logits on a fixed-stride sample of the flows that reach the MLP."""
    import torch
    import paper_2402_03694_amd as sf
    cfg = synth.get_config(6)
    n = cfg.n_flows
    pk = synth.make_packets(cfg)
    thr = oracle.default_threads()
    o_feat, _ = oracle.featurize(pk.flow_off, pk.pkt_size, pk.pkt_iat, pk.pkt_dir, cfg.depths, n_threads=thr)
    calib = o_feat[:cfg.calib_flows]
    tree, forest, mlp = synth.make_tree(cfg, calib), synth.make_forest(cfg, calib), synth.make_mlp(cfg, calib)
    o_pred0, o_top0, o_tot0, _ = oracle.tree_infer(o_feat, tree, n_threads=thr)
    o_esc1 = oracle.route_ratio(o_top0, o_tot0, cfg.theta0)
    _, o_pred1, o_top1, _ = oracle.fast_infer(o_feat[o_esc1], forest, want_votes=False, n_threads=thr)
    o_esc2 = o_esc1[oracle.route(o_top1, o_pred1, cfg.vmin)]

    dev = "cuda:0"
    ctx = sf.ServeFlow(sf.sf_workspace_bytes(n, cfg.n_trees, cfg.tree_depth, *mlp.dims[:3]))
    d_pk = sf.packets_to_device(pk, dev)
    d_tree, d_forest, d_mlp = sf.tree_to_device(tree, dev), sf.forest_to_device(forest, dev), sf.mlp_to_device(mlp, dev)
    feat = torch.empty((n, cfg.n_features), dtype=torch.float32, device=dev)
    i16 = lambda: torch.full((n,), -1, dtype=torch.int16, device=dev)
    top0, tot0, pred1, top1, labels = i16(), i16(), i16(), i16(), i16()
    esc1 = torch.full((n,), -1, dtype=torch.int32, device=dev)
    esc2 = torch.full((n,), -1, dtype=torch.int32, device=dev)
    cnt1 = torch.zeros(1, dtype=torch.int32, device=dev)
    cnt2 = torch.zeros(1, dtype=torch.int32, device=dev)
    logits = torch.full((n, cfg.n_classes), float("nan"), dtype=torch.float32, device=dev)
    ctx.sf_forest_pack(d_forest)
    ctx.sf_mlp_order(d_mlp)
    for _ in range(2):
        ctx.sf_featurize(d_pk, cfg.depths, feat)
        ctx.sf_fastest_infer(feat, d_tree, labels, top0, tot0)
        ctx.sf_route_ratio(top0, tot0, cfg.theta0, esc1, cnt1)
        ctx.sf_fast_infer_subset(feat, esc1, cnt1, d_forest, pred1, top1, labels=labels)
        ctx.sf_route_subset(top1, pred1, esc1, cnt1, cfg.vmin, esc2, cnt2)
        ctx.sf_slow_infer(d_mlp, esc2, cnt2, labels, feat=feat, logits=logits)
    torch.cuda.synchronize()

    u16 = lambda t: t.cpu().numpy().view(np.uint16)
    u32 = lambda t: t.cpu().numpy().view(np.uint32)
    assert np.array_equal(u16(top0), o_top0) and np.array_equal(u16(tot0), o_tot0)
    n1, n2 = int(u32(cnt1)[0]), int(u32(cnt2)[0])
    assert n1 == o_esc1.size and np.array_equal(u32(esc1)[:n1], o_esc1)
    assert np.array_equal(u16(pred1)[:n1], o_pred1) and np.array_equal(u16(top1)[:n1], o_top1)
    assert n2 == o_esc2.size and np.array_equal(u32(esc2)[:n2], o_esc2)
    assert 0.3 < n1 / n < 0.6 and 0.03 < n2 / n < 0.12
    g_lab = u16(labels)
    want = o_pred0.copy()
    want[o_esc1] = o_pred1
    rest = np.ones(n, bool)
    rest[o_esc2] = False
    assert np.array_equal(g_lab[rest], want[rest])
    rows = np.arange(0, n2, max(1, n2 // 32768))
    sub = o_esc2[rows]
    o_logits, o_lab = oracle.slow_infer(sub, mlp, n, feat=o_feat, n_threads=thr)
    err = np.abs(logits.cpu().numpy()[rows] - o_logits)
    assert err.max() <= 2e-2, err.max()
    srt = np.sort(o_logits, axis=1)
    clear = (srt[:, -1] - srt[:, -2]) > 5e-2
    assert np.array_equal(g_lab[sub][clear], o_lab[sub][clear])
