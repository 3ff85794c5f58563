"""Empty and degenerate inputs of the entry points beyond the four basic ones: nothing is launched on
nothing, counts come back as zero, and a request that cannot be answered is an error, not a crash."""
import numpy as np
import pytest

import oracle
import synth

pytestmark = pytest.mark.gpu


def _u32(t):
    return t.cpu().numpy().view(np.uint32)


def test_empty_inputs_everywhere():
    import torch
    import paper_2402_03694_amd as sf
    dev = "cuda:0"
    cfg6, cfg7 = synth.get_config(6), synth.get_config(7)
    pk = synth.make_packets(cfg6, n_flows=300)
    feat_np, _ = oracle.featurize(pk.flow_off, pk.pkt_size, pk.pkt_iat, pk.pkt_dir, cfg6.depths)
    tree, forest, mlp = synth.make_tree(cfg6, feat_np), synth.make_forest(cfg6, feat_np), synth.make_mlp(cfg6, feat_np)
    gbdt = synth.make_gbdt(cfg7, feat_np)
    ctx = sf.ServeFlow(sf.sf_workspace_bytes(300, cfg7.n_trees, 12, *mlp.dims[:3]))
    feat = torch.from_numpy(feat_np).to(dev)
    empty_feat = feat[:0]
    i16 = lambda n, v=-7: torch.full((n,), v, dtype=torch.int16, device=dev)
    i32 = lambda n, v=-7: torch.full((n,), v, dtype=torch.int32, device=dev)
    f32 = lambda n, v=-7.0: torch.full((n,), v, dtype=torch.float32, device=dev)
    cnt = i32(1)
    a, b, c = i16(4), i16(4), i16(4)
    # no flows: the outputs stay untouched
    ctx.sf_fastest_infer(empty_feat, sf.tree_to_device(tree), a, b, c, n_flows=0)
    ctx.sf_gbdt_infer(empty_feat, sf.gbdt_to_device(gbdt), sf.SF_SCORE_LC, a, f32(4), n_flows=0)
    ctx.sf_route_ratio(b, c, 0.5, i32(4), cnt, n_flows=0)
    torch.cuda.synchronize()
    assert int(_u32(cnt)[0]) == 0 and np.all(a.cpu().numpy() == -7)
    cnt.fill_(-7)
    ctx.sf_route_score(f32(4), 0.5, i32(4), cnt, n_flows=0)
    torch.cuda.synchronize()
    assert int(_u32(cnt)[0]) == 0
    # a list of capacity zero, and a list whose device-side length is zero
    zero = torch.zeros(1, dtype=torch.int32, device=dev)
    idx = i32(8, 3)
    p1, t1 = i16(8), i16(8)
    ctx.sf_fast_infer_subset(feat, idx, zero, sf.forest_to_device(forest), p1, t1, idx_cap=0)
    ctx.sf_fast_infer_subset(feat, idx, zero, sf.forest_to_device(forest), p1, t1)
    cnt.fill_(-7)
    ctx.sf_route_subset(t1, p1, idx, zero, 14, i32(8), cnt)
    torch.cuda.synchronize()
    assert int(_u32(cnt)[0]) == 0 and np.all(p1.cpu().numpy() == -7)
    cnt.fill_(-7)
    ctx.sf_route_subset(t1, p1, idx, zero, 14, i32(8), cnt, idx_cap=0)
    torch.cuda.synchronize()
    assert int(_u32(cnt)[0]) == 0
    # the slow model on no pairs
    labels = i16(300, 5)
    ctx.sf_slow_infer_pairs(sf.mlp_to_device(mlp), feat, idx, idx, zero, labels)
    ctx.sf_slow_infer_pairs(sf.mlp_to_device(mlp), feat, idx, idx, cnt, labels, pair_cap=0)
    torch.cuda.synchronize()
    assert np.all(labels.cpu().numpy() == 5)
    # quantiles of nothing cannot be answered
    with pytest.raises(sf.ServeFlowError) as e:
        ctx.sf_score_quantiles(f32(4), [0.5], n_flows=0)
    assert e.value.code == -1


def test_one_flow_through_every_model():
    """a single flow: partial waves everywhere"""
    import torch
    import paper_2402_03694_amd as sf
    dev = "cuda:0"
    cfg6, cfg7 = synth.get_config(6), synth.get_config(7)
    pk = synth.make_packets(cfg6, n_flows=4100)
    feat_all, _ = oracle.featurize(pk.flow_off, pk.pkt_size, pk.pkt_iat, pk.pkt_dir, cfg6.depths, n_threads=8)
    tree, gbdt = synth.make_tree(cfg6, feat_all[:4096]), synth.make_gbdt(cfg7, feat_all[:4096])
    one = np.ascontiguousarray(feat_all[4099:4100])
    ctx = sf.ServeFlow(sf.sf_workspace_bytes(1, cfg7.n_trees, cfg7.tree_depth))
    feat = torch.from_numpy(one).to(dev)
    a, b, c = (torch.zeros(1, dtype=torch.int16, device=dev) for _ in range(3))
    ctx.sf_fastest_infer(feat, sf.tree_to_device(tree), a, b, c)
    score = torch.zeros(1, dtype=torch.float32, device=dev)
    pred = torch.zeros(1, dtype=torch.int16, device=dev)
    ctx.sf_gbdt_infer(feat, sf.gbdt_to_device(gbdt), sf.SF_SCORE_ENTROPY, pred, score)
    torch.cuda.synchronize()
    o_pred, o_top, o_tot, _ = oracle.tree_infer(one, tree)
    assert (int(a[0]), int(b[0]), int(c[0])) == (int(o_pred[0]), int(o_top[0]), int(o_tot[0]))
    _, g_pred, _, g_ent = oracle.gbdt_infer(one, gbdt)
    assert int(pred[0]) == int(g_pred[0]) and abs(float(score[0]) - g_ent[0]) < 1e-6
    assert ctx.sf_score_quantiles(score, [0.0, 0.5, 1.0]) == [float(score[0])] * 3
