"""sf_classify (all four steps in one call; features, forest and score in one kernel where the shape allows)
against the CPU oracle, element by element: pred, top_votes, the escalation list, logits, final labels, and
the feature rows of the escalated flows (the only rows the fused kernel writes)."""
from dataclasses import replace

import numpy as np
import pytest

import oracle
import synth

pytestmark = pytest.mark.gpu

BF16_TOL, BF16_MARGIN = 2e-2, 5e-2
F32_TOL, F32_MARGIN = 1e-4, 1e-3
SENTINEL = -777.0


def _classify(cfg, pk, forest, mlp, vmin, feat_ld=None, use_feat=True):
    import torch
    import paper_2402_03694_amd as sf
    dev, n = "cuda:0", pk.n_flows
    ctx = sf.ServeFlow(sf.sf_workspace_bytes(max(n, 1), forest.n_trees, forest.depth, *mlp.dims[:3]))
    d_pk, d_forest, d_mlp = sf.packets_to_device(pk, dev), sf.forest_to_device(forest, dev), sf.mlp_to_device(mlp, dev)
    ld = cfg.n_features if feat_ld is None else feat_ld
    feat = torch.full((n, ld), SENTINEL, dtype=torch.float32, device=dev) if use_feat else None
    pred = torch.full((n,), -1, dtype=torch.int16, device=dev)
    top = torch.full((n,), -1, dtype=torch.int16, device=dev)
    esc_idx = torch.full((max(n, 1),), -1, dtype=torch.int32, device=dev)
    esc_count = torch.full((1,), -1, dtype=torch.int32, device=dev)
    labels = torch.full((n,), -1, dtype=torch.int16, device=dev)
    logits = torch.full((max(n, 1), mlp.dims[3]), float("nan"), dtype=torch.float32, device=dev)
    for _ in range(2):      # the second call runs on a warm workspace
        ctx.sf_classify(d_pk, cfg.depths, d_forest, vmin, d_mlp, feat, pred, top, esc_idx, esc_count, labels, logits=logits,
                        raw_pkts=cfg.raw_pkts, raw_bits=cfg.raw_bits)
    torch.cuda.synchronize()
    u16 = lambda t: t.cpu().numpy().view(np.uint16)
    cnt = int(esc_count.cpu().numpy().view(np.uint32)[0])
    return dict(feat=None if feat is None else feat.cpu().numpy(), pred=u16(pred), top=u16(top),
                esc=esc_idx.cpu().numpy().view(np.uint32)[:cnt].copy(), labels=u16(labels), logits=logits.cpu().numpy()[:cnt])


def _check(cfg, pk, forest, mlp, vmin, fused, **kw):
    want = oracle.classify(pk, cfg.depths, forest, vmin, mlp, raw_pkts=cfg.raw_pkts, raw_bits=cfg.raw_bits, n_threads=8)
    got = _classify(cfg, pk, forest, mlp, vmin, **kw)
    n, F = pk.n_flows, cfg.n_features
    assert np.array_equal(got["pred"], want["pred"]) and np.array_equal(got["top"], want["top_votes"])
    assert np.array_equal(got["esc"], want["esc_idx"])
    esc = want["esc_idx"]
    bf = cfg.mlp_dtype == "bf16"
    tol, margin = (BF16_TOL, BF16_MARGIN) if bf else (F32_TOL, F32_MARGIN)
    if esc.size:
        err = np.abs(got["logits"] - want["logits"])
        assert np.all(np.isfinite(got["logits"])) and err.max() <= tol, err.max()
        srt = np.sort(want["logits"], axis=1)
        clear = (srt[:, -1] - srt[:, -2]) > margin
        assert np.array_equal(got["labels"][esc][clear], want["labels"][esc][clear])
    kept = np.ones(n, bool)
    kept[esc] = False
    assert np.array_equal(got["labels"][kept], want["pred"][kept])
    if got["feat"] is not None:
        g = got["feat"]
        assert np.array_equal(g[esc, :F].view(np.uint32), want["feat"][esc].view(np.uint32))
        assert np.all(g[:, F:] == SENTINEL)
        if fused and not cfg.raw_pkts:
            assert np.all(g[kept] == SENTINEL)       # rows of flows that stay with the fast model never left the chip
        elif not fused:
            assert np.array_equal(g[:, :F].view(np.uint32), want["feat"].view(np.uint32))
    return esc.size


def _models(cfg, pk):
    feat, _ = oracle.featurize(pk.flow_off, pk.pkt_size, pk.pkt_iat, pk.pkt_dir, cfg.depths, n_threads=8)
    return synth.make_forest(cfg, feat[:4096]), synth.make_mlp(cfg, None if cfg.raw_pkts else feat[:4096])


@pytest.mark.parametrize("cfg_id,n,vmin", [(1, 4096 + 37, 7), (2, 6000 + 13, 15), (2, 300, 14), (2, 1, 101)])
def test_fused_shapes(cfg_id, n, vmin):
    cfg = synth.get_config(cfg_id)
    pk = synth.make_packets(cfg, n_flows=n)
    forest, mlp = _models(cfg, pk)
    assert _check(cfg, pk, forest, mlp, vmin, fused=True) > 0


def test_fused_per_class_thresholds_and_wide_rows():
    cfg = synth.get_config(2)
    pk = synth.make_packets(cfg, n_flows=5000 + 3)
    forest, mlp = _models(cfg, pk)
    vm = [14, 19, 0, 17, 12, 0, 16, 15, 13, 101]
    assert _check(cfg, pk, forest, mlp, vm, fused=True, feat_ld=72) > 500
    assert _check(cfg, pk, forest, mlp, vm, fused=True, feat_ld=67) > 500       # rows off the 16-byte grid


def test_fused_ragged_flows_and_empty_list():
    """Ragged flows (1..64 packets, windows of 3 and 16), zero-length flows; a threshold nothing is below."""
    cfg = replace(synth.get_config(2), pkts_per_flow=None, depths=(3, 16))
    pk = synth.make_packets(cfg, n_flows=3000 + 11)
    off = pk.flow_off.copy()
    off[10] = off[9]
    off[700:703] = off[699]
    pk.flow_off = np.maximum.accumulate(off)
    forest, mlp = _models(cfg, pk)
    assert _check(cfg, pk, forest, mlp, 15, fused=True) > 300
    assert _check(cfg, pk, forest, mlp, 0, fused=True) == 0


def test_fused_forest_on_fewer_columns_than_the_tile():
    """The cascade's forest splits on the first window's 32 columns only; the tile still holds both windows."""
    cfg = synth.get_config(6)
    pk = synth.make_packets(cfg, n_flows=4000 + 5)
    forest, mlp = _models(cfg, pk)
    assert forest.n_features == 32 and cfg.n_features == 64
    assert _check(cfg, pk, forest, mlp, 14, fused=True) > 300


def test_fused_header_bit_slow_model_without_a_feature_matrix():
    """Deep forest in front of the header-bit model: the fused kernel writes no feature row at all."""
    cfg = replace(synth.get_config(3), tree_depth=12)
    pk = synth.make_packets(cfg, n_flows=1500 + 5)
    forest, mlp = _models(cfg, pk)
    assert _check(cfg, pk, forest, mlp, 14, fused=True, use_feat=False) > 100


def test_fused_where_the_separate_forest_would_share_flows_between_lanes():
    """Workload 3 as it stands (depth 10: the stand-alone forest kernel runs two lanes per flow): the fused kernel
    runs one lane per flow and, the slow model reading header bits, writes no feature row."""
    cfg = synth.get_config(3)
    pk = synth.make_packets(cfg, n_flows=1500 + 5)
    forest, mlp = _models(cfg, pk)
    assert _check(cfg, pk, forest, mlp, 14, fused=True, use_feat=False) > 100


@pytest.mark.parametrize("cfg_id,n,vmin", [(4, 3000 + 61, 19), (5, 1200 + 3, 25)])
def test_shapes_that_run_the_separate_kernels(cfg_id, n, vmin):
    cfg = synth.get_config(cfg_id)
    pk = synth.make_packets(cfg, n_flows=n)
    forest, mlp = _models(cfg, pk)
    assert _check(cfg, pk, forest, mlp, vmin, fused=False) > 0


@pytest.mark.parametrize("cfg_id,n", [(2, 3000 + 7), (4, 2000 + 3)])
def test_steps_one_to_three_alone(cfg_id, n):
    """sf_featurize_fast_infer by itself (fused for the first shape, separate kernels inside for the second):
    pred, top_votes, labels = pred, and the rows of the flows below the threshold."""
    import torch
    import paper_2402_03694_amd as sf
    cfg = synth.get_config(cfg_id)
    pk = synth.make_packets(cfg, n_flows=n)
    forest, _ = _models(cfg, pk)
    o_feat, _ = oracle.featurize(pk.flow_off, pk.pkt_size, pk.pkt_iat, pk.pkt_dir, cfg.depths, n_threads=8)
    _, o_pred, o_top, _ = oracle.fast_infer(o_feat, forest, want_votes=False, n_threads=8)
    vmin = 15 if cfg_id == 2 else 19
    dev = "cuda:0"
    ctx = sf.ServeFlow(sf.sf_workspace_bytes(n, forest.n_trees, forest.depth))
    d_pk, d_forest = sf.packets_to_device(pk, dev), sf.forest_to_device(forest, dev)
    feat = torch.full((n, cfg.n_features), SENTINEL, dtype=torch.float32, device=dev)
    pred, top, labels = (torch.full((n,), -1, dtype=torch.int16, device=dev) for _ in range(3))
    ctx.sf_featurize_fast_infer(d_pk, cfg.depths, d_forest, vmin, feat, pred, top, labels=labels)
    torch.cuda.synchronize()
    u16 = lambda t: t.cpu().numpy().view(np.uint16)
    assert np.array_equal(u16(pred), o_pred) and np.array_equal(u16(top), o_top) and np.array_equal(u16(labels), o_pred)
    esc = o_top < vmin
    g = feat.cpu().numpy()
    assert np.array_equal(g[esc].view(np.uint32), o_feat[esc].view(np.uint32))
    if cfg_id == 2:
        assert np.all(g[~esc] == SENTINEL)


def test_classify_errors_and_no_flows():
    import torch
    import paper_2402_03694_amd as sf
    cfg = synth.get_config(2)
    pk = synth.make_packets(cfg, n_flows=64)
    forest, mlp = _models(cfg, pk)
    got = _classify(cfg, pk, forest, mlp, 14)
    assert got["pred"].size == 64
    ctx = sf.ServeFlow(sf.sf_workspace_bytes(64, forest.n_trees, forest.depth, *mlp.dims[:3]))
    d_pk, d_forest, d_mlp = sf.packets_to_device(pk), sf.forest_to_device(forest), sf.mlp_to_device(mlp)
    i16 = lambda: torch.zeros(64, dtype=torch.int16, device="cuda:0")
    i32 = lambda k: torch.full((k,), -1, dtype=torch.int32, device="cuda:0")
    narrow = torch.zeros((64, 32), dtype=torch.float32, device="cuda:0")
    with pytest.raises(sf.ServeFlowError) as e:
        ctx.sf_classify(d_pk, cfg.depths, d_forest, 14, d_mlp, narrow, i16(), i16(), i32(64), i32(1), i16())
    assert e.value.code == -1 and "feat_ld" in str(e.value)
    with pytest.raises(sf.ServeFlowError) as e:
        ctx.sf_classify(d_pk, [8], d_forest, 14, d_mlp, narrow, i16(), i16(), i32(64), i32(1), i16())
    assert e.value.code == -1 and "forest" in str(e.value)
    empty = sf.DevicePackets(d_pk.flow_off[:1], d_pk.pkt_size[:0], d_pk.pkt_iat[:0], d_pk.pkt_dir[:0])
    cnt = i32(1)
    feat = torch.zeros((0, 64), dtype=torch.float32, device="cuda:0")
    ctx.sf_classify(empty, cfg.depths, d_forest, 14, d_mlp, feat, i16()[:0], i16()[:0], i32(1), cnt, i16()[:0])
    torch.cuda.synchronize()
    assert int(cnt.cpu().numpy().view(np.uint32)[0]) == 0
