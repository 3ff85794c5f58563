"""The four calls of the hot path captured into a HIP graph and replayed: every replay must reproduce the
eager results (which the parity tests tie to the oracle).  Between replays the outputs are overwritten and
other eager work runs, so a replay that depended on anything but the graph's own nodes would show."""
import numpy as np
import pytest

import oracle
import synth

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("cfg_id,n,vmin", [(2, 20000 + 11, 14), (4, 8000 + 3, 18), (1, 4096, 7)])
def test_graph_replay_matches_eager_and_oracle(cfg_id, n, vmin):
    import torch
    import paper_2402_03694_amd as sf
    cfg = synth.get_config(cfg_id)
    pk = synth.make_packets(cfg, n_flows=n)
    o_feat, _ = oracle.featurize(pk.flow_off, pk.pkt_size, pk.pkt_iat, pk.pkt_dir, cfg.depths, n_threads=8)
    forest, mlp = synth.make_forest(cfg, o_feat[:4096]), synth.make_mlp(cfg, o_feat[:4096])
    _, o_pred, o_top, _ = oracle.fast_infer(o_feat, forest, want_votes=False, n_threads=8)
    o_esc = oracle.route(o_top, o_pred, vmin)

    dev = "cuda:0"
    stream = torch.cuda.Stream()                       # default priority
    ctx = sf.ServeFlow(sf.sf_workspace_bytes(n, cfg.n_trees, cfg.tree_depth, *mlp.dims[:3]), stream=stream)
    d_pk, d_forest, d_mlp = sf.packets_to_device(pk, dev), sf.forest_to_device(forest, dev), sf.mlp_to_device(mlp, dev)
    feat = torch.zeros((n, cfg.n_features), dtype=torch.float32, device=dev)
    pred = torch.zeros(n, dtype=torch.int16, device=dev)
    top = torch.zeros(n, dtype=torch.int16, device=dev)
    esc = torch.zeros(n, dtype=torch.int32, device=dev)
    cnt = torch.zeros(1, dtype=torch.int32, device=dev)
    labels = torch.zeros(n, dtype=torch.int16, device=dev)
    logits = torch.zeros((n, cfg.n_classes), dtype=torch.float32, device=dev)
    outs = (feat, pred, top, esc, cnt, labels, logits)

    def step():
        ctx.sf_featurize(d_pk, cfg.depths, feat)
        ctx.sf_fast_infer(feat, d_forest, pred, top)
        ctx.sf_route(top, pred, vmin, esc, cnt)
        ctx.sf_slow_infer(d_mlp, esc, cnt, labels, feat=feat, logits=logits, pred=pred)

    torch.cuda.synchronize()
    with torch.cuda.stream(stream):
        step()                                          # eager, also warms every kernel up before the capture
    stream.synchronize()
    eager = [t.clone() for t in outs]
    k = int(eager[4].cpu().numpy().view(np.uint32)[0])
    assert k == o_esc.size and np.array_equal(eager[3].cpu().numpy().view(np.uint32)[:k], o_esc)
    assert np.array_equal(eager[0].cpu().numpy().view(np.uint32), o_feat.view(np.uint32))

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        step()
    for rep in range(4):
        for t in outs:                                  # wipe the outputs, run unrelated eager work
            t.fill_(-3)
        junk = torch.randn(1 << 20, device=dev).sum()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, got, want in zip(("feat", "pred", "top", "esc", "cnt", "labels", "logits"), outs, eager):
            if name == "esc":
                assert torch.equal(got[:k], want[:k]), (rep, name)
            elif name == "logits":
                assert torch.equal(got[:k], want[:k]), (rep, name)
            else:
                assert torch.equal(got, want), (rep, name)
        del junk
