"""sf_route_static (the gate for callers that cannot allocate: its block counts live in a static
device array of the library) against sf_route, through the C ABI, bit for bit: two calls in a row on
one GPU, the second with a smaller input, so that what the first call left in the array is still
there; then the per-class form and the size limit."""
import ctypes

import numpy as np
import pytest

import oracle

pytestmark = pytest.mark.gpu


def _scores(n, n_trees, n_classes, seed):
    rng = np.random.default_rng(seed)
    top = rng.integers(0, n_trees + 1, size=n, dtype=np.uint16)
    pred = rng.integers(0, n_classes, size=n, dtype=np.uint16)
    return top, pred


def _both(ctx, sf, top, pred, vmin):
    """Escalation list and count from sf_route and from sf_route_static on the same device arrays."""
    import torch
    dev = "cuda:0"
    n = top.size
    d_top = torch.from_numpy(top.view(np.int16)).to(dev)
    d_pred = torch.from_numpy(pred.view(np.int16)).to(dev)
    out = []
    for call in (ctx.sf_route, ctx.sf_route_static):
        idx = torch.full((max(n, 1),), -1, dtype=torch.int32, device=dev)
        cnt = torch.full((1,), -1, dtype=torch.int32, device=dev)
        call(d_top, d_pred, vmin, idx, cnt)
        torch.cuda.synchronize()
        c = int(cnt.cpu().numpy().view(np.uint32)[0])
        out.append((idx.cpu().numpy().view(np.uint32)[:c].copy(), c))
    return out


def test_static_scratch_gate_matches_workspace_gate():
    import paper_2402_03694_amd as sf
    ctx = sf.ServeFlow(sf.sf_workspace_bytes(1 << 20))
    # first call: 1,000,003 flows (several blocks, a ragged tail); second: 70,001 flows, fewer blocks
    for n, vmin, seed in ((1000003, 40, 11), (70001, 55, 12)):
        top, pred = _scores(n, 100, 10, seed)
        (want, wc), (got, gc) = _both(ctx, sf, top, pred, vmin)
        assert gc == wc and np.array_equal(got, want), "n = %d" % n
        assert np.array_equal(got, oracle.route(top, pred, vmin))
    # per-class thresholds, smaller again, and an input of one flow
    top, pred = _scores(3001, 100, 10, 13)
    vm = [30, 35, 40, 45, 50, 55, 60, 65, 70, 75]
    (want, wc), (got, gc) = _both(ctx, sf, top, pred, vm)
    assert gc == wc and np.array_equal(got, want)
    assert np.array_equal(got, oracle.route(top, pred, np.array(vm, np.uint16)))
    top, pred = _scores(1, 100, 10, 14)
    (want, wc), (got, gc) = _both(ctx, sf, top, pred, 101)
    assert gc == wc == 1 and np.array_equal(got, want)


def test_static_scratch_gate_on_a_second_context_and_empty_input():
    """The array belongs to the GPU, not to a context: a second context finds it in use by nobody."""
    import torch
    import paper_2402_03694_amd as sf
    a, b = sf.ServeFlow(4096), sf.ServeFlow(1 << 20)
    top, pred = _scores(250007, 200, 16, 15)
    (want, wc), (got, gc) = _both(b, sf, top, pred, 90)
    assert gc == wc and np.array_equal(got, want)
    # context a has a workspace too small for sf_route's block counts; the static form does not need it
    d_top = torch.from_numpy(top.view(np.int16)).to("cuda:0")
    idx = torch.full((top.size,), -1, dtype=torch.int32, device="cuda:0")
    cnt = torch.full((1,), -1, dtype=torch.int32, device="cuda:0")
    a.sf_route_static(d_top, None, 90, idx, cnt)
    torch.cuda.synchronize()
    assert int(cnt.cpu().numpy().view(np.uint32)[0]) == wc
    assert np.array_equal(idx.cpu().numpy().view(np.uint32)[:wc], want)
    a.sf_route_static(d_top, None, 90, idx, cnt, n_flows=0)
    torch.cuda.synchronize()
    assert int(cnt.cpu().numpy().view(np.uint32)[0]) == 0


def test_static_scratch_gate_rejects_sizes_beyond_its_limit():
    import torch
    import paper_2402_03694_amd as sf
    from paper_2402_03694_amd import binding
    ctx = sf.ServeFlow(4096)
    buf = torch.zeros(16, dtype=torch.int32, device="cuda:0")
    vm = (ctypes.c_uint16 * 1)(5)
    p = ctypes.c_void_p(buf.data_ptr())
    rc = binding.lib().sf_route_static(ctx._h, p, None, 2147483649, vm, 1, p, p)   # refused before any launch
    assert rc == binding.SF_EUNSUPPORTED
    assert b"at most" in binding.lib().sf_last_error(ctx._h)
