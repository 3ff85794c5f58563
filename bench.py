#!/usr/bin/env python3
"""Throughput of the whole hot path (featurize -> fast trees -> gate -> slow MLP) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2] [--no-cpu-baseline]

A step is one pass of all four calls over one batch of synthetic flows that is already resident
in HBM.  Prints one JSON line: flows/s, ms per step, the roofline of the dominant kernel (and of
every call, under "kernels"), and the CPU oracle timed on this host's cores on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16, published
F32_VECTOR_PEAK_TFLOPS = 157.3
NOMINAL_CLOCK_HZ = 2.4e9
TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
CSRC = os.path.join(ROOT, "paper_2402_03694_amd", "csrc")


def source_digest(files):
    """First 16 hex digits of the SHA-256 over the named kernel source files, in the order given."""
    import hashlib
    h = hashlib.sha256()
    for f in files:
        with open(os.path.join(CSRC, f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def measured_traffic(call, cfg_id, n_flows):
    """HBM bytes per launch from the committed counter table (rocprofv3 FETCH_SIZE / WRITE_SIZE runs, each
    scaled by what the counter reads for a device copy of known size), or None: when the table has no line for
    this workload and call, or the kernel sources named on the line have changed since the counters were taken.
    Line format: <config> <flows> <call> <bytes per launch> <comma-separated source files> <digest of them>."""
    try:
        with open(TRAFFIC_TABLE) as f:
            lines = [l.split() for l in f if l.strip() and not l.startswith("#")]
    except OSError:
        return None
    for l in lines:
        if len(l) == 6 and l[0] == "cfg%d" % cfg_id and int(l[1]) == n_flows and l[2] == call:
            try:
                return int(l[3]) if source_digest(l[4].split(",")) == l[5] else None
            except OSError:
                return None
    return None


def gather_probe(ctx, dev):
    """What a 64-lane gather costs a compute unit on this device, in nominal clock cycles, measured with the
    library's probe kernel (eight dependent chains per lane, eight blocks of 256 lanes per unit): the numbers
    the tree walk is priced against.  A node visit needs one 4-byte feature gather from the lane's own
    shared-memory column and half a 16-byte record gather (a record holds two levels); if every record came
    from shared memory a unit could retire 64 / (c_column + c_record / 2) lane-visits per clock."""
    import torch
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    table = torch.randint(-2 ** 31, 2 ** 31 - 1, (1 << 22,), dtype=torch.int32, device=dev)   # 2^20 records, 16 MB
    blocks, iters = 8 * n_cu, 1024
    sink = torch.empty(blocks * 256, dtype=torch.int32, device=dev)
    out = {}
    for name, kind, log2 in (("lds_column_b32", 0, 12), ("lds_random_b128", 1, 12), ("l1_random_b128", 2, 10),
                             ("l2_random_b128", 2, 17)):
        tab = table[: 4 << log2]
        ctx.sf_probe_gather(kind, tab, sink, iters, blocks)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        done = ctx.sf_probe_gather(kind, tab, sink, iters, blocks)
        e1.record()
        torch.cuda.synchronize()
        out[name + "_cycles"] = e0.elapsed_time(e1) * 1e-3 * NOMINAL_CLOCK_HZ * n_cu / done
    out["clock_hz"] = NOMINAL_CLOCK_HZ
    out["compute_units"] = n_cu
    out["bound_visits_per_s"] = 64.0 / (out["lds_column_b32_cycles"] + out["lds_random_b128_cycles"] / 2.0) * n_cu * NOMINAL_CLOCK_HZ
    return out


def copy_bandwidth(dev):
    """What a plain device-to-device copy of 256 MiB reaches on this device (bytes read + bytes written per second,
    in GB/s): the practical ceiling next to the published HBM peak the rooflines are priced at."""
    import torch
    src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    for _ in range(2):
        dst.copy_(src)
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(6)]
    for i in range(5):
        ev[i].record()
        dst.copy_(src)
    ev[5].record()
    torch.cuda.synchronize()
    ms = float(np.median([ev[i].elapsed_time(ev[i + 1]) for i in range(5)]))
    return 2.0 * (256 << 20) / (ms * 1e-3) / 1e9


def algorithmic_bytes(cfg, n_flows, n_pkts, esc_frac):
    """Bytes the method itself must move per call (inputs read once + outputs written once)."""
    F = cfg.n_features
    k1 = 7 * n_pkts + 4 * (n_flows + 1) + 4 * F * n_flows           # packet records + offsets + features out
    k2 = 4 * F * n_flows + 4 * n_flows                              # features in + pred/top out
    k3 = 2 * n_flows + 4 * esc_frac * n_flows                       # scores in + index list out
    return k1, k2, k3


def mlp_flops(cfg, n_rows):
    a, b, c, d = cfg.mlp_dims
    return 2.0 * (a * b + b * c + c * d) * n_rows


def _oracle_cost_per_flow(cfg, esc_frac):
    """Rough CPU seconds per flow of the oracle on one core (to bound the timed sample, nothing else)."""
    a, b, c, d = cfg.mlp_dims
    pk = cfg.pkts_per_flow or 10
    return 60e-9 * pk * len(cfg.depths) + 9e-9 * cfg.n_trees * cfg.tree_depth + esc_frac * 1.5e-9 * (a * b + b * c + c * d)


def _oracle_pass(cfg, pk, models, vmin, threads):
    """One timed pass of the oracle over pk: (seconds per stage, escalated count)."""
    import oracle
    st = {}
    t0 = time.perf_counter()
    feat, _ = oracle.featurize(pk.flow_off, pk.pkt_size, pk.pkt_iat, pk.pkt_dir, cfg.depths, n_threads=threads)
    st["featurize"] = time.perf_counter() - t0
    t0 = time.perf_counter()
    if cfg.fast_kind == "gbdt":
        _, pred, lc, ent = oracle.gbdt_infer(feat, models["fast"], want_margins=False, n_threads=threads)
        st["fast"] = time.perf_counter() - t0
        t0 = time.perf_counter()
        esc = oracle.route_score((ent if cfg.score == "entropy" else lc).astype(np.float32), vmin)
    else:
        _, pred, top, _ = oracle.fast_infer(feat, models["fast"], want_votes=False, n_threads=threads)
        st["fast"] = time.perf_counter() - t0
        t0 = time.perf_counter()
        esc = oracle.route(top, pred, vmin)
    st["route"] = time.perf_counter() - t0
    t0 = time.perf_counter()
    if cfg.raw_pkts:
        oracle.slow_infer(esc, models["mlp"], pk.n_flows, flow_off=pk.flow_off, pkt_hdr=pk.pkt_hdr, raw_pkts=cfg.raw_pkts,
                          raw_bits=cfg.raw_bits, labels=pred.copy(), n_threads=threads)
    else:
        oracle.slow_infer(esc, models["mlp"], pk.n_flows, feat=feat, labels=pred.copy(), n_threads=threads)
    st["slow"] = time.perf_counter() - t0
    return st, esc.size


def cpu_baseline(cfg, n, vmin, esc_frac, budget_s=20.0):
    """The oracle as it stands, all four steps, on a bounded sample of the same workload, twice: with its outer
    parallel-for on the host's cores (the figure reported as the baseline), and on one thread over the first
    flows of the sample (per-flow work is independent and identically distributed, so flows/s carries over to
    the full size: an extrapolation, and said so).  vmin: the gate's threshold(s), as the timed GPU path uses."""
    import oracle
    import synth
    threads = oracle.default_threads()
    per_flow = _oracle_cost_per_flow(cfg, esc_frac)
    sample = int(max(4096, min(n, 1 << 20, budget_s * threads / per_flow)))
    pk = synth.make_packets(cfg, n_flows=sample)
    calib, _ = oracle.featurize(pk.flow_off[: cfg.calib_flows + 1], pk.pkt_size, pk.pkt_iat, pk.pkt_dir, cfg.depths,
                                n_threads=threads)
    models = {"mlp": synth.make_mlp(cfg, None if cfg.raw_pkts else calib),
              "fast": synth.make_gbdt(cfg, calib) if cfg.fast_kind == "gbdt" else synth.make_forest(cfg, calib)}
    st, n_esc = _oracle_pass(cfg, pk, models, vmin, threads)
    dt = sum(st.values())
    out = {"value": sample / dt, "unit": "flows/s", "cores": threads, "kind": "oracle",
           "sample": "first %d flows of the workload, all four steps, %.1f s wall, %.1f%% escalated"
                     % (sample, dt, 100.0 * n_esc / sample),
           "stage_seconds": st}
    one = int(max(1024, min(sample, 65536, 0.5 * budget_s / per_flow)))
    import copy
    pk1 = copy.copy(pk)
    pk1.flow_off = pk.flow_off[: one + 1]
    st1, n_esc1 = _oracle_pass(cfg, pk1, models, vmin, 1)
    dt1 = sum(st1.values())
    out["single_thread"] = {"value": one / dt1, "unit": "flows/s", "cores": 1,
                            "sample": "first %d flows on one thread, %.1f s wall, %.1f%% escalated; flows/s carries over "
                                      "to the full %d flows by extrapolation (independent, identically distributed flows)"
                                      % (one, dt1, 100.0 * n_esc1 / one, n),
                            "stage_seconds": st1}
    return out


def three_tier(args, cfg):
    """--config 6: the cascade of Section 3.1 (tree on every flow, forest on the tree's uncertain flows,
    MLP on the forest's uncertain flows); a step is all seven calls over one device-resident batch."""
    import torch
    import synth
    import paper_2402_03694_amd as sf
    dev = "cuda:0"
    n = args.flows or cfg.n_flows
    pk = synth.make_packets(cfg, n_flows=n)
    F, C = cfg.n_features, cfg.n_classes
    ctx = sf.ServeFlow(sf.sf_workspace_bytes(n, cfg.n_trees, cfg.tree_depth, *cfg.mlp_dims[:3]))
    d_pk = sf.packets_to_device(pk, dev)
    feat = torch.empty((n, F), dtype=torch.float32, device=dev)
    i16 = lambda m: torch.empty(m, dtype=torch.int16, device=dev)
    i32 = lambda m: torch.zeros(m, dtype=torch.int32, device=dev)
    top0, tot0, pred1, top1, labels = i16(n), i16(n), i16(n), i16(n), i16(n)
    esc1, cnt1, esc2, cnt2 = i32(n), i32(1), i32(n), i32(1)
    ctx.sf_featurize(d_pk, cfg.depths, feat)
    torch.cuda.synchronize()
    calib = feat[: cfg.calib_flows].cpu().numpy()
    tree, forest, mlp = synth.make_tree(cfg, calib), synth.make_forest(cfg, calib), synth.make_mlp(cfg, calib)
    d_tree, d_forest, d_mlp = sf.tree_to_device(tree, dev), sf.forest_to_device(forest, dev), sf.mlp_to_device(mlp, dev)
    ctx.sf_validate_tree(d_tree)
    ctx.sf_validate_forest(d_forest)
    ctx.sf_forest_pack(d_forest)       # the models are laid out for the kernels once, not per batch
    ctx.sf_mlp_order(d_mlp)
    names = ["sf_featurize", "sf_fastest_infer", "sf_route_ratio", "sf_fast_infer_subset", "sf_route_subset",
             "sf_slow_infer"]

    def step(ev=None):
        rec = (lambda i: ev[i].record()) if ev else (lambda i: None)
        rec(0)
        ctx.sf_featurize(d_pk, cfg.depths, feat)
        rec(1)
        ctx.sf_fastest_infer(feat, d_tree, labels, top0, tot0)      # the tree's label is the flow's label ...
        rec(2)
        ctx.sf_route_ratio(top0, tot0, cfg.theta0, esc1, cnt1)
        rec(3)
        ctx.sf_fast_infer_subset(feat, esc1, cnt1, d_forest, pred1, top1, labels=labels)   # ... until the forest's
        rec(4)
        ctx.sf_route_subset(top1, pred1, esc1, cnt1, cfg.vmin, esc2, cnt2)
        rec(5)
        ctx.sf_slow_infer(d_mlp, esc2, cnt2, labels, feat=feat)     # ... or the MLP's replaces it (Section 4.4)
        rec(6)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(7)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for s in range(args.steps):
        step(events[s])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    n1 = int(cnt1.cpu().numpy().view(np.uint32)[0])
    n2 = int(cnt2.cpu().numpy().view(np.uint32)[0])
    call_ms = np.array([[ev[i].elapsed_time(ev[i + 1]) for i in range(6)] for ev in events])
    avg = call_ms.mean(axis=0)
    k1b, _, _ = algorithmic_bytes(cfg, n, pk.n_pkts, 0.0)
    used = cfg.tree0_features or F
    bytes_ = [k1b, (4 * used + 6) * n, 4 * n + 4 * n1, (4 * used + 4 + 4) * n1, (2 + 4) * n1 + 4 * n2, None]
    kernels = {}
    for i, nm in enumerate(names[:5]):
        a = bytes_[i] / (avg[i] * 1e-3) / 1e9
        kernels[nm] = {"bound": "hbm", "achieved": a, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": a / HBM_PEAK_GBS,
                       "traffic": measured_traffic(nm, args.config, n), "ms": float(avg[i]), "bytes": bytes_[i]}
    visits = float(n1) * cfg.n_trees * cfg.tree_depth
    kernels["sf_fast_infer_subset"].update(node_visits=visits, visits_per_s=visits / (avg[3] * 1e-3))
    tf = mlp_flops(cfg, n2) / (avg[5] * 1e-3) / 1e12
    kernels["sf_slow_infer"] = {"bound": "mfma", "achieved": tf, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                                "frac": tf / MFMA_BF16_PEAK_TFLOPS, "traffic": measured_traffic("sf_slow_infer", args.config, n),
                                "ms": float(avg[5]), "flops": mlp_flops(cfg, n2)}
    dominant = names[int(np.argmax(avg))]
    roof = {k: kernels[dominant][k] for k in ("bound", "achieved", "peak", "unit", "frac", "traffic")}
    roof["kernel"] = dominant
    out = {
        "metric": "flows/sec end-to-end (tree + gated forest + gated slow)",
        "value": n * args.steps / (t1 - t0), "unit": "flows/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": (t1 - t0) * 1e3 / args.steps, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None,
        "dtype": "f32 features, integer counts and votes, %s MLP" % cfg.mlp_dtype, "data": "synthetic",
        "config": {"workload": "%s: %d flows, %d packets, F=%d, tree depth %d theta0=%.2f, T=%d depth %d C=%d vmin=%d, "
                               "MLP %s %s" % (cfg.name, n, pk.n_pkts, F, cfg.tree0_depth, cfg.theta0, cfg.n_trees,
                                              cfg.tree_depth, C, cfg.vmin, cfg.mlp_dtype, "x".join(map(str, cfg.mlp_dims))),
                   "to_forest_fraction": n1 / n, "to_mlp_fraction": n2 / n},
        "roofline": roof, "kernels": kernels,
    }
    if not args.no_cpu_baseline:
        import oracle
        threads = oracle.default_threads()
        sample = min(n, 1 << 20)
        spk = synth.make_packets(cfg, n_flows=sample)
        t0 = time.perf_counter()
        o = oracle.classify3(spk, cfg.depths, tree, cfg.theta0, forest, cfg.vmin, mlp, n_threads=threads)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": sample / dt, "unit": "flows/s", "cores": threads, "kind": "oracle",
                               "sample": "first %d flows, all three tiers, %.1f s wall, %.1f%% to the forest, %.1f%% to "
                                         "the MLP" % (sample, dt, 100.0 * o["esc1"].size / sample,
                                                      100.0 * o["esc2"].size / sample)}
    print(json.dumps(out))


def join_bench(args):
    """--join: the queue join in front of the slow model at config 2's rates: per step 179,427 flows are handed
    on (queue 3) and as many late-feature records arrive (queue 2); 70 % of a flow's two records arrive in the
    same step, 20 % one step apart, 10 % never (and are discarded after the timeout)."""
    import torch
    import paper_2402_03694_amd as sf
    dev = "cuda:0"
    per_step, cap_log2, timeout = 179427, 20, 3
    steps = args.steps + args.warmup
    rng = np.random.default_rng(7)
    n = per_step * steps
    ids = rng.permutation(np.arange(1, n + 1, dtype=np.uint64) * np.uint64(0x9E3779B97F4A7C15))   # distinct, well spread
    t3 = np.repeat(np.arange(steps), per_step)
    u = rng.random(n)
    t2 = np.where(u < 0.7, t3, np.where(u < 0.8, t3 + 1, np.where(u < 0.9, t3 - 1, -1)))
    t2 = np.where((t2 < 0) | (t2 >= steps), -1, t2)
    ctx = sf.ServeFlow(sf.sf_join_workspace_bytes(cap_log2))
    table = sf.DeviceJoinTable(cap_log2, dev)
    t64 = lambda a: torch.from_numpy(np.ascontiguousarray(a, np.uint64).view(np.int64)).to(dev)
    t32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, np.uint32).view(np.int32)).to(dev)
    batches = []
    for s_ in range(steps):
        a, b = np.flatnonzero(t3 == s_), np.flatnonzero(t2 == s_)
        batches.append((t64(ids[a]), t32(a % (1 << 20)), t64(ids[b]), t32(b % (1 << 20)), a.size + b.size))
    p3 = torch.empty(2 * per_step, dtype=torch.int32, device=dev)
    p2 = torch.empty(2 * per_step, dtype=torch.int32, device=dev)
    k = torch.zeros(1, dtype=torch.int32, device=dev)
    stats = torch.zeros(4, dtype=torch.int32, device=dev)
    for s_ in range(args.warmup):
        b = batches[s_]
        ctx.sf_join_step(table, s_, timeout, b[0], b[1], b[2], b[3], p3, p2, k, stats)
    torch.cuda.synchronize()
    records = 0
    t0 = time.perf_counter()
    for s_ in range(args.warmup, steps):
        b = batches[s_]
        ctx.sf_join_step(table, s_, timeout, b[0], b[1], b[2], b[3], p3, p2, k, stats)
        records += b[4]
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms = (t1 - t0) * 1e3 / args.steps
    # per step the method must read every arrival (12 B) and write the pairs (8 B each); the tables are state
    pairs_last = int(k.cpu().numpy().view(np.uint32)[0])
    alg = 12.0 * records / args.steps + 8.0 * pairs_last
    table_bytes = 3.0 * sf.sf_join_table_bytes(cap_log2)        # scan, clear, plus the survivors' round trip (bound)
    out = {"metric": "records/sec through the queue join", "value": records / (t1 - t0), "unit": "records/s", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "u64 keys, u32 values", "data": "synthetic",
           "config": {"workload": "queue join: %d + ~%d arrivals per step, 2^%d slots per side, timeout %d steps"
                                  % (per_step, per_step * 9 // 10, cap_log2, timeout), "pairs_last_step": pairs_last},
           "roofline": {"bound": "hbm", "achieved": alg / (ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": alg / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "traffic": None, "kernel": "sf_join_step",
                        "table_sweep_bytes": table_bytes}}
    if not args.no_cpu_baseline:
        import oracle
        j = oracle.FlowJoin()
        sample_steps = min(steps, 4)
        c0 = time.perf_counter()
        done = 0
        for s_ in range(sample_steps):
            a, b = np.flatnonzero(t3 == s_), np.flatnonzero(t2 == s_)
            j.step(s_, timeout, ids[a], a, ids[b], b)
            done += a.size + b.size
        dt = time.perf_counter() - c0
        out["cpu_baseline"] = {"value": done / dt, "unit": "records/s", "cores": 1, "kind": "oracle",
                               "sample": "first %d steps of the same stream, %.1f s wall" % (sample_steps, dt)}
    print(json.dumps(out))


class TwoTier:
    """Device state of one two-tier workload: context, models laid out once, output buffers."""

    def __init__(self, cfg, n, dev="cuda:0"):
        import torch
        import synth
        import paper_2402_03694_amd as sf
        self.cfg, self.n, self.dev, self.sf = cfg, n, dev, sf
        F = cfg.n_features
        h1, h2 = cfg.mlp_dims[1], cfg.mlp_dims[2]
        self.pk = synth.make_packets(cfg, n_flows=n)
        self.ctx = sf.ServeFlow(sf.sf_workspace_bytes(n, cfg.n_trees, cfg.tree_depth, cfg.mlp_dims[0], h1, h2))
        self.d_pk = sf.packets_to_device(self.pk, dev)
        self.feat = torch.empty((n, F), dtype=torch.float32, device=dev)
        self.pred = torch.empty(n, dtype=torch.int16, device=dev)
        self.top = torch.empty(n, dtype=torch.int16, device=dev)
        self.esc_idx = torch.empty(n, dtype=torch.int32, device=dev)
        self.esc_count = torch.zeros(1, dtype=torch.int32, device=dev)
        self.labels = torch.empty(n, dtype=torch.int16, device=dev)
        ctx = self.ctx
        # models: thresholds and standardisation constants come from the first calib_flows flows' features
        ctx.sf_featurize(self.d_pk, cfg.depths, self.feat)
        torch.cuda.synchronize()
        calib = self.feat[: cfg.calib_flows].cpu().numpy()
        self.gbdt = cfg.fast_kind == "gbdt"
        self.d_mlp = sf.mlp_to_device(synth.make_mlp(cfg, None if cfg.raw_pkts else calib), dev)
        ctx.sf_mlp_order(self.d_mlp)            # the models are laid out for the kernels once, not per batch
        ctx.sf_validate_packets(self.d_pk)
        if self.gbdt:
            self.d_model = sf.gbdt_to_device(synth.make_gbdt(cfg, calib), dev)
            ctx.sf_gbdt_pack(self.d_model)
            self.kind = sf.SF_SCORE_ENTROPY if cfg.score == "entropy" else sf.SF_SCORE_LC
            self.score = torch.empty(n, dtype=torch.float32, device=dev)
        else:
            self.d_model = sf.forest_to_device(synth.make_forest(cfg, calib), dev)
            ctx.sf_validate_forest(self.d_model)
            ctx.sf_forest_pack(self.d_model)

    def fast(self, d_pk=None):
        """Steps 1-3 once, outside any timed region (for calibrating the gate)."""
        import torch
        self.ctx.sf_featurize(d_pk or self.d_pk, self.cfg.depths, self.feat)
        if self.gbdt:
            self.ctx.sf_gbdt_infer(self.feat, self.d_model, self.kind, self.pred, self.score)
        else:
            self.ctx.sf_fast_infer(self.feat, self.d_model, self.pred, self.top)
        torch.cuda.synchronize()

    fused = False   # steps 1-3 through sf_featurize_fast_infer (one kernel) instead of two calls

    def step(self, vmin, ev=None, d_pk=None):
        """The calls of one pass over one device-resident batch; ev: five events recorded around them
        (features | fast model | gate | slow model; in the fused form the first interval is empty)."""
        cfg, ctx = self.cfg, self.ctx
        d_pk = d_pk or self.d_pk
        n = d_pk.n_flows
        if ev:
            ev[0].record()
        if not self.fused:
            ctx.sf_featurize(d_pk, cfg.depths, self.feat)
        if ev:
            ev[1].record()
        if self.fused:
            ctx.sf_featurize_fast_infer(d_pk, cfg.depths, self.d_model, vmin, None if cfg.raw_pkts else self.feat, self.pred,
                                        self.top, labels=self.labels)    # labels start as the fast prediction
        elif self.gbdt:
            ctx.sf_gbdt_infer(self.feat, self.d_model, self.kind, self.pred, self.score, n_flows=n)
        else:
            ctx.sf_fast_infer(self.feat, self.d_model, self.pred, self.top, n_flows=n)
        if ev:
            ev[2].record()
        if self.gbdt:
            ctx.sf_route_score(self.score, vmin, self.esc_idx, self.esc_count, n_flows=n)
        else:
            ctx.sf_route(self.top, self.pred, vmin, self.esc_idx, self.esc_count, n_flows=n)
        if ev:
            ev[3].record()
        pred = None if self.fused else self.pred
        if cfg.raw_pkts:
            ctx.sf_slow_infer(self.d_mlp, self.esc_idx, self.esc_count, self.labels, raw_src=d_pk, raw_pkts=cfg.raw_pkts,
                              raw_bits=cfg.raw_bits, esc_cap=n, pred=pred)
        else:
            ctx.sf_slow_infer(self.d_mlp, self.esc_idx, self.esc_count, self.labels, feat=self.feat, esc_cap=n, pred=pred)
        if ev:
            ev[4].record()

    def calibrate(self, args):
        """The gate's threshold(s) for this run, outside the timed region.  Returns (vmin, how, reached fraction).
        Target-portion rule of Section 3.2: the library histograms the integer score on the device and picks the
        threshold whose escalated fraction is nearest the target.  Per-class thresholds: Algorithm 2 on the
        device's per-class histogram against synthetic validation labels (drawn by the workload generator from
        the fast model's own outputs)."""
        import torch
        import synth
        cfg, ctx, sf, n = self.cfg, self.ctx, self.sf, self.n
        self.fast()
        target = args.target if args.target >= 0 else (cfg.target_fracs[len(cfg.target_fracs) // 2] if cfg.target_fracs else None)
        if self.gbdt:
            # boosted form: Algorithm 1's quantile rule on the real-valued score, on the device
            return ctx.sf_score_quantiles(self.score, [1.0 - target])[0], "Algorithm 1 quantile on the score", target
        hist = ctx.sf_score_histogram(self.top, cfg.n_trees)
        self.hist = hist
        if args.gate == "per-class" and target is not None:
            truth = synth.make_truth(cfg, self.pred.cpu().numpy().view(np.uint16), self.top.cpu().numpy().view(np.uint16))
            d_truth = torch.from_numpy(truth.view(np.int16)).to(self.dev)
            ch = ctx.sf_class_score_histogram(self.top, self.pred, d_truth, cfg.n_trees, cfg.n_classes)
            vm, reached = sf.sf_per_class_thresholds(ch, cfg.n_trees, cfg.n_classes, target)
            return vm, "per-class thresholds (Algorithm 2), target %.3f" % target, reached
        if args.target >= 0 or (cfg.vmin is None and cfg.theta is None):
            vmin, reached = sf.sf_vmin_for_target(hist, cfg.n_trees, target)
            return vmin, "universal threshold nearest the target %.3f" % target, reached
        vmin = cfg.vmin if cfg.vmin is not None else sf.sf_vmin_from_theta(cfg.theta, cfg.n_trees)
        return vmin, "universal threshold of the workload", sum(hist[:vmin]) / float(n)


def timed_steps(tt, vmin, steps, warmup, batches=None):
    """W warm-ups, then K timed steps bracketed by synchronisation; events on the kernels' stream around each call.
    batches: optional list of device packet batches, step s runs batch s mod len.  Returns (seconds, [steps][4] ms)."""
    import torch
    pick = (lambda s: batches[s % len(batches)]) if batches else (lambda s: None)
    for s in range(warmup):
        tt.step(vmin, d_pk=pick(s))
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(steps):
        tt.step(vmin, events[s], d_pk=pick(s))
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    call_ms = np.array([[ev[i].elapsed_time(ev[i + 1]) for i in range(4)] for ev in events])
    return t1 - t0, call_ms


def kernel_report(tt, cfg_id, n, n_pkts, n_esc, avg, probe):
    """Per-call rooflines from the average call durations avg[4] (ms)."""
    cfg = tt.cfg
    k1b, k2b, k3b = algorithmic_bytes(cfg, n, n_pkts, n_esc / max(n, 1))
    if tt.fused:
        # one kernel for steps 1-3: packet records and offsets in, pred / top_votes out, and the feature rows of
        # the escalated flows only (none when the slow model reads header bits)
        fb = 7 * n_pkts + 4 * (n + 1) + 4 * n + (0 if cfg.raw_pkts else 4 * cfg.n_features * n_esc)
        visits = float(n) * cfg.n_trees * cfg.tree_depth
        a = fb / (avg[1] * 1e-3) / 1e9
        fk = {"bound": "hbm", "achieved": a, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": a / HBM_PEAK_GBS,
              "traffic": measured_traffic("sf_featurize_fast_infer", cfg_id, n), "ms": float(avg[1]), "bytes": fb,
              "node_visits": visits, "visits_per_s": visits / (avg[1] * 1e-3),
              "note": "features, forest walk and score in one kernel: bound by gathers and vector arithmetic, not by HBM"}
        if probe:
            fk.update(gather_probe=probe, gather_bound_visits_per_s=probe["bound_visits_per_s"],
                      gather_frac=fk["visits_per_s"] / probe["bound_visits_per_s"])
        a3 = k3b / (avg[2] * 1e-3) / 1e9
        tf = mlp_flops(cfg, n_esc) / (avg[3] * 1e-3) / 1e12
        kernels = {"sf_featurize_fast_infer": fk,
                   "sf_route": {"bound": "hbm", "achieved": a3, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": a3 / HBM_PEAK_GBS,
                                "traffic": measured_traffic("sf_route", cfg_id, n), "ms": float(avg[2]), "bytes": k3b},
                   "sf_slow_infer": {"bound": "mfma", "achieved": tf, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                                     "frac": tf / MFMA_BF16_PEAK_TFLOPS, "traffic": measured_traffic("sf_slow_infer", cfg_id, n),
                                     "ms": float(avg[3]), "flops": mlp_flops(cfg, n_esc)}}
        dominant = ["sf_featurize_fast_infer", "sf_featurize_fast_infer", "sf_route", "sf_slow_infer"][int(np.argmax(avg))]
        roof = {k: kernels[dominant][k] for k in ("bound", "achieved", "peak", "unit", "frac", "traffic")}
        roof["kernel"] = dominant
        for k in ("visits_per_s", "gather_bound_visits_per_s", "gather_frac"):   # see below
            if k in kernels[dominant]:
                roof[k] = kernels[dominant][k]
        return roof, kernels
    flops = mlp_flops(cfg, n_esc)
    visits = float(n) * cfg.n_trees * cfg.tree_depth

    def hbm(call, bytes_, ms):
        a = bytes_ / (ms * 1e-3) / 1e9
        return {"bound": "hbm", "achieved": a, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": a / HBM_PEAK_GBS,
                "traffic": measured_traffic(call, cfg_id, n), "ms": float(ms), "bytes": bytes_}

    kernels = {"sf_featurize": hbm("sf_featurize", k1b, avg[0]),
               "sf_fast_infer": dict(hbm("sf_fast_infer", k2b, avg[1]), node_visits=visits,
                                     visits_per_s=visits / (avg[1] * 1e-3)),
               "sf_route": hbm("sf_route", k3b, avg[2])}
    if probe:
        kernels["sf_fast_infer"].update(gather_probe=probe, gather_bound_visits_per_s=probe["bound_visits_per_s"],
                                        gather_frac=visits / (avg[1] * 1e-3) / probe["bound_visits_per_s"])
    tf = flops / (avg[3] * 1e-3) / 1e12
    bf16 = cfg.mlp_dtype == "bf16"
    peak = MFMA_BF16_PEAK_TFLOPS if bf16 else F32_VECTOR_PEAK_TFLOPS
    kernels["sf_slow_infer"] = {"bound": "mfma" if bf16 else "alu", "achieved": tf, "peak": peak, "unit": "TFLOP/s",
                                "frac": tf / peak, "traffic": measured_traffic("sf_slow_infer", cfg_id, n) if bf16 else None,
                                "ms": float(avg[3]), "flops": flops}
    if tt.gbdt:   # the boosted workload runs the same two steps through its own entry points
        kernels = {{"sf_fast_infer": "sf_gbdt_infer", "sf_route": "sf_route_score"}.get(k, k): v for k, v in kernels.items()}
    names = list(kernels)
    dominant = names[int(np.argmax(avg))]
    roof = {k: kernels[dominant][k] for k in ("bound", "achieved", "peak", "unit", "frac", "traffic")}
    roof["kernel"] = dominant
    # a tree walk is bound by its gathers, not by HBM: its rate against the all-from-shared-memory gather bound
    # (from the probe of this same run) goes beside the HBM fraction
    for k in ("visits_per_s", "gather_bound_visits_per_s", "gather_frac"):
        if k in kernels[dominant]:
            roof[k] = kernels[dominant][k]
    return roof, kernels


def result_line(tt, args, cfg_id, vmin, how, n, n_pkts, n_esc, steps, wall, call_ms, probe, extra_cfg=None):
    cfg = tt.cfg
    avg = call_ms.mean(axis=0)
    roof, kernels = kernel_report(tt, cfg_id, n, n_pkts, n_esc, avg, probe)
    per_step = call_ms.sum(axis=1)
    vtxt = ("%.6g" % vmin) if tt.gbdt else (str(vmin) if isinstance(vmin, int) else "[" + ",".join(map(str, vmin)) + "]")
    conf = {"workload": "%s: %d flows, %d packets, F=%d, T=%d depth %d C=%d, vmin=%s, MLP %s %s"
                        % (cfg.name, n, n_pkts, cfg.n_features, cfg.n_trees, cfg.tree_depth, cfg.n_classes, vtxt,
                           cfg.mlp_dtype, "x".join(map(str, cfg.mlp_dims))),
            "escalated_fraction": n_esc / max(n, 1), "gate": how,
            "fast_model": ("boosted trees, %s score" % cfg.score) if tt.gbdt else "hard-voting forest"}
    if extra_cfg:
        conf.update(extra_cfg)
    return {
        "metric": "flows/sec end-to-end (fast+gated slow)",
        "value": n * steps / wall, "unit": "flows/s",
        "n_gpus": 1, "steps": steps, "warmup": args.warmup,
        "ms_per_step": wall * 1e3 / steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32 features, integer votes, %s MLP" % cfg.mlp_dtype,
        "data": "synthetic",
        "config": conf,
        "roofline": roof,
        "kernels": kernels,
        "fast_ms": float(avg[0] + avg[1] + avg[2]), "slow_ms": float(avg[3]),
        "p50_ms": float(np.median(per_step)), "p99_ms": float(np.percentile(per_step, 99)),
    }


def stream_bench(args, cfg):
    """--config 4: the streaming workload as stated: 200 distinct consecutive batches of 65,536 ragged flows through
    one context and one model.  First figure: every batch already resident in HBM (the metric's definition).
    Second figure ("with_h2d"): each batch's packet arrays start in pinned host memory and are copied to the
    device on the same stream in front of its four calls."""
    import torch
    import synth
    sf = __import__("paper_2402_03694_amd")
    dev = "cuda:0"
    n = args.flows or cfg.n_flows
    n_batches = min(args.batches or cfg.n_batches, max(args.steps, 1))
    tt = TwoTier(cfg, n, dev)
    vmin, how, _ = tt.calibrate(args)
    host = [tt.pk] + [synth.make_packets(cfg, batch=b, n_flows=n) for b in range(1, n_batches)]
    resident = [tt.d_pk] + [sf.packets_to_device(p, dev) for p in host[1:]]
    probe = gather_probe(tt.ctx, dev)
    wall, call_ms = timed_steps(tt, vmin, args.steps, args.warmup, resident)
    n_pkts = int(np.mean([p.n_pkts for p in host]))
    esc = []
    for b in resident[: min(8, n_batches)]:        # escalated share over the first batches (outside the timed region)
        tt.step(vmin, d_pk=b)
        torch.cuda.synchronize()
        esc.append(int(tt.esc_count.cpu().numpy().view(np.uint32)[0]))
    n_esc = int(np.mean(esc))
    out = result_line(tt, args, args.config, vmin, how, n, n_pkts, n_esc, args.steps, wall, call_ms, probe,
                      {"distinct_batches": n_batches, "packets_per_batch_mean": n_pkts})
    out["sustained_flows_per_s"] = out["value"]

    # the same stream fed from pinned host memory
    cap = max(p.n_pkts for p in host)
    pin = lambda a: torch.from_numpy(a).pin_memory()
    pinned = [(pin(p.flow_off.view(np.int32)), pin(p.pkt_size.view(np.int16)), pin(p.pkt_iat), pin(p.pkt_dir), p.n_pkts)
              for p in host]
    s_off = torch.empty(n + 1, dtype=torch.int32, device=dev)
    s_size = torch.empty(cap, dtype=torch.int16, device=dev)
    s_iat = torch.empty(cap, dtype=torch.float32, device=dev)
    s_dir = torch.empty(cap, dtype=torch.uint8, device=dev)

    def fed_step(b, ev=None):
        off, size, iat, dr, m = pinned[b % n_batches]
        if ev:
            ev[0].record()
        s_off.copy_(off, non_blocking=True)
        s_size[:m].copy_(size, non_blocking=True)
        s_iat[:m].copy_(iat, non_blocking=True)
        s_dir[:m].copy_(dr, non_blocking=True)
        tt.step(vmin, d_pk=sf.DevicePackets(s_off, s_size[:m], s_iat[:m], s_dir[:m]))
        if ev:
            ev[1].record()

    for b in range(args.warmup):
        fed_step(b)
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for b in range(args.steps):
        fed_step(b, events[b])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    lat = np.array([ev[0].elapsed_time(ev[1]) for ev in events])
    copied = float(np.mean([4 * (n + 1) + 7 * p[4] for p in pinned]))
    out["with_h2d"] = {"value": n * args.steps / (t1 - t0), "unit": "flows/s", "ms_per_batch": (t1 - t0) * 1e3 / args.steps,
                       "p50_ms": float(np.median(lat)), "p99_ms": float(np.percentile(lat, 99)),
                       "bytes_copied_per_batch": copied,
                       "note": "packet arrays of every batch copied from pinned host memory on the kernels' stream"}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, n, vmin, n_esc / n)
    print(json.dumps(out))


def sweep_bench(args, cfg):
    """--config 5: the assigned-portion study: one line per target portion (5 %, 25 %, 50 % of the flows), each with
    the time split between the fast path (featurize, trees, gate) and the slow model."""
    import torch
    dev = "cuda:0"
    n = args.flows or cfg.n_flows
    tt = TwoTier(cfg, n, dev)
    probe = gather_probe(tt.ctx, dev)
    targets = [args.target] if args.target >= 0 else list(cfg.target_fracs)
    for i, target in enumerate(targets):
        args.target = target
        vmin, how, _ = tt.calibrate(args)
        wall, call_ms = timed_steps(tt, vmin, args.steps, args.warmup)
        n_esc = int(tt.esc_count.cpu().numpy().view(np.uint32)[0])
        out = result_line(tt, args, args.config, vmin, how, n, tt.pk.n_pkts, n_esc, args.steps, wall, call_ms, probe,
                          {"target_fraction": target})
        if abs(target - 0.25) > 1e-9:
            # the counter runs behind the traffic table were taken at the middle target: what depends on the
            # escalated portion is not known for the others
            for k in ("sf_route", "sf_slow_infer"):
                out["kernels"][k]["traffic"] = None
            if out["roofline"]["kernel"] in ("sf_route", "sf_slow_infer"):
                out["roofline"]["traffic"] = None
        if not args.no_cpu_baseline and i == len(targets) // 2:
            out["cpu_baseline"] = cpu_baseline(cfg, n, vmin, n_esc / n)
        print(json.dumps(out), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="timed steps (default 20; 200 for the streaming workload)")
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=2, help="workload 1..7 (2 = the 1M-flow headline workload, 4 = 200 streaming "
                    "batches, 5 = one line per target portion, 6 = the three-tier cascade, 7 = boosted trees)")
    ap.add_argument("--flows", type=int, default=0, help="override the flow count (for quick runs)")
    ap.add_argument("--batches", type=int, default=0, help="streaming workload: distinct batches (default: the workload's 200)")
    ap.add_argument("--target", type=float, default=-1.0, help="override the escalated-fraction target")
    ap.add_argument("--gate", choices=["auto", "universal", "per-class"], default="auto",
                    help="how the gate's threshold is chosen where the workload names a target portion: one threshold "
                         "for all classes, or one per predicted class (Algorithm 2); auto = per-class for the headline "
                         "workload, universal elsewhere")
    ap.add_argument("--calls", choices=["auto", "fused", "separate"], default="auto",
                    help="steps 1-3 as one kernel (sf_featurize_fast_infer) or as sf_featurize + sf_fast_infer; auto = fused "
                         "for workloads 2 and 3 (whose shapes the fused kernel covers), for workload 2 with the separate calls timed "
                         "beside it")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="time the main step only (no separate-calls leg, no universal-gate leg): for profiler runs")
    ap.add_argument("--join", action="store_true", help="time the queue join in front of the slow model instead")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain 256 MiB device copy (a known-size reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on one GPU; --gpus %d is not supported (across devices the flows would be "
              "sharded and the models replicated, with no exchange on the hot path)" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    import synth
    from paper_2402_03694_amd import build as hip_build
    if hip_build.is_stale():
        hip_build.build(force=True)
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"

    cfg = synth.get_config(args.config)
    if not args.steps:
        args.steps = cfg.n_batches if cfg.n_batches > 1 else 20
    if args.gate == "auto":
        args.gate = "per-class" if args.config == 2 else "universal"
    if args.copy_probe:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)              # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst
    if args.join:
        return join_bench(args)
    if cfg.tree0_depth:
        return three_tier(args, cfg)
    if cfg.n_batches > 1:
        return stream_bench(args, cfg)
    if len(cfg.target_fracs) > 1:
        return sweep_bench(args, cfg)
    n = args.flows or cfg.n_flows
    tt = TwoTier(cfg, n, dev)
    vmin, how, _ = tt.calibrate(args)
    want_fused = args.calls == "fused" or (args.calls == "auto" and args.config in (2, 3))
    if want_fused:
        # the fused kernel leaves the rows of the flows that stay with the fast model untouched: check that it ran
        tt.fused = True
        tt.feat.fill_(float("nan"))
        tt.step(vmin)
        torch.cuda.synchronize()
        rows_written = int((~torch.isnan(tt.feat[:, 0])).sum().item())
        n_esc0 = int(tt.esc_count.cpu().numpy().view(np.uint32)[0])
        if cfg.raw_pkts == 0 and rows_written != n_esc0:
            tt.fused = False        # this shape ran the separate kernels inside the library
    probe = gather_probe(tt.ctx, dev)
    wall, call_ms = timed_steps(tt, vmin, args.steps, args.warmup)
    n_esc = int(tt.esc_count.cpu().numpy().view(np.uint32)[0])
    out = result_line(tt, args, args.config, vmin, how, n, tt.pk.n_pkts, n_esc, args.steps, wall, call_ms, probe)
    out["measured_copy_GBps"] = copy_bandwidth(dev)
    out["config"]["calls"] = "sf_featurize_fast_infer + sf_route + sf_slow_infer" if tt.fused else \
                             "sf_featurize + sf_fast_infer + sf_route + sf_slow_infer"
    if tt.fused and not args.no_extras:
        # the same step through the four separate calls
        tt.fused = False
        s_wall, s_ms = timed_steps(tt, vmin, args.steps, args.warmup)
        _, s_kernels = kernel_report(tt, args.config, n, tt.pk.n_pkts, n_esc, s_ms.mean(axis=0), probe)
        for v in s_kernels.values():
            v.pop("gather_probe", None)
        out["separate_calls"] = {"value": n * args.steps / s_wall, "unit": "flows/s", "ms_per_step": s_wall * 1e3 / args.steps,
                                 "kernels": s_kernels}
        tt.fused = True
    if args.gate == "per-class" and not tt.gbdt and not args.no_extras:
        # the same workload behind one threshold for all classes: the integer score then reaches only a few portions
        u_vmin, reached = tt.sf.sf_vmin_for_target(tt.hist, cfg.n_trees, args.target if args.target >= 0 else cfg.target_fracs[0])
        u_wall, u_ms = timed_steps(tt, u_vmin, args.steps, args.warmup)
        u_esc = int(tt.esc_count.cpu().numpy().view(np.uint32)[0])
        out["universal_gate"] = {"vmin": u_vmin, "escalated_fraction": u_esc / n, "value": n * args.steps / u_wall,
                                 "unit": "flows/s", "ms_per_step": u_wall * 1e3 / args.steps,
                                 "call_ms": [float(v) for v in u_ms.mean(axis=0)]}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, n, vmin, n_esc / n)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
