"""Pins for the oracle's slow model and the end-to-end label rule (not gpu): a network worked
by hand, numpy's float64 matmul, the identity / one-hot / dead-ReLU special cases, the input
map against exact rational arithmetic, and the rule that the slow label replaces the fast one
on escalated flows only."""
import os
from fractions import Fraction
from types import SimpleNamespace

import numpy as np
import pytest

import oracle
import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "mlp_handworked.txt")


def _mlp(w1, b1, w2, b2, w3, b3, dtype="f32", mu=None, inv_sigma=None, clamp=8.0):
    w1, w2, w3 = (np.asarray(w, np.float32) for w in (w1, w2, w3))
    return SimpleNamespace(dims=(w1.shape[1], w1.shape[0], w2.shape[0], w3.shape[0]), dtype=dtype,
                           w1=w1, b1=np.asarray(b1, np.float32), w2=w2, b2=np.asarray(b2, np.float32),
                           w3=w3, b3=np.asarray(b3, np.float32), mu=mu, inv_sigma=inv_sigma, clamp=clamp)


def test_handworked_network():
    p, xs, want_logits, want_labels = {}, [], [], []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, rest = line.split(None, 1)
        if key == "x":
            a, b = rest.split("->")
            lg, lab = b.split("|")
            xs.append([float(v) for v in a.split()])
            want_logits.append([float(v) for v in lg.split()])
            want_labels.append(int(lab))
        else:
            p[key] = [float(v) for v in rest.split()]
    m = _mlp(np.reshape(p["w1"], (2, 2)), p["b1"], np.reshape(p["w2"], (2, 2)), p["b2"],
             np.reshape(p["w3"], (3, 2)), p["b3"])
    x = np.array(xs, np.float32)
    n = x.shape[0]
    logits, labels = oracle.slow_infer(np.arange(n, dtype=np.uint32), m, n, feat=x)
    assert logits.tolist() == want_logits
    assert labels.tolist() == want_labels
    # same network declared bf16: all values are bf16-representable, nothing changes
    m.dtype = "bf16"
    logits2, labels2 = oracle.slow_infer(np.arange(n, dtype=np.uint32), m, n, feat=x)
    assert np.array_equal(logits, logits2) and np.array_equal(labels, labels2)


def _numpy_chain(z, m):
    h1 = np.maximum(z @ m.w1.astype(np.float64).T + m.b1.astype(np.float64), 0.0)
    h2 = np.maximum(h1 @ m.w2.astype(np.float64).T + m.b2.astype(np.float64), 0.0)
    return h2 @ m.w3.astype(np.float64).T + m.b3.astype(np.float64)


@pytest.mark.parametrize("cfg_id", [1, 2])
def test_against_numpy_matmul(cfg_id):
    cfg = synth.get_config(cfg_id)
    n = 256
    pk = synth.make_packets(cfg, n_flows=n)
    feat, _ = oracle.featurize(pk.flow_off, pk.pkt_size, pk.pkt_iat, pk.pkt_dir, cfg.depths)
    m = synth.make_mlp(cfg, feat)
    esc = np.arange(0, n, 3, dtype=np.uint32)
    logits, labels = oracle.slow_infer(esc, m, n, feat=feat)
    # the input map in numpy binary32, one rounding per operation
    z = np.clip((feat[esc] - m.mu) * m.inv_sigma, np.float32(-8), np.float32(8)).astype(np.float32)
    if cfg.mlp_dtype == "bf16":
        z = synth.round_to_bf16(z)
    ref = _numpy_chain(z.astype(np.float64), m)
    np.testing.assert_allclose(logits, ref, rtol=0, atol=1e-6)       # both binary64; order differs
    assert np.array_equal(labels[esc], np.argmax(ref.astype(np.float32), axis=1))
    assert np.all(np.abs(ref) < 50)                                  # standardised inputs keep logits O(1)


def test_special_cases():
    rng = np.random.default_rng(11)
    n_in, h, C = 6, 6, 6
    eye = np.eye(6, dtype=np.float32)
    b = [rng.uniform(-0.1, 0.1, 6).astype(np.float32) for _ in range(3)]
    x = rng.uniform(0.5, 2.0, size=(5, 6)).astype(np.float32)        # positive: ReLU is transparent
    esc = np.arange(5, dtype=np.uint32)
    # zero weights: logits = b3 whatever the input
    z = np.zeros((6, 6), np.float32)
    lg, lab = oracle.slow_infer(esc, _mlp(z, b[0], z, b[1], z, b[2]), 5, feat=x)
    assert np.array_equal(lg, np.tile(b[2], (5, 1))) and np.all(lab == np.argmax(b[2]))
    # identity weights, zero biases: logits = x
    zb = np.zeros(6, np.float32)
    lg, lab = oracle.slow_infer(esc, _mlp(eye, zb, eye, zb, eye, zb), 5, feat=x)
    assert np.array_equal(lg, x) and np.array_equal(lab, np.argmax(x, axis=1))
    # a transposed weight operand would show here: one-hot input picks out a *column* of W1
    w1 = rng.uniform(0.1, 1.0, size=(6, 6)).astype(np.float32)
    onehot = np.zeros((6, 6), np.float32)
    onehot[np.arange(6), np.arange(6)] = 1.0
    lg, _ = oracle.slow_infer(np.arange(6, dtype=np.uint32), _mlp(w1, zb, eye, zb, eye, zb), 6, feat=onehot)
    assert np.array_equal(lg, w1.T)
    # all first-layer pre-activations negative: hidden zeros, logits = W3 relu(b2) + b3
    wneg = -np.abs(w1)
    b2 = np.array([0.5, -0.5, 0.25, -1, 2, 0], np.float32)
    w3 = rng.integers(-3, 4, size=(6, 6)).astype(np.float32)
    lg, _ = oracle.slow_infer(esc, _mlp(wneg, -np.ones(6, np.float32), eye, b2, w3, zb), 5, feat=x)
    want = w3.astype(np.float64) @ np.maximum(b2, 0).astype(np.float64)
    assert np.array_equal(lg, np.tile(want.astype(np.float32), (5, 1)))
    # ties in the arg-max go to the lowest class
    lg, lab = oracle.slow_infer(esc[:1], _mlp(z, zb, z, zb, z, np.array([1, 3, 3, 0, 3, 2], np.float32)),
                                1, feat=x[:1])
    assert lab[0] == 1


def test_input_map_exact():
    """z = clamp((x - mu) * inv_sigma, -c, c), every step rounded to binary32, then to bf16."""
    from exact import round_f32
    x = np.array([[1.0, 3.0, 100.0, -100.0, 0.1, 7.0]], np.float32)
    mu = np.array([0.5, 1.0, 0.0, 0.0, 0.3, 7.0], np.float32)
    isg = np.array([3.0, 0.1, 1.0, 1.0, 1.7, 5.0], np.float32)
    eye, zb = np.eye(6, dtype=np.float32), np.zeros(6, np.float32)
    want32, want16 = [], []
    for f in range(6):
        d = Fraction(float(x[0, f])) - Fraction(float(mu[f]))
        d32 = round_f32(abs(d)) * (1 if d >= 0 else -1) if d != 0 else np.float32(0)
        p = Fraction(float(d32)) * Fraction(float(isg[f]))
        p32 = round_f32(abs(p)) * (1 if p >= 0 else -1) if p != 0 else np.float32(0)
        p32 = np.float32(min(max(float(p32), -4.0), 4.0))
        want32.append(p32)
        want16.append(synth.round_to_bf16(np.array([p32]))[0])
    for dtype, want in (("f32", want32), ("bf16", want16)):
        m = _mlp(eye, zb, eye, zb, eye, zb, dtype=dtype, mu=mu, inv_sigma=isg, clamp=4.0)
        m.b1 = np.full(6, 10, np.float32)           # shift so ReLU passes negatives; remove below
        m.b3 = np.full(6, -10, np.float32)
        lg, _ = oracle.slow_infer(np.zeros(1, np.uint32), m, 1, feat=x)
        assert lg[0].tolist() == [float(v) for v in want]
    assert want32[2] == 4.0 and want32[3] == -4.0 and want32[5] == 0.0


def test_bf16_rounding_ties_to_even():
    eye, zb = np.eye(4, dtype=np.float32), np.zeros(4, np.float32)
    # 1 + 2^-8 is halfway between bf16 neighbours 1 and 1+2^-7: ties to even -> 1
    # 1 + 3*2^-8 is halfway between 1+2^-7 and 1+2^-6: -> 1+2^-6 (even significand)
    x = np.array([[1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, 1 + 2.0 ** -8 + 2.0 ** -20, 1 + 2.0 ** -9]], np.float32)
    m = _mlp(eye, zb, eye, zb, eye, zb, dtype="bf16")
    lg, _ = oracle.slow_infer(np.zeros(1, np.uint32), m, 1, feat=x)
    assert lg[0].tolist() == [1.0, 1 + 2.0 ** -6, 1 + 2.0 ** -7, 1.0]
    assert np.array_equal(synth.round_to_bf16(x)[0], lg[0])


def test_raw_bit_input_matches_feature_matrix():
    """Reading header bits straight from the packed words gives the same logits as running the
    network on the unpacked {0,1} feature matrix."""
    cfg = synth.get_config(3)
    n = 48
    pk = synth.make_packets(cfg, n_flows=n)
    _, raw = oracle.featurize(pk.flow_off, pk.pkt_size, pk.pkt_iat, pk.pkt_dir, cfg.depths,
                              pkt_hdr=pk.pkt_hdr, raw_pkts=10, raw_bits=480, want_raw=True)
    m = synth.make_mlp(cfg, None)
    esc = np.array([0, 5, 6, 40, 47], np.uint32)
    lg_a, lab_a = oracle.slow_infer(esc, m, n, flow_off=pk.flow_off, pkt_hdr=pk.pkt_hdr,
                                    raw_pkts=10, raw_bits=480)
    lg_b, lab_b = oracle.slow_infer(esc, m, n, feat=raw.astype(np.float32))
    assert np.array_equal(lg_a, lg_b) and np.array_equal(lab_a, lab_b)
    ref = _numpy_chain(raw[esc].astype(np.float64), m)
    np.testing.assert_allclose(lg_a, ref, rtol=0, atol=1e-5)


def test_end_to_end_label_rule():
    cfg = synth.get_config(1)
    n = 512
    pk = synth.make_packets(cfg, n_flows=n)
    feat, _ = oracle.featurize(pk.flow_off, pk.pkt_size, pk.pkt_iat, pk.pkt_dir, cfg.depths)
    forest, mlp = synth.make_forest(cfg, feat), synth.make_mlp(cfg, feat)
    out = oracle.classify(pk, cfg.depths, forest, 7, mlp)
    esc = out["esc_idx"]
    kept = np.setdiff1d(np.arange(n), esc)
    assert 0 < esc.size < n and esc.size + kept.size == n
    assert np.array_equal(out["labels"][kept], out["pred"][kept])
    assert np.array_equal(out["labels"][esc], np.argmax(out["logits"], axis=1))
    assert out["logits"].shape == (esc.size, 4)
    assert np.all(out["top_votes"][esc] < 7) and np.all(out["top_votes"][kept] >= 7)
    # the stated gate of the small workload: theta = 0.75 of 16 trees escalates nearly everything
    out12 = oracle.classify(pk, cfg.depths, forest, oracle.vmin_from_theta(cfg.theta, cfg.n_trees), mlp)
    assert out12["esc_idx"].size >= 0.99 * n
