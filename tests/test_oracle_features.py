"""Pins for the oracle's feature step (not gpu): hand-derived values, numpy's statistics,
window/raggedness invariants and a brute-force bit loop for the raw header bits."""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
import synth
from exact import round_f32, sqrt_f32

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "features_handbuilt.txt")
U = Fraction(1, 1 << 12)


def _token(tok: str) -> np.float32:
    scale = Fraction(1)
    if tok.endswith("u"):
        tok, scale = tok[:-1], U
    if tok.startswith("S"):
        a, b = tok[1:].split("/")
        var = round_f32(Fraction(int(a), int(b)))
        val = Fraction(float(sqrt_f32(Fraction(float(var)))))
    else:
        val = Fraction(int(tok))
    out = np.float32(float(val * scale))
    assert Fraction(float(out)) == val * scale
    return out


def _load_golden():
    flows, cur = [], None
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, *rest = line.split()
        if key == "flow":
            cur = {"name": rest[0]}
            flows.append(cur)
        elif key == "expect":
            cur["expect"] = np.array([_token(t) for t in rest], dtype=np.float32)
        else:
            cur[key] = [int(x) for x in rest]
    return flows


@pytest.mark.parametrize("flow", _load_golden(), ids=lambda f: f["name"])
def test_handbuilt_flow(flow):
    n = len(flow["sizes"])
    off = np.array([0, n], np.uint32)
    iat = np.array([float(Fraction(k) * U) for k in flow["iats"]], np.float32)
    feat, _ = oracle.featurize(off, np.array(flow["sizes"], np.uint16), iat,
                               np.array(flow["dirs"], np.uint8), flow["depths"])
    exp = flow["expect"]
    assert feat.shape == (1, 32 * len(flow["depths"])) and exp.shape[0] == feat.shape[1]
    assert np.array_equal(feat[0].view(np.uint32), exp.view(np.uint32)), \
        list(zip(range(exp.shape[0]), feat[0], exp))


def _numpy_stats(x32):
    if x32.size == 0:
        return np.zeros(5)
    x = x32.astype(np.float64)
    return np.array([x.mean(), x.std(), x.min(), x.max(), np.median(x)])


@pytest.mark.parametrize("cfg_id,n", [(1, 300), (2, 200), (4, 400), (5, 100)])
def test_against_numpy(cfg_id, n):
    """numpy on float64 copies: min/max/median/counts/bytes/size-means are exact in binary32,
    so equal bit for bit; inter-arrival mean/std agree to a few ulp (different summation)."""
    cfg = synth.get_config(cfg_id)
    pk = synth.make_packets(cfg, n_flows=n)
    feat, _ = oracle.featurize(pk.flow_off, pk.pkt_size, pk.pkt_iat, pk.pkt_dir, cfg.depths)
    for i in range(n):
        o, e = int(pk.flow_off[i]), int(pk.flow_off[i + 1])
        for w, dep in enumerate(cfg.depths):
            m = min(e - o, dep)
            sz = pk.pkt_size[o:o + m].astype(np.float32)
            ia = pk.pkt_iat[o:o + m]
            dr = pk.pkt_dir[o:o + m]
            row = feat[i, 32 * w:32 * w + 32]
            assert row[30] == np.float32(pk.pkt_size[o:o + m].astype(np.int64).sum())
            assert row[31] == np.float32(m)
            for g in range(3):
                sel = np.ones(m, bool) if g == 2 else dr == g
                s_ref, i_ref = _numpy_stats(sz[sel]), _numpy_stats(ia[sel])
                got_s, got_i = row[10 * g:10 * g + 5], row[10 * g + 5:10 * g + 10]
                # exact ones
                assert got_s[2] == np.float32(s_ref[2]) and got_s[3] == np.float32(s_ref[3])
                assert got_s[4] == np.float32(s_ref[4])
                assert got_i[2] == np.float32(i_ref[2]) and got_i[3] == np.float32(i_ref[3])
                c = int(sel.sum())
                if c:
                    # size sum is an exact integer < 2^24, so the mean is one correctly rounded division
                    assert got_s[0] == np.float32(sz[sel].astype(np.float64).sum()) / np.float32(c)
                # median of an even count: (a+b)*0.5 in binary32; the double-precision mean of two
                # binary32 values rounds to the same value
                assert got_i[4] == np.float32(i_ref[4])
                np.testing.assert_allclose(got_s[1], s_ref[1], rtol=2e-6, atol=0)
                np.testing.assert_allclose(got_i[0], i_ref[0], rtol=1e-6, atol=0)
                np.testing.assert_allclose(got_i[1], i_ref[1], rtol=4e-6, atol=1e-12)


def test_empty_direction_group_is_zero():
    off = np.array([0, 3], np.uint32)
    feat, _ = oracle.featurize(off, np.array([50, 60, 70], np.uint16), np.array([1, 2, 3], np.float32),
                               np.array([0, 0, 0], np.uint8), [8])
    assert np.all(feat[0, 10:20] == 0)
    assert np.array_equal(feat[0, 0:10], feat[0, 20:30])


def test_window_prefix_consistency():
    """Window 0 of a two-window run equals a one-window run of the same depth, and windows at or
    beyond the flow length equal each other (apart from nothing: count and bytes agree too)."""
    cfg = synth.get_config(4)
    pk = synth.make_packets(cfg, n_flows=500)
    two, _ = oracle.featurize(pk.flow_off, pk.pkt_size, pk.pkt_iat, pk.pkt_dir, [8, 64])
    one, _ = oracle.featurize(pk.flow_off, pk.pkt_size, pk.pkt_iat, pk.pkt_dir, [8])
    assert np.array_equal(two[:, :32].view(np.uint32), one.view(np.uint32))
    lens = np.diff(pk.flow_off.astype(np.int64))
    short = lens <= 8
    assert short.any() and (~short).any()
    assert np.array_equal(two[short, :32].view(np.uint32), two[short, 32:].view(np.uint32))
    wide, _ = oracle.featurize(pk.flow_off, pk.pkt_size, pk.pkt_iat, pk.pkt_dir, [64, 200])
    assert np.array_equal(wide[:, :32].view(np.uint32), wide[:, 32:].view(np.uint32))
    assert np.array_equal(two[:, 32:].view(np.uint32), wide[:, :32].view(np.uint32))


def test_zero_length_flow_and_leading_dimension():
    off = np.array([0, 0, 2, 2], np.uint32)
    feat, _ = oracle.featurize(off, np.array([10, 20], np.uint16), np.array([0.5, 0.25], np.float32),
                               np.array([1, 0], np.uint8), [4], feat_ld=40)
    assert feat.shape == (3, 40)
    assert np.all(feat[0] == 0) and np.all(feat[2] == 0)
    assert feat[1, 31] == 2 and feat[1, 30] == 30 and np.all(feat[1, 32:] == 0)
    assert feat[1, 20] == 15 and feat[1, 21] == 5      # mean, std of 10,20


def test_rejects_bad_windows():
    off = np.array([0, 1], np.uint32)
    args = (off, np.array([1], np.uint16), np.array([1], np.float32), np.array([0], np.uint8))
    for bad in ([], [4, 4], [8, 4], [0]):
        with pytest.raises(ValueError):
            oracle.featurize(*args, bad)


def _bit_loop(words_row, n_bits):
    """Brute force: rebuild the header's bytes, then read bit b MSB-first."""
    by = []
    for w in words_row:
        by += [(int(w) >> (8 * k)) & 0xFF for k in range(4)]
    return [(by[b // 8] >> (7 - b % 8)) & 1 for b in range(n_bits)]


def test_raw_bits_bruteforce_and_popcount():
    cfg = synth.get_config(3)
    pk = synth.make_packets(cfg, n_flows=64)
    _, raw = oracle.featurize(pk.flow_off, pk.pkt_size, pk.pkt_iat, pk.pkt_dir, cfg.depths,
                              pkt_hdr=pk.pkt_hdr, raw_pkts=10, raw_bits=480, want_raw=True)
    assert raw.shape == (64, 4800) and set(np.unique(raw)) <= {0, 1}
    for i in (0, 17, 63):
        o = int(pk.flow_off[i])
        for j in (0, 9):
            assert list(raw[i, 480 * j:480 * j + 480]) == _bit_loop(pk.pkt_hdr[o + j], 480)
    pop_words = sum(bin(int(w)).count("1") for w in pk.pkt_hdr[:640].ravel())
    assert int(raw.sum()) == pop_words
    # one set bit: header byte 0 bit 7 (wire bit 0) lives in word 0 bit 7
    hdr = np.zeros((2, 15), np.uint32)
    hdr[0, 0] = 1 << 7
    hdr[1, 14] = 1 << 24          # byte 59, least significant bit -> wire bit 479
    off = np.array([0, 2], np.uint32)
    _, r = oracle.featurize(off, np.zeros(2, np.uint16), np.zeros(2, np.float32), np.zeros(2, np.uint8),
                            [2], pkt_hdr=hdr, raw_pkts=3, raw_bits=480, want_raw=True)
    assert np.flatnonzero(r[0]).tolist() == [0, 480 + 479]      # third packet absent -> zeros


def test_raw_bits_class_pattern_survives():
    cfg = synth.get_config(3)
    pk = synth.make_packets(cfg, n_flows=400)
    _, raw = oracle.featurize(pk.flow_off, pk.pkt_size, pk.pkt_iat, pk.pkt_dir, cfg.depths,
                              pkt_hdr=pk.pkt_hdr, raw_pkts=10, raw_bits=480, want_raw=True)
    first = raw[:, :480]
    for c in range(cfg.n_classes):
        rows = first[pk.hidden_class == c]
        const = np.all(rows == rows[0], axis=0)
        assert const.sum() >= 64          # the 64 planted positions (others vary)
