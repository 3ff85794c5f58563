"""Pins for the oracle's queue join (not gpu)."""
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "join_handworked.txt")


def _kv(text, n):
    out = []
    for tok in text.split():
        parts = tok.replace("@", ":").split(":")
        assert len(parts) == n
        out.append(tuple(int(p) for p in parts))
    return out


def test_hand_worked_run():
    j = oracle.FlowJoin()
    steps = 0
    lines = [l.strip() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    i = 0
    while i < len(lines):
        head, res = lines[i].split("->")
        _, now, timeout = head.split("|")[0].split()
        q3, q2 = _kv(head.split("|")[1], 2), _kv(head.split("|")[2], 2)
        want_pairs, want_exp = _kv(res.split("|")[0], 3), int(res.split("|")[1].split()[1])
        pairs, expired = j.step(int(now), int(timeout), [k for k, _ in q3], [v for _, v in q3], [k for k, _ in q2],
                                [v for _, v in q2])
        assert pairs == want_pairs and expired == want_exp, lines[i]
        assert j.pending(3) == _kv(lines[i + 1][5:], 3), lines[i + 1]
        assert j.pending(2) == _kv(lines[i + 2][5:], 3), lines[i + 2]
        i += 3
        steps += 1
    assert steps == 6


def test_one_step_is_a_set_intersection():
    """with nothing waiting and no timeout in play, a step's matches are the IDs common to both batches"""
    rng = np.random.default_rng(0)
    ids = rng.choice(1 << 40, size=3000, replace=False).astype(np.uint64)
    a, b = ids[:2000], ids[1200:]
    j = oracle.FlowJoin()
    pairs, expired = j.step(1, 10, a, np.arange(a.size), b, np.arange(b.size) + 5000)
    common = np.intersect1d(a, b)
    assert expired == 0 and [p[0] for p in pairs] == common.tolist()
    pos_a = {int(k): i for i, k in enumerate(a)}
    pos_b = {int(k): i + 5000 for i, k in enumerate(b)}
    assert all(v3 == pos_a[k] and v2 == pos_b[k] for k, v3, v2 in pairs)
    assert [p[0] for p in j.pending(3)] == np.setdiff1d(a, b).tolist()
    assert [p[0] for p in j.pending(2)] == np.setdiff1d(b, a).tolist()


def test_every_flow_matches_once_and_only_within_the_timeout():
    """random arrival times on both sides: a flow is paired iff its two records arrive within `timeout` ticks of
    each other (checked from the arrival times alone), and then exactly once"""
    rng = np.random.default_rng(1)
    n, T, timeout = 4000, 60, 7
    ids = rng.choice(1 << 50, size=n, replace=False).astype(np.uint64)
    t3 = rng.integers(0, T, size=n)
    t2 = np.where(rng.random(n) < 0.15, -1, t3 + rng.integers(-12, 13, size=n))     # some never arrive
    t2 = np.where((t2 >= T) | (t2 < -1), -1, t2)
    j = oracle.FlowJoin()
    matched = {}
    total_expired = 0
    for now in range(T):
        a, b = np.flatnonzero(t3 == now), np.flatnonzero(t2 == now)
        pairs, expired = j.step(now, timeout, ids[a], a, ids[b], b)
        total_expired += expired
        for k, v3, v2 in pairs:
            assert k not in matched and ids[v3] == k and v3 == v2
            matched[k] = now
    want = {int(ids[i]) for i in range(n) if t2[i] >= 0 and abs(int(t3[i]) - int(t2[i])) <= timeout}
    assert set(matched) == want
    for i in range(n):
        if int(ids[i]) in matched:
            assert matched[int(ids[i])] == max(t3[i], t2[i])
    # what is still waiting at the end arrived within the last `timeout` ticks; everything else was discarded
    left = j.pending(3) + j.pending(2)
    assert all(T - 1 - st <= timeout for _, _, st in left)
    arrivals = n + int((t2 >= 0).sum())
    assert arrivals == 2 * len(matched) + total_expired + len(left)


def test_duplicates_are_rejected():
    j = oracle.FlowJoin()
    with pytest.raises(ValueError):
        j.step(0, 5, [3, 3], [0, 1], [], [])
    j = oracle.FlowJoin()
    j.step(0, 5, [3], [0], [], [])
    with pytest.raises(ValueError):
        j.step(1, 5, [3], [1], [], [])
