"""Pins for the CPU oracle (no GPU).

The oracle is checked against things other than itself: values worked by hand
(tests/golden), closed forms, invariants of the problem, special cases that
reduce to a max / a sum, and the exhaustive search of Section IV ("Naive
search") on tiny inputs.  The three routes inside the oracle (naive,
definition, sweep) are written independently of one another, so agreement
between them on thousands of random tiny cases, ties included, catches a
dropped term, a wrong sign or index or a transposed operand in any of them.
"""
import itertools
import json
import math
import os

import numpy as np
import pytest

from paper_2001_01347_amd import workloads

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "worked_examples.json")


def run(oracle, t, method="sweep"):
    b, it, w, rc, _ = oracle.zipline(np.asarray(t, dtype=np.int64), method=method)
    assert (rc == 0).all()
    return b, it, w


@pytest.mark.parametrize("method", ["sweep", "definition", "naive"])
def test_hand_worked_examples(oracle, method):
    cases = json.load(open(GOLDEN))["cases"]
    assert len(cases) >= 4
    for c in cases:
        b, it, w = run(oracle, c["t"], method)
        assert b[0] == c["barrier"], c["name"]
        assert w[0] == c["wait"], c["name"]
        assert list(it[0]) == c["iters"], c["name"]
        # the fixture is self-consistent: listed minimum and first-minimum rule
        assert min(c["waits"]) == c["wait"]
        assert c["candidates"][c["waits"].index(min(c["waits"]))] == c["barrier"]


def test_naive_definition_sweep_agree_on_tiny_random(oracle):
    rng = np.random.default_rng(20010134)
    n = 0
    for P in range(1, 6):
        for R in range(1, 7):
            if R ** P > 20000:
                continue
            for rep in range(60):
                t = workloads.random_small(rng, P, R, ties=(rep % 3 == 0))
                ref = run(oracle, t, "naive")
                for m in ("definition", "sweep"):
                    got = run(oracle, t, m)
                    for a, b in zip(ref, got):
                        assert np.array_equal(a, b), (P, R, rep, m, t)
                n += 1
    assert n > 1000


def test_definition_equals_sweep_on_medium_random(oracle):
    rng = np.random.default_rng(7)
    for P, R in [(8, 16), (16, 8), (3, 64), (32, 5)]:
        ts = np.stack([workloads.random_small(rng, P, R, 1, 50, ties=(i % 2 == 0))
                       for i in range(40)])
        a = oracle.zipline(ts, "definition")
        b = oracle.zipline(ts, "sweep")
        for x, y in zip(a[:3], b[:3]):
            assert np.array_equal(x, y)


def test_config1_bruteforce(oracle):
    # configuration 1: P = 4, R = 8 -> 4096 choices, exhaustive search feasible
    ts = workloads.make(1)
    assert ts.shape == (1, 4, 8)
    a = oracle.zipline(ts, "naive")
    b = oracle.zipline(ts, "sweep")
    for x, y in zip(a[:3], b[:3]):
        assert np.array_equal(x, y)


def _instances():
    rng = np.random.default_rng(99)
    out = [workloads.random_small(rng, P, R, 1, 1000, ties=False)
           for P, R in [(2, 3), (3, 5), (5, 9), (7, 4), (16, 32), (11, 17)]]
    out += [workloads.random_small(rng, 6, 10, 3, 7, ties=True) for _ in range(4)]
    out += [workloads.make(2, instances=[0, 1, 2])[i] for i in range(3)]
    return out


def test_invariants(oracle):
    rng = np.random.default_rng(5)
    for t in _instances():
        P, R = t.shape
        b, it, w = run(oracle, t)
        b, w, it = int(b[0]), int(w[0]), it[0]
        # wait >= 0 and no worse than classic BSP (one iteration each, Section I)
        first = t[:, 0]
        assert 0 <= w <= int((first.max() - first).sum())
        # the barrier is one of the timestamps and every worker has finished one iteration
        assert b in t and b >= first.max()
        assert ((1 <= it) & (it <= R)).all()
        # the three outputs describe the same stop: worker p stops at t[p][iters-1] <= barrier
        stop = t[np.arange(P), it - 1]
        assert (stop <= b).all()
        nxt = np.where(it < R, t[np.arange(P), np.minimum(it, R - 1)], np.iinfo(np.int64).max)
        assert (nxt > b).all()
        assert int((b - stop).sum()) == w
        # permuting workers permutes iters and changes nothing else
        perm = rng.permutation(P)
        b2, it2, w2 = run(oracle, t[perm])
        assert (int(b2[0]), int(w2[0])) == (b, w) and np.array_equal(it2[0], it[perm])
        # adding a constant shifts the barrier and leaves wait and iters unchanged
        for k in (12345, -777, 1_700_000_000_000_000):
            b3, it3, w3 = run(oracle, t + k)
            assert (int(b3[0]), int(w3[0])) == (b + k, w) and np.array_equal(it3[0], it)
        # scaling time by a positive integer scales barrier and wait
        b4, it4, w4 = run(oracle, t * 3)
        assert (int(b4[0]), int(w4[0])) == (3 * b, 3 * w) and np.array_equal(it4[0], it)
        # a shorter lookahead only removes candidates: the optimum cannot improve
        if R > 1:
            _, _, w5 = run(oracle, t[:, : R - 1])
            assert int(w5[0]) >= w


def test_closed_forms(oracle):
    # identical workers: everyone finishes together at the first timestamp
    row = np.array([7, 19, 40, 41], dtype=np.int64)
    b, it, w = run(oracle, np.tile(row, (5, 1)))
    assert (int(b[0]), int(w[0]), list(it[0])) == (7, 0, [1] * 5)
    # R = 1 is classic BSP: barrier at the slowest worker, wait = sum of gaps
    t = np.array([[13], [4], [29], [29], [1]], dtype=np.int64)
    b, it, w = run(oracle, t)
    assert (int(b[0]), int(w[0]), list(it[0])) == (29, (29 - t[:, 0]).sum(), [1] * 5)
    # P = 1: the first timestamp, nobody waits
    b, it, w = run(oracle, np.array([[5, 6, 9]], dtype=np.int64))
    assert (int(b[0]), int(w[0]), list(it[0])) == (5, 0, [1])
    # two periodic workers meet at the least common multiple of their periods
    for a, c, R in [(4, 6, 5), (3, 5, 7), (10, 15, 4), (7, 7, 3), (6, 4, 3)]:
        l = math.lcm(a, c)
        t = np.array([[a * (i + 1) for i in range(R)], [c * (i + 1) for i in range(R)]])
        b, it, w = run(oracle, t)
        if l <= min(a, c) * R:
            assert (int(b[0]), int(w[0]), list(it[0])) == (l, 0, [l // a, l // c])
        else:
            assert int(w[0]) > 0


def test_two_workers_equals_range_objective(oracle):
    # For P = 2 the summed wait of a choice Z is max(Z) - min(Z), the paper's d_Z
    # (Section III); the minimum of d_Z over all pairs is computed here directly.
    rng = np.random.default_rng(31)
    for _ in range(200):
        R = int(rng.integers(1, 9))
        t = workloads.random_small(rng, 2, R, 1, 30, ties=bool(rng.integers(0, 2)))
        d_best = min(abs(int(x) - int(y)) for x, y in itertools.product(t[0], t[1]))
        _, _, w = run(oracle, t)
        assert int(w[0]) == d_best


def test_tie_rule_earliest_barrier(oracle):
    # wait(c) is 3 at c = 10 (worker B idle since 7) and again at c = 20; first wins
    t = np.array([[10, 20, 30], [7, 17, 27]], dtype=np.int64)
    b, it, w = run(oracle, t)
    assert (int(b[0]), int(w[0]), list(it[0])) == (10, 3, [1, 1])


def test_rejects_unsorted_rows(oracle):
    t = np.array([[[1, 5, 4], [2, 3, 9]]], dtype=np.int64)
    for m in ("sweep", "definition", "naive"):
        *_, rc, _ = oracle.zipline(t, m)
        assert rc[0] == 1


def test_batch_and_threads(oracle):
    ts = workloads.make(2, instances=range(64))
    one = oracle.zipline(ts, "sweep", threads=1)
    many = oracle.zipline(ts, "sweep", threads=4)
    for x, y in zip(one[:3], many[:3]):
        assert np.array_equal(x, y)
    for j in (0, 17, 63):
        s = oracle.zipline(ts[j], "sweep")
        assert s[0][0] == one[0][j] and s[2][0] == one[2][j] and np.array_equal(s[1][0], one[1][j])


def test_workers_with_one_common_interval_closed_form(oracle):
    # the closed form the large-instance GPU tests rely on, against every route of both oracles
    from closed_forms import same_interval_workers
    rng = np.random.default_rng(31)
    for P, R, D, distinct in [(2, 3, 10, True), (5, 4, 50, True), (7, 9, 13, False), (40, 6, 1000, True), (64, 12, 37, False)]:
        for _ in range(20):
            off = rng.choice(D, size=P, replace=False) if distinct else rng.integers(0, D, size=P)
            t = (off[:, None] + np.arange(R)[None, :] * D).astype(np.int64)
            want = same_interval_workers(off, D, R)
            for m in ("sweep", "definition"):
                b, it, w, rc, _ = oracle.zipline(t, m)
                assert (int(b[0]), int(w[0])) == want["sum"][:2] and np.array_equal(it[0], want["sum"][2]), (P, R, D, off)
                b, it, d, rc, _ = oracle.zipline_range(t, m)
                assert (int(b[0]), int(d[0])) == want["range"][:2] and np.array_equal(it[0], want["range"][2]), (P, R, D, off)
