"""Pins of the GridScan / FullGridScan oracle (Section IV, Algorithm 1 and the FullGridScan paragraph):
hand-worked fixtures, the two routes against each other, a slow search written out in Python from the
definition, and what the mathematics fixes (never below the exact optimum, exact for two workers, the
full scan never worse than the heuristic, closed forms, invariances)."""
import json
import os

import numpy as np
import pytest

from paper_2001_01347_amd import workloads

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "worked_examples_gridscan.json")


def cases():
    return json.load(open(GOLDEN))["cases"]


@pytest.mark.parametrize("case", cases(), ids=lambda c: c["name"])
@pytest.mark.parametrize("method", ["scan", "bisect"])
def test_hand_worked(oracle, case, method):
    t = np.array([case["t"]], dtype=np.int64)
    for full, key in ((False, "gridscan"), (True, "fullgridscan")):
        bar, it, dz, rc, _ = oracle.gridscan(t, full, method)
        want = case[key]
        assert (int(dz[0]), int(bar[0]), list(it[0]), int(rc[0])) == (want["dz"], want["barrier"], want["iters"], 0), (key, method)


def slow_search(t, full):
    """Algorithm 1 from its words: Z = the designated point and every other row's nearest point."""
    P, R = t.shape
    rows = range(P) if full else [min(range(P), key=lambda p: (t[p][0], p))]
    best = None
    for pb in rows:
        for j in range(R):
            e = int(t[pb][j])
            z = []
            for p in range(P):
                if p == pb:
                    z.append(j)
                else:
                    z.append(min(range(R), key=lambda i: (abs(int(t[p][i]) - e), i)))
            vals = [int(t[p][z[p]]) for p in range(P)]
            d = max(vals) - min(vals)
            if best is None or d < best[0]:
                best = (d, max(vals), [i + 1 for i in z])
    return best


def test_against_the_definition_in_python(oracle):
    rng = np.random.default_rng(11)
    for k in range(60):
        P, R = int(rng.integers(1, 6)), int(rng.integers(1, 8))
        t = workloads.random_small(rng, P, R, 1, 12 if k % 2 else 1000, ties=(k % 3 == 0))
        for full in (False, True):
            want = slow_search(t, full)
            for method in ("scan", "bisect"):
                bar, it, dz, rc, _ = oracle.gridscan(t, full, method)
                assert (int(dz[0]), int(bar[0]), list(it[0])) == want, (k, full, method)


def test_routes_agree_on_larger_inputs(oracle):
    rng = np.random.default_rng(12)
    ts = np.stack([workloads.random_small(rng, 24, 70, 1, 400, ties=(i % 2 == 0)) for i in range(6)])
    for full in (False, True):
        a = oracle.gridscan(ts, full, "scan", threads=8)
        b = oracle.gridscan(ts, full, "bisect", threads=8)
        for x, y in zip(a[:4], b[:4]):
            assert np.array_equal(x, y)


def test_bounds_from_the_exact_search(oracle):
    # every Z the scans build is one timestamp per worker, so neither can beat the exact optimum of
    # max(Z) - min(Z) (the range oracle); the full scan looks at a superset of the heuristic's sets
    rng = np.random.default_rng(13)
    ts = np.stack([workloads.random_small(rng, 7, 20, 1, 300, ties=(i % 2 == 0)) for i in range(40)])
    _, _, exact, _, _ = oracle.zipline_range(ts, "sweep")
    _, _, heur, _, _ = oracle.gridscan(ts, False)
    _, _, full, _, _ = oracle.gridscan(ts, True)
    assert (full >= exact).all() and (heur >= full).all()
    assert (heur > full).any() or (full > exact).any()      # the inputs do tell the three apart


def test_two_workers_is_exact(oracle):
    # with two workers the closest pair holds, for either of its points, the other row's nearest point
    rng = np.random.default_rng(14)
    ts = np.stack([workloads.random_small(rng, 2, 30, 1, 500, ties=(i % 2 == 0)) for i in range(50)])
    _, _, exact, _, _ = oracle.zipline_range(ts, "sweep")
    assert np.array_equal(oracle.gridscan(ts, False)[2], exact)
    assert np.array_equal(oracle.gridscan(ts, True)[2], exact)


def test_closed_forms_and_invariances(oracle):
    rng = np.random.default_rng(15)
    t = workloads.random_small(rng, 6, 15, 1, 200, ties=False)[None]
    for full in (False, True):
        bar, it, dz, rc, _ = oracle.gridscan(t, full)
        # the three outputs describe one set Z*
        vals = t[0, np.arange(6), it[0] - 1]
        assert vals.max() == bar[0] and vals.max() - vals.min() == dz[0]
        # a shift of all timestamps moves the barrier and nothing else
        b2, i2, d2, _, _ = oracle.gridscan(t + 1_700_000_000_000_000, full)
        assert b2[0] == bar[0] + 1_700_000_000_000_000 and d2[0] == dz[0] and np.array_equal(i2, it)
        # identical workers: every Z is one timestamp n times
        same = np.tile(np.cumsum(rng.integers(1, 50, size=12)), (1, 5, 1)).astype(np.int64)
        b3, i3, d3, _, _ = oracle.gridscan(same, full)
        assert d3[0] == 0 and b3[0] == same[0, 0, 0] and (i3 == 1).all()
    # the full scan does not depend on the order of the workers (values; the tie order may)
    perm = rng.permutation(6)
    assert oracle.gridscan(t[:, perm], True)[2][0] == oracle.gridscan(t, True)[2][0]
    # an unsorted row is refused
    bad = t.copy()
    bad[0, 2, 5] = bad[0, 2, 4] - 1
    assert oracle.gridscan(bad, True)[3][0] == 1


def test_c_entry_point_of_the_zipline_oracle(oracle):
    # ebsp_zipline_oracle (include/ebsp_zipline_oracle.h) is the sweep route over a batch
    rng = np.random.default_rng(16)
    ts = np.stack([workloads.random_small(rng, 9, 33, 1, 700, ties=(i % 2 == 0)) for i in range(12)])
    bar, it, w, rc = oracle.zipline_c_abi(ts, threads=4)
    ob, oi, ow, orc, _ = oracle.zipline(ts, "sweep")
    assert rc == 0 and np.array_equal(bar, ob) and np.array_equal(it, oi) and np.array_equal(w, ow)
    ob2, oi2, ow2, _, _ = oracle.zipline(ts[:3], "definition")
    assert np.array_equal(bar[:3], ob2) and np.array_equal(w[:3], ow2) and np.array_equal(it[:3], oi2)
    bad = ts.copy()
    bad[4, 1, 7] = bad[4, 1, 6] - 1
    bar, it, w, rc = oracle.zipline_c_abi(bad)
    assert rc == 1 and bar[4] == 0 and np.array_equal(np.delete(bar, 4), np.delete(ob, 4))
