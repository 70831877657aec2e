"""Pins for the CPU oracle of the paper's formal objective d_Z = max(Z) - min(Z)
(Section III "The Problem"; Algorithm 2; Fig. 3 caption).  Everything here runs on the CPU.

The oracle has four routes (exhaustive search over all choices Z, the definition
written out, Algorithm 2 as printed, a queue-based sweep for large inputs).  They are
pinned by hand-worked fixtures, by each other on random inputs with many ties, by the
case P = 2 in which this objective and the summed waiting time are the same number
(computed by the other oracle file), by a closed form, and by properties checked with
numpy code that shares nothing with the C file.
"""
import json
import os

import numpy as np
import pytest

from paper_2001_01347_amd import workloads

ROUTES = ["sweep", "definition", "naive", "latest"]


def run(oracle, ts, method="sweep"):
    bar, it, d, rc, _ = oracle.zipline_range(ts, method, threads=8)
    assert (rc == 0).all()
    return bar, it, d


def lowest_last(t, c):
    """min_p of the latest timestamp of row p at or before c (numpy, independent of the C code)."""
    lasts = []
    for row in t:
        k = np.searchsorted(row, c, side="right")
        assert k > 0
        lasts.append(row[k - 1])
    return min(lasts)


def test_hand_worked_examples(oracle):
    path = os.path.join(os.path.dirname(__file__), "golden", "worked_examples_range.json")
    for c in json.load(open(path))["cases"]:
        t = np.array([c["t"]], dtype=np.int64)
        for m in ROUTES:
            bar, it, d = run(oracle, t, m)
            assert (int(bar[0]), int(d[0]), list(it[0])) == (c["barrier"], c["dmin"], c["iters"]), (c["name"], m)


def test_routes_agree_on_random_small_inputs(oracle):
    rng = np.random.default_rng(20010134)
    for trial in range(400):
        P, R = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        if R ** P > 4000:
            continue
        ts = np.stack([workloads.random_small(rng, P, R, 0, 25, ties=(trial % 2 == 0)) for _ in range(3)])
        ref = run(oracle, ts, "naive")
        for m in ["sweep", "definition", "latest"]:
            got = run(oracle, ts, m)
            for a, b in zip(ref, got):
                assert np.array_equal(a, b), (trial, m)


def test_sweeps_agree_with_the_definition_on_medium_inputs(oracle):
    rng = np.random.default_rng(7)
    for P, R in [(7, 40), (30, 12), (64, 9)]:
        ts = np.stack([workloads.random_small(rng, P, R, 0, 300, ties=(i % 2 == 0)) for i in range(4)])
        ref = run(oracle, ts, "definition")
        for m in ["sweep", "latest"]:
            for a, b in zip(ref, run(oracle, ts, m)):
                assert np.array_equal(a, b), (P, R, m)


def test_two_workers_same_as_summed_wait(oracle):
    # with two workers the worker at the barrier waits 0 and the other one max(Z) - min(Z):
    # both objectives are the same function, so the other oracle file must give the same answer
    rng = np.random.default_rng(3)
    ts = np.stack([workloads.random_small(rng, 2, 60, 0, 2000, ties=(i % 2 == 0)) for i in range(64)])
    bar, it, d = run(oracle, ts)
    sbar, sit, swait, rc, _ = oracle.zipline(ts, "sweep", threads=8)
    assert np.array_equal(bar, sbar) and np.array_equal(d, swait) and np.array_equal(it, sit)


def test_staggered_periodic_workers_closed_form(oracle):
    # worker p ends iterations at p*g + i*T with T = P*g: at every time from (P-1)*g on the
    # oldest of the latest timestamps is (P-1)*g old, so d* = (P-1)*g at the first admissible time
    for P, g, R in [(2, 5, 4), (5, 3, 7), (16, 11, 30)]:
        T = P * g
        t = np.array([[p * g + i * T for i in range(R)] for p in range(P)], dtype=np.int64)
        for m in ["sweep", "latest"] + (["definition"] if P * R <= 200 else []):
            bar, it, d = run(oracle, t[None], m)
            assert (int(bar[0]), int(d[0])) == ((P - 1) * g, (P - 1) * g), (P, m)
            assert list(it[0]) == [1] * P


def test_result_satisfies_its_definition_and_is_minimal(oracle):
    ts = workloads.make(2, instances=range(24))
    bar, it, d = run(oracle, ts)
    for b in range(ts.shape[0]):
        t = ts[b]
        thr = t[:, 0].max()
        assert bar[b] >= thr and (t == bar[b]).any()
        assert d[b] == bar[b] - lowest_last(t, bar[b])
        assert np.array_equal(it[b], (t <= bar[b]).sum(axis=1))
        cands = np.unique(t[t >= thr])
        vals = np.array([c - lowest_last(t, c) for c in cands])
        assert d[b] == vals.min() and bar[b] == cands[np.argmin(vals)]       # argmin: the first minimum


def test_shift_scale_and_added_worker(oracle):
    rng = np.random.default_rng(11)
    ts = np.stack([workloads.random_small(rng, 6, 20, 0, 500, ties=True) for _ in range(8)])
    bar, it, d = run(oracle, ts)
    sb, si, sd = run(oracle, ts + 1_700_000_000_000_000)
    assert np.array_equal(sb, bar + 1_700_000_000_000_000) and np.array_equal(sd, d) and np.array_equal(si, it)
    kb, ki, kd = run(oracle, ts * 1000)
    assert np.array_equal(kb, bar * 1000) and np.array_equal(kd, d * 1000) and np.array_equal(ki, it)
    # one more worker can only make the fastest worker wait longer
    more = np.concatenate([ts, np.stack([workloads.random_small(rng, 1, 20, 0, 500, ties=True) for _ in range(8)])], axis=1)
    _, _, d_more = run(oracle, more)
    assert (d_more >= d).all()


def test_degenerate_shapes_and_bad_rows(oracle):
    bar, it, d = run(oracle, np.array([[[4, 9, 9, 12]]], dtype=np.int64))
    assert (int(bar[0]), int(d[0]), list(it[0])) == (4, 0, [1])
    bar, it, d = run(oracle, np.full((1, 5, 3), 8, dtype=np.int64))
    assert (int(bar[0]), int(d[0]), list(it[0])) == (8, 0, [3] * 5)
    t = np.array([[[1, 2, 3], [5, 4, 6]]], dtype=np.int64)
    for m in ROUTES:
        assert oracle.zipline_range(t, m)[3][0] == 1
