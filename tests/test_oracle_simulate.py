"""Pins for the oracle's prediction and superstep run (no GPU).

Neither has a value printed in the paper, so they are pinned to what the
mathematics fixes: runs worked by hand, the closed form of BSP (R = 1), the
closed form of identical workers, a per-worker time balance that must close in
every superstep, shift invariance, and the bound that a lookahead barrier never
costs more waiting than the BSP barrier from the same start.  A dropped
sync_cost, a barrier carried to the wrong instance, an off-by-one in the
predicted rows or a start time that is not reset fails at least one of them.
"""
import numpy as np
import pytest

from paper_2001_01347_amd import workloads


def test_predicted_rows_by_hand(oracle):
    rows = oracle.predicted_rows([[10, 0]], [[3, 7]], 4)
    assert rows.dtype == np.int64 and rows.shape == (1, 2, 4)
    assert rows.tolist() == [[[13, 16, 19, 22], [7, 14, 21, 28]]]
    # no axis is mixed up: a [S, B, P] input gains R as its last axis
    big = oracle.predicted_rows(np.zeros((2, 3, 5), dtype=np.int64), np.arange(30).reshape(2, 3, 5), 6)
    assert big.shape == (2, 3, 5, 6) and big[1, 2, 4].tolist() == [29 * i for i in range(1, 7)]
    # zero interval: the worker's row stays at its last end
    assert oracle.predicted_rows([[5]], [[0]], 3).tolist() == [[[5, 5, 5]]]


def test_two_workers_by_hand(oracle):
    # iteration times 2 and 3, both start at 0.
    # R = 3: rows (2,4,6), (3,6,9); candidates >= 3: c=3 -> (3-2)+0 = 1, c=4 -> 0+(4-3) = 1,
    # c=6 -> 0+0 = 0, c=9 -> (9-6)+0 = 3: barrier 6, wait 0, iterations (3, 2).  The next superstep
    # starts at 6 + sync_cost and repeats the pattern.
    iv = np.broadcast_to(np.array([[[2, 3]]], dtype=np.int64), (3, 1, 2))
    b, it, w, rc, _ = oracle.simulate([[0, 0]], iv, 3)
    assert (rc == 0).all()
    assert b[:, 0].tolist() == [6, 12, 18] and w[:, 0].tolist() == [0, 0, 0]
    assert it[:, 0].tolist() == [[3, 2]] * 3
    b, it, w, rc, _ = oracle.simulate([[0, 0]], iv, 3, sync_cost=5)
    assert b[:, 0].tolist() == [6, 17, 28] and w[:, 0].tolist() == [0, 0, 0]
    # R = 2: rows (2,4), (3,6); c=3 -> 1, c=4 -> 1, c=6 -> (6-4)+0 = 2: the first minimum, barrier 3,
    # wait 1, one iteration each
    b, it, w, rc, _ = oracle.simulate([[0, 0]], iv, 2)
    assert b[:, 0].tolist() == [3, 6, 9] and w[:, 0].tolist() == [1, 1, 1] and it[:, 0].tolist() == [[1, 1]] * 3
    # different start times only matter in the first superstep: worker 0 starts at 1 -> rows (3,5,7), (3,6,9):
    # c=3 -> 0, so barrier 3 with one iteration each; from then on the pattern above
    b, it, w, rc, _ = oracle.simulate([[1, 0]], iv, 3)
    assert b[:, 0].tolist() == [3, 9, 15] and w[:, 0].tolist() == [0, 0, 0]
    assert it[:, 0].tolist() == [[1, 1], [3, 2], [3, 2]]


def test_interval_changes_between_supersteps_by_hand(oracle):
    # superstep 0: times (2, 3) from 0, R = 2 -> barrier 3 (see above); superstep 1: times (4, 2) from 3 + 1:
    # rows (8, 12), (6, 8): candidates >= 8: c=8 -> 0+0: barrier 8, iterations (1, 2)
    iv = np.array([[[2, 3]], [[4, 2]]], dtype=np.int64)
    b, it, w, rc, _ = oracle.simulate([[0, 0]], iv, 2, sync_cost=1)
    assert b[:, 0].tolist() == [3, 8] and w[:, 0].tolist() == [1, 0] and it[:, 0].tolist() == [[1, 1], [1, 2]]


def test_r1_is_bsp_closed_form(oracle):
    rng = np.random.default_rng(7)
    S, B, P, sync = 9, 5, 13, 4
    le = rng.integers(0, 50, size=(B, P), dtype=np.int64)
    iv = rng.integers(1, 40, size=(S, B, P), dtype=np.int64)
    b, it, w, rc, _ = oracle.simulate(le, iv, 1, sync_cost=sync)
    assert (rc == 0).all() and (it == 1).all()
    first = (le + iv[0]).max(axis=1)
    assert np.array_equal(b[0], first) and np.array_equal(w[0], (first[:, None] - le - iv[0]).sum(axis=1))
    slowest = iv.max(axis=2)                                   # [S, B]
    for s in range(1, S):                                      # all workers start together: the slowest sets the barrier
        assert np.array_equal(b[s], b[s - 1] + sync + slowest[s])
        assert np.array_equal(w[s], (slowest[s][:, None] - iv[s]).sum(axis=1))


@pytest.mark.parametrize("R", [1, 4, 15])
def test_identical_workers_never_wait(oracle, R):
    S, B, P = 6, 3, 8
    rng = np.random.default_rng(11)
    per_step = rng.integers(1, 30, size=(S, B), dtype=np.int64)
    iv = np.repeat(per_step[:, :, None], P, axis=2)
    le = np.repeat(rng.integers(0, 9, size=(B, 1), dtype=np.int64), P, axis=1)
    b, it, w, rc, _ = oracle.simulate(le, iv, R, sync_cost=2)
    assert (w == 0).all() and (it == 1).all()                  # the first candidate already has no waiting
    assert np.array_equal(b, le[:, 0][None] + np.cumsum(per_step, axis=0) + 2 * np.arange(S)[:, None])


@pytest.mark.parametrize("R", [2, 5, 15, 30])
def test_time_balance_shift_invariance_and_bsp_bound(oracle, R):
    rng = np.random.default_rng(100 + R)
    S, B, P, sync = 7, 6, 9, 3
    le = rng.integers(0, 300, size=(B, P), dtype=np.int64)
    iv = rng.integers(20, 60, size=(S, B, P), dtype=np.int64)
    b, it, w, rc, _ = oracle.simulate(le, iv, R, sync_cost=sync)
    assert (rc == 0).all()
    start = le.copy()
    for s in range(S):
        # every worker's time from its start to the barrier is its finished iterations plus its waiting,
        # a waiting worker has not time left for another iteration, and the waits add up to the reported sum
        idle = b[s][:, None] - start - it[s] * iv[s]
        assert (idle >= 0).all() and (it[s] >= 1).all() and (it[s] <= R).all()
        assert ((idle < iv[s]) | (it[s] == R)).all()
        assert np.array_equal(idle.sum(axis=1), w[s])
        # the lookahead barrier never waits longer than the barrier after one iteration each (BSP)
        bsp = (start + iv[s]).max(axis=1)
        assert (w[s] <= (bsp[:, None] - start - iv[s]).sum(axis=1)).all() and (b[s] >= bsp).all()
        start = np.repeat((b[s] + sync)[:, None], P, axis=1)
    off = 10 ** 15
    b2, it2, w2, rc2, _ = oracle.simulate(le + off, iv, R, sync_cost=sync)
    assert np.array_equal(b2, b + off) and np.array_equal(it2, it) and np.array_equal(w2, w)
    # instances do not leak into one another: a run of one instance alone gives the same
    b3, it3, w3, _, _ = oracle.simulate(le[4:5], iv[:, 4:5], R, sync_cost=sync)
    assert np.array_equal(b3[:, 0], b[:, 4]) and np.array_equal(it3[:, 0], it[:, 4]) and np.array_equal(w3[:, 0], w[:, 4])


def test_rejected_instance_keeps_its_start_times(oracle):
    # a negative interval makes the predicted row decrease: the search rejects the instance in that
    # superstep (rc 1); the other instance is not touched and the rejected one goes on from where it was
    iv = np.array([[[2, 3], [2, 3]], [[2, 3], [2, 3]]], dtype=np.int64)
    iv[0, 1, 0] = -1
    b, it, w, rc, _ = oracle.simulate([[0, 0], [0, 0]], iv, 3)
    assert rc.tolist() == [[0, 1], [0, 0]]
    assert b[:, 0].tolist() == [6, 12]
    assert b[1, 1] == 6 and w[1, 1] == 0 and it[1, 1].tolist() == [3, 2]


def test_superstep_workload_runs_and_lookahead_reduces_waiting(oracle):
    # on the generator's workers (2 % jitter) the waiting per finished iteration falls as R grows
    le, iv = workloads.make_supersteps(2, 8, instances=range(4))
    per_iter = []
    for R in (1, 15, 60):
        b, it, w, rc, _ = oracle.simulate(le, iv, R)
        assert (rc == 0).all()
        per_iter.append(w.sum() / it.sum())
    assert per_iter[0] > per_iter[1] > per_iter[2]


def test_hand_worked_fixture(oracle):
    import json
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "worked_examples_supersteps.json")
    cases = json.load(open(path))["cases"]
    assert len(cases) >= 6
    for c in cases:
        b, it, w, rc, _ = oracle.simulate(c["last_end0"], c["interval"], c["R"], c["sync_cost"])
        assert (rc == 0).all(), c["name"]
        assert b.tolist() == c["barrier"] and w.tolist() == c["wait"] and it.tolist() == c["iters"], c["name"]


def test_fixture_is_what_its_script_writes():
    # the stored expected values come from the committed script, which calls the oracle and nothing else
    import importlib.util
    import json
    import os
    here = os.path.join(os.path.dirname(__file__), "golden")
    spec = importlib.util.spec_from_file_location("make_supersteps_fixture", os.path.join(here, "make_supersteps_fixture.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    assert json.load(open(os.path.join(here, "worked_examples_supersteps.json"))) == mod.build()
    text = open(os.path.join(here, "make_supersteps_fixture.py")).read()
    assert "paper_2001_01347_amd" not in text and "torch" not in text


def test_supersteps_worked_on_paper(oracle):
    # Values worked on paper (not read from the fixture): two workers with iteration times 2 and 3 and R = 3 have rows
    # (2,4,6) and (3,6,9); candidates from 3 on: c=3 waits (3-2)+0 = 1, c=4 waits 0+(4-3) = 1, c=6 waits 0, c=9 waits 3.
    # They meet at 6 and, restarting together, again every 6; with a synchronisation of 5 the restarts are at 11 and 22.
    le, iv = np.zeros((1, 2), dtype=np.int64), np.tile(np.array([[[2, 3]]], dtype=np.int64), (3, 1, 1))
    b, it, w, rc, _ = oracle.simulate(le, iv, 3, 0)
    assert b.ravel().tolist() == [6, 12, 18] and w.ravel().tolist() == [0, 0, 0] and it.reshape(3, 2).tolist() == [[3, 2]] * 3
    b, it, w, rc, _ = oracle.simulate(le, iv, 3, 5)
    assert b.ravel().tolist() == [6, 17, 28] and w.ravel().tolist() == [0, 0, 0]
    # R = 2: rows (2,4) and (3,6): c=3 waits 1, c=4 waits 1, c=6 waits 2: the first minimum is 3; then (5,7),(6,9): c=6 waits 1
    b, it, w, rc, _ = oracle.simulate(le, iv, 2, 0)
    assert b.ravel().tolist() == [3, 6, 9] and w.ravel().tolist() == [1, 1, 1] and it.reshape(3, 2).tolist() == [[1, 1]] * 3
    # R = 1 is BSP: three workers ending at 5, 7, 6 wait 2 + 0 + 1 at barrier 7; with a synchronisation of 2 they restart at 9
    # and, now taking 4, 4 and 9, end at 13, 13, 18: barrier 18, waits 5 + 5 + 0
    b, it, w, rc, _ = oracle.simulate(np.zeros((1, 3), dtype=np.int64), np.array([[[5, 7, 6]], [[4, 4, 9]]], dtype=np.int64), 1, 2)
    assert b.ravel().tolist() == [7, 18] and w.ravel().tolist() == [3, 10] and it.reshape(2, 3).tolist() == [[1, 1, 1]] * 2
