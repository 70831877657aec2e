"""Parity of ``ebsp_simulate_supersteps`` (S supersteps of predict -> search -> resume at the
barrier, all on the device) with the CPU oracle's run, through the C ABI (needs an MI355X).
Bar: bit-exact on barrier, iters and wait of every superstep.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2001_01347_amd import workloads  # noqa: E402

EPOCH = 1_700_000_000_000_000


@pytest.fixture(scope="module")
def zl():
    assert torch.cuda.is_available(), "these tests need a GPU"
    from paper_2001_01347_amd import zipline
    zipline.load()
    return zipline


def gpu_run(zl, le, iv, R, sync_cost=0):
    out = zl.ebsp_simulate_supersteps(torch.from_numpy(np.ascontiguousarray(le)).cuda(),
                                      torch.from_numpy(np.ascontiguousarray(iv)).cuda(), R, sync_cost)
    torch.cuda.synchronize()
    return tuple(x.cpu().numpy() for x in out)


def assert_same(zl, oracle, le, iv, R, sync_cost=0, label=""):
    bar, it, w, st = gpu_run(zl, le, iv, R, sync_cost)
    ob, oi, ow, rc, _ = oracle.simulate(le, iv, R, sync_cost, threads=16)
    assert (rc == 0).all()
    assert (st == 0).all(), f"{label}: status {np.unique(st)}"
    for s in range(iv.shape[0]):
        assert np.array_equal(w[s], ow[s]), f"{label}: superstep {s}: wait differs at {np.nonzero(w[s] != ow[s])[0][:5]}"
        assert np.array_equal(bar[s], ob[s]), f"{label}: superstep {s}: barrier differs"
        assert np.array_equal(it[s], oi[s]), f"{label}: superstep {s}: iters differ"


def test_hand_worked_run(zl):
    # iteration times 2 and 3 from time 0, R = 3: rows (2,4,6), (3,6,9) -> barrier 6 without waiting,
    # iterations (3, 2); with a synchronisation of 5 the next superstep starts at 11
    iv = np.broadcast_to(np.array([[[2, 3]]], dtype=np.int64), (3, 1, 2))
    bar, it, w, st = gpu_run(zl, np.zeros((1, 2), dtype=np.int64), iv, 3, 5)
    assert (st == 0).all()
    assert bar[:, 0].tolist() == [6, 17, 28] and w[:, 0].tolist() == [0, 0, 0] and it[:, 0].tolist() == [[3, 2]] * 3
    bar, it, w, st = gpu_run(zl, np.zeros((1, 2), dtype=np.int64), iv, 2)
    assert bar[:, 0].tolist() == [3, 6, 9] and w[:, 0].tolist() == [1, 1, 1] and it[:, 0].tolist() == [[1, 1]] * 3


@pytest.mark.parametrize("P,R", [(1, 1), (5, 1), (2, 3), (7, 15), (16, 30), (64, 60), (100, 120), (64, 240), (300, 15)])
def test_single_workgroup_shapes(zl, oracle, P, R):
    rng = np.random.default_rng(5000 * P + R)
    S, B = 6, 5
    mean = rng.integers(50, 400, size=(B, P))
    iv = np.maximum(np.rint(mean[None] * (1.0 + 0.05 * rng.standard_normal((S, B, P)))).astype(np.int64), 1)
    le = rng.integers(0, 400, size=(B, P)).astype(np.int64)
    assert_same(zl, oracle, le, iv, R, 0, f"P={P} R={R}")
    assert_same(zl, oracle, le + EPOCH, iv, R, 7, f"P={P} R={R} shifted, sync 7")


@pytest.mark.parametrize("P,R,cap", [(1024, 240, 0), (600, 1000, 0), (2048, 120, 0), (256, 4096, 4096)])
def test_multi_window_shapes(zl, oracle, P, R, cap):
    # shapes the library cuts into windows (several windows per instance, a ragged last one)
    rng = np.random.default_rng(P + R)
    S, B = 4, 3
    mean = rng.integers(90_000, 300_000, size=(B, P))
    iv = np.maximum(np.rint(mean[None] * (1.0 + 0.02 * rng.standard_normal((S, B, P)))).astype(np.int64), 1)
    le = rng.integers(0, 300_000, size=(B, P)).astype(np.int64) + EPOCH
    zl.ebsp_zipline_tune(cap, 0, 0)
    try:
        assert zl.ebsp_zipline_shape_info(B, P, R)["multi"] == 1
        assert_same(zl, oracle, le, iv, R, 1500, f"P={P} R={R} cap={cap}")
    finally:
        zl.ebsp_zipline_tune(0, 0, 0)


@pytest.mark.parametrize("k,S,n", [(2, 8, 32), (3, 5, 16), (4, 3, 2), (5, 2, 1)])
def test_generator_workloads(zl, oracle, k, S, n):
    cfg = workloads.CONFIGS[k]
    le, iv = workloads.make_supersteps(k, S, instances=range(n))
    assert_same(zl, oracle, le, iv, cfg.R, 2000, f"config {k}, {S} supersteps, {n} instances")


def test_every_superstep_is_one_search_from_the_previous_barrier(zl):
    # the device run against the library's own single search, step by step (sizes the oracle would take long for)
    cfg = workloads.CONFIGS[5]
    S, n, sync = 3, 4, 2500
    le, iv = workloads.make_supersteps(5, S, instances=range(n))
    bar, it, w, st = gpu_run(zl, le, iv, cfg.R, sync)
    assert (st == 0).all()
    start = torch.from_numpy(le).cuda()
    for s in range(S):
        b1, i1, w1, s1 = zl.ebsp_predict_zipline_batch(start, torch.from_numpy(np.ascontiguousarray(iv[s])).cuda(), cfg.R)
        assert np.array_equal(b1.cpu().numpy(), bar[s]) and np.array_equal(w1.cpu().numpy(), w[s])
        assert np.array_equal(i1.cpu().numpy(), it[s])
        start = (b1 + sync)[:, None].expand(n, cfg.P).contiguous()


def test_flagged_instance_keeps_its_start_and_others_go_on(zl, oracle):
    # a negative iteration time in superstep 0 of instance 1: that superstep is flagged for it, its
    # workers start superstep 1 where they started superstep 0; instance 0 is not touched
    S, B, P, R = 3, 2, 40, 20
    rng = np.random.default_rng(77)
    iv = rng.integers(10, 50, size=(S, B, P)).astype(np.int64)
    le = rng.integers(0, 50, size=(B, P)).astype(np.int64)
    bad = iv.copy()
    bad[0, 1, 3] = -5
    bar, it, w, st = gpu_run(zl, le, bad, R, 3)
    assert st.tolist() == [[0, zl.STATUS_UNSORTED], [0, 0], [0, 0]]
    ob, oi, ow, rc, _ = oracle.simulate(le, bad, R, 3)
    assert rc.tolist() == [[0, 1], [0, 0], [0, 0]]
    assert np.array_equal(bar[:, 0], ob[:, 0]) and np.array_equal(w[:, 0], ow[:, 0]) and np.array_equal(it[:, 0], oi[:, 0])
    assert np.array_equal(bar[1:, 1], ob[1:, 1]) and np.array_equal(w[1:, 1], ow[1:, 1]) and np.array_equal(it[1:, 1], oi[1:, 1])


def test_outputs_and_workspace_passed_in_are_used(zl, oracle):
    S, B, P, R = 4, 3, 600, 240
    le, iv = np.zeros((B, P), dtype=np.int64), np.random.default_rng(3).integers(1000, 3000, size=(S, B, P)).astype(np.int64)
    need = zl.ebsp_simulate_workspace_bytes(B, P, R)
    assert need >= B * P * 8
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    outs = (torch.full((S, B), -1, dtype=torch.int64, device="cuda"), torch.full((S, B, P), -1, dtype=torch.int32, device="cuda"),
            torch.full((S, B), -1, dtype=torch.int64, device="cuda"), torch.full((S, B), -1, dtype=torch.int32, device="cuda"))
    got = zl.ebsp_simulate_supersteps(torch.from_numpy(le).cuda(), torch.from_numpy(iv).cuda(), R, 10, *outs, workspace=ws)
    torch.cuda.synchronize()
    assert all(a is b for a, b in zip(got, outs))
    ob, oi, ow, rc, _ = oracle.simulate(le, iv, R, 10, threads=16)
    assert np.array_equal(outs[0].cpu().numpy(), ob) and np.array_equal(outs[1].cpu().numpy(), oi)
    assert np.array_equal(outs[2].cpu().numpy(), ow) and (outs[3].cpu().numpy() == 0).all()
    # a workspace that is too small, outputs of the wrong type or shape (refused by the binding, before any address
    # reaches the library), a negative synchronisation time (refused by the library): nothing runs
    with pytest.raises(ValueError):
        zl.ebsp_simulate_supersteps(torch.from_numpy(le).cuda(), torch.from_numpy(iv).cuda(), R, 10, workspace=ws[:need - 256])
    with pytest.raises(ValueError):
        zl.ebsp_simulate_supersteps(torch.from_numpy(le).cuda(), torch.from_numpy(iv).cuda(), R, 10, outs[0].to(torch.int32))
    with pytest.raises(ValueError):
        zl.ebsp_simulate_supersteps(torch.from_numpy(le).cuda(), torch.from_numpy(iv).cuda(), R, 10, outs[0], outs[1][:, :, :P - 1])
    with pytest.raises(ValueError):
        zl.ebsp_simulate_supersteps(torch.from_numpy(le).cuda(), torch.from_numpy(iv).cuda(), R, 10, outs[0].cpu())
    with pytest.raises(zl.ZipLineError):
        zl.ebsp_simulate_supersteps(torch.from_numpy(le).cuda(), torch.from_numpy(iv).cuda(), R, -1)


def test_empty_runs(zl):
    le = torch.zeros((3, 4), dtype=torch.int64, device="cuda")
    b, it, w, st = zl.ebsp_simulate_supersteps(le, torch.zeros((0, 3, 4), dtype=torch.int64, device="cuda"), 5)
    assert b.shape == (0, 3) and it.shape == (0, 3, 4)
    b, it, w, st = zl.ebsp_simulate_supersteps(le[:0], torch.zeros((2, 0, 4), dtype=torch.int64, device="cuda"), 5)
    assert b.shape == (2, 0)


def test_study_rows_follow_from_the_oracle_run(zl, oracle):
    from paper_2001_01347_amd import superstep_study
    S, n, sync = 6, 8, 2000
    rows = superstep_study.study(2, (1, 15, 60), S, n, sync)
    le, iv = workloads.make_supersteps(2, S, instances=range(n))
    for row in rows:
        ob, oi, ow, rc, _ = oracle.simulate(le, iv, row["R"], sync, threads=8)
        total = float((ob[S - 1][:, None] - le).sum())
        assert row["wait_per_iteration"] == pytest.approx(ow.sum() / oi.sum(), rel=1e-12)
        assert row["waiting_share"] == pytest.approx(ow.sum() / total, rel=1e-12)
        assert row["iterations_per_superstep"] == pytest.approx(oi.sum() / (S * n * 16), rel=1e-12)
        # computing, waiting and synchronising account for all of the workers' time
        assert row["waiting_share"] + row["sync_share"] + row["computing_share"] == pytest.approx(1.0, abs=1e-12)
    assert rows[0]["R"] == 1 and rows[0]["iterations_per_superstep"] == 1.0
    assert rows[0]["waiting_share"] > rows[1]["waiting_share"] > rows[2]["waiting_share"]


@pytest.mark.parametrize("B,P,R", [(64, 16, 64), (3, 600, 240)])
def test_run_replays_from_a_hip_graph(zl, oracle, B, P, R):
    # the call enqueues kernels only (no allocation, no memset, no host round trip), so a caller can
    # capture it once and replay it on new inputs written into the same buffers
    S, sync = 10, 1200
    rng = np.random.default_rng(B + P)
    le_dev = torch.zeros((B, P), dtype=torch.int64, device="cuda")
    iv_dev = torch.ones((S, B, P), dtype=torch.int64, device="cuda")
    outs = (torch.empty((S, B), dtype=torch.int64, device="cuda"), torch.empty((S, B, P), dtype=torch.int32, device="cuda"),
            torch.empty((S, B), dtype=torch.int64, device="cuda"), torch.empty((S, B), dtype=torch.int32, device="cuda"))
    ws = torch.empty(zl.ebsp_simulate_workspace_bytes(B, P, R), dtype=torch.uint8, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        zl.ebsp_simulate_supersteps(le_dev, iv_dev, R, sync, *outs, workspace=ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        zl.ebsp_simulate_supersteps(le_dev, iv_dev, R, sync, *outs, workspace=ws)
    for rep in range(3):
        le = rng.integers(0, 100_000, size=(B, P)).astype(np.int64) + rep * EPOCH
        iv = rng.integers(50_000, 150_000, size=(S, B, P)).astype(np.int64)
        le_dev.copy_(torch.from_numpy(le))                  # eager work between the replays
        iv_dev.copy_(torch.from_numpy(iv))
        for o in outs:
            o.fill_(-1)
        graph.replay()
        torch.cuda.synchronize()
        ob, oi, ow, rc, _ = oracle.simulate(le, iv, R, sync, threads=16)
        assert (outs[3].cpu().numpy() == 0).all(), rep
        assert np.array_equal(outs[0].cpu().numpy(), ob) and np.array_equal(outs[2].cpu().numpy(), ow), rep
        assert np.array_equal(outs[1].cpu().numpy(), oi), rep
        eager = zl.ebsp_simulate_supersteps(le_dev, iv_dev, R, sync)
        assert all(torch.equal(a, b) for a, b in zip(eager, outs)), rep


def test_hand_worked_fixture(zl):
    import json
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "worked_examples_supersteps.json")
    for c in json.load(open(path))["cases"]:
        bar, it, w, st = gpu_run(zl, np.array(c["last_end0"], dtype=np.int64), np.array(c["interval"], dtype=np.int64),
                                 c["R"], c["sync_cost"])
        assert (st == 0).all(), c["name"]
        assert bar.tolist() == c["barrier"] and w.tolist() == c["wait"] and it.tolist() == c["iters"], c["name"]
