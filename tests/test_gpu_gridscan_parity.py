"""GridScan / FullGridScan on the GPU (``ebsp_gridscan_batch``) against their CPU oracle, bit for bit: the
smallest max(Z) - min(Z) found, the barrier max(Z*) and the position of every worker's point in Z*
(Section IV, Algorithm 1 and the FullGridScan paragraph).  Needs an MI355X."""
import json
import os

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


def gpu_run(zl, ts, full):
    d = torch.from_numpy(np.ascontiguousarray(ts)).cuda()
    out = zl.ebsp_gridscan_batch(d, full)
    torch.cuda.synchronize()
    return [x.cpu().numpy() for x in out]


def assert_same(zl, oracle, ts, label, method="bisect"):
    for full in (False, True):
        bar, it, dz, st = gpu_run(zl, ts, full)
        ob, oi, od, rc, _ = oracle.gridscan(ts, full, method, threads=16)
        assert (rc == 0).all() and (st == 0).all(), label
        assert np.array_equal(dz, od), f"{label} full={full}: d_Z differs at {np.nonzero(dz != od)[0][:5]}"
        assert np.array_equal(bar, ob), f"{label} full={full}: barrier differs at {np.nonzero(bar != ob)[0][:5]}"
        assert np.array_equal(it, oi), f"{label} full={full}: Z* differs at {np.nonzero((it != oi).any(axis=1))[0][:5]}"


def test_hand_worked_examples(zl):
    path = os.path.join(os.path.dirname(__file__), "golden", "worked_examples_gridscan.json")
    for c in json.load(open(path))["cases"]:
        for full, key in ((False, "gridscan"), (True, "fullgridscan")):
            bar, it, dz, st = gpu_run(zl, np.array([c["t"]], dtype=np.int64), full)
            assert (int(dz[0]), int(bar[0]), list(it[0]), int(st[0])) == (c[key]["dz"], c[key]["barrier"], c[key]["iters"], 0), c["name"]


@pytest.mark.parametrize("P,R", [(1, 1), (1, 9), (6, 1), (2, 3), (3, 5), (7, 9), (13, 19), (33, 31), (64, 64), (17, 241),
                                 (300, 40), (5, 4096), (3, 5000), (2, 70001), (1100, 3)])
def test_shapes(zl, oracle, P, R):
    rng = np.random.default_rng(31 * P + R)
    ts = np.stack([workloads.random_small(rng, P, R, 1, 1000, ties=(i % 2 == 0)) for i in range(4)])
    small = P * R * R * P <= 4_000_000
    assert_same(zl, oracle, ts, f"P={P} R={R}", "scan" if small else "bisect")
    assert_same(zl, oracle, ts + EPOCH, f"P={P} R={R} shifted")
    assert_same(zl, oracle, ts - 5_000_000, f"P={P} R={R} negative")


@pytest.mark.parametrize("P,R,n", [(10, 15, 64), (10, 150, 32), (100, 15, 16), (100, 150, 8), (1000, 15, 4), (1000, 150, 2)])
def test_the_shapes_of_table_two(zl, oracle, P, R, n):
    assert_same(zl, oracle, workloads.make_workers(P, R, n), f"{P} workers, R={R}")


def test_configs(zl, oracle):
    assert_same(zl, oracle, workloads.make(1), "config 1", "scan")
    assert_same(zl, oracle, workloads.make(2, instances=range(256)), "config 2")
    assert_same(zl, oracle, workloads.make(3, instances=range(8)), "config 3")
    assert_same(zl, oracle, workloads.make(4, instances=range(1)), "config 4 (ties)")


def test_degenerate_and_extreme_values(zl, oracle):
    assert_same(zl, oracle, np.full((3, 8, 16), 42, dtype=np.int64), "all equal", "scan")
    rng = np.random.default_rng(17)
    base = np.stack([workloads.random_small(rng, 9, 33, 1, 1000, ties=True) for _ in range(3)])
    assert_same(zl, oracle, base + (1 << 62) - 40_000, "near the top of int64 / 2", "scan")
    assert_same(zl, oracle, base - (1 << 62), "near the bottom of int64 / 2", "scan")
    wide = base.copy()
    wide[:, ::2, :] += (1 << 61)                     # every other worker far away: the nearest point is a row's first or last
    assert_same(zl, oracle, wide, "two groups of workers 2^61 apart", "scan")
    far = np.sort(rng.integers(-(1 << 61), 1 << 61, size=(2, 5, 40)), axis=2)
    assert_same(zl, oracle, far, "values all over +-2^61", "scan")


def test_empty_batch_and_buffers_passed_in(zl, oracle):
    empty = torch.zeros((0, 4, 8), dtype=torch.int64, device="cuda")
    out = zl.ebsp_gridscan_batch(empty, True)
    torch.cuda.synchronize()
    assert [tuple(t.shape) for t in out] == [(0,), (0, 4), (0,), (0,)]
    ts = workloads.make_workers(12, 30, 5)
    d = torch.from_numpy(ts).cuda()
    bufs = (torch.full((5,), -1, dtype=torch.int64, device="cuda"), torch.full((5, 12), -1, dtype=torch.int32, device="cuda"),
            torch.full((5,), -1, dtype=torch.int64, device="cuda"), torch.full((5,), -1, dtype=torch.int32, device="cuda"))
    ws = torch.empty(zl.ebsp_gridscan_workspace_bytes(5, 12, 30, True), dtype=torch.uint8, device="cuda")
    got = zl.ebsp_gridscan_batch(d, True, *bufs, workspace=ws)
    torch.cuda.synchronize()
    assert all(a is b for a, b in zip(got, bufs))
    ob, oi, od, rc, _ = oracle.gridscan(ts, True, "scan")
    assert np.array_equal(bufs[0].cpu().numpy(), ob) and np.array_equal(bufs[1].cpu().numpy(), oi)
    assert np.array_equal(bufs[2].cpu().numpy(), od) and (bufs[3].cpu().numpy() == 0).all()
    with pytest.raises(ValueError):
        zl.ebsp_gridscan_batch(d, True, bufs[0].to(torch.int32))
    with pytest.raises(ValueError):
        zl.ebsp_gridscan_batch(d, True, workspace=ws[:ws.numel() - 256])


def test_never_below_the_exact_search(zl):
    # both scans build sets of one timestamp per worker: ebsp_zipline_range_batch's optimum bounds them from below
    ts = torch.from_numpy(workloads.make(2, instances=range(512))).cuda()
    exact = zl.ebsp_zipline_range_batch(ts)[2]
    heur = zl.ebsp_gridscan_batch(ts, False)[2]
    full = zl.ebsp_gridscan_batch(ts, True)[2]
    torch.cuda.synchronize()
    assert bool((full >= exact).all()) and bool((heur >= full).all())


def test_unsorted_row_is_flagged(zl):
    rng = np.random.default_rng(5)
    ts = np.stack([workloads.random_small(rng, 12, 80, 1, 100) for _ in range(4)])
    ts[1, 3, 40] = ts[1, 3, 39] - 1
    for full in (False, True):
        st = gpu_run(zl, ts, full)[3]
        assert st[1] == zl.STATUS_UNSORTED and (np.delete(st, 1) == 0).all()


def test_argument_errors(zl):
    lib = zl.load()
    ts = torch.zeros((1, 2, 2), dtype=torch.int64, device="cuda")
    assert lib.ebsp_gridscan_batch(ts.data_ptr(), 1, 0, 2, 0, ts.data_ptr(), ts.data_ptr(), ts.data_ptr(), None, None, 0, None) == -2
    assert lib.ebsp_gridscan_batch(None, 1, 2, 2, 0, ts.data_ptr(), ts.data_ptr(), ts.data_ptr(), None, None, 0, None) == -1
    assert lib.ebsp_gridscan_batch(ts.data_ptr(), 1, 2, 2, 1, ts.data_ptr(), ts.data_ptr(), ts.data_ptr(), None, ts.data_ptr(), 0, None) == -3
    assert zl.ebsp_gridscan_workspace_bytes(4, 100, 15, True) >= 4 * 100 * 16 and zl.ebsp_gridscan_workspace_bytes(4, 0, 15, True) == 0
