"""Parity of the HIP path with the CPU oracle for the paper's formal objective
d_Z = max(Z) - min(Z) (``ebsp_zipline_range_batch``), through the C ABI (needs an MI355X).

Bar: bit-exact on barrier (int64), dmin (int64) and iters (int32); the result is unique
(first minimum), also for instances whose value spread does not fit 32 bits.
"""
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


def gpu_run(zl, ts):
    d = torch.from_numpy(np.ascontiguousarray(ts)).cuda()
    bar, it, dm, st = zl.ebsp_zipline_range_batch(d)
    torch.cuda.synchronize()
    return bar.cpu().numpy(), it.cpu().numpy(), dm.cpu().numpy(), st.cpu().numpy()


def assert_same(zl, oracle, ts, label=""):
    bar, it, dm, st = gpu_run(zl, ts)
    ob, oi, od, rc, _ = oracle.zipline_range(ts, "sweep", threads=16)
    assert (rc == 0).all()
    assert (st == 0).all(), f"{label}: status {np.unique(st)}"
    assert np.array_equal(dm, od), f"{label}: dmin differs at {np.nonzero(dm != od)[0][:5]}"
    assert np.array_equal(bar, ob), f"{label}: barrier differs at {np.nonzero(bar != ob)[0][:5]}"
    assert np.array_equal(it, oi), f"{label}: iters differ at {np.nonzero((it != oi).any(axis=1))[0][:5]}"


def test_hand_worked_examples(zl):
    path = os.path.join(os.path.dirname(__file__), "golden", "worked_examples_range.json")
    for c in json.load(open(path))["cases"]:
        bar, it, dm, st = gpu_run(zl, np.array([c["t"]], dtype=np.int64))
        assert (int(bar[0]), int(dm[0]), list(it[0]), int(st[0])) == (c["barrier"], c["dmin"], c["iters"], 0), c["name"]


def test_config1_and_config2_full(zl, oracle):
    assert_same(zl, oracle, workloads.make(1), "config 1")
    assert_same(zl, oracle, workloads.make(2), "config 2")
    assert_same(zl, oracle, workloads.make(2, instances=range(64)) + EPOCH, "config 2 shifted")


@pytest.mark.parametrize("P,R", [(1, 1), (1, 9), (6, 1), (2, 3), (3, 5), (7, 9), (4, 16), (13, 19), (64, 64),
                                 (8, 1024), (8192, 1), (100, 81), (16, 64), (1, 1024), (1025, 1), (30, 60), (2, 1024),
                                 (2049, 1), (33, 100), (64, 64), (4097, 1), (90, 90)])
def test_single_workgroup_shapes(zl, oracle, P, R):
    rng = np.random.default_rng(1000 * P + R)
    ts = np.stack([workloads.random_small(rng, P, R, 1, 1000, ties=(i % 2 == 0)) for i in range(6)])
    assert_same(zl, oracle, ts, f"P={P} R={R}")
    assert_same(zl, oracle, ts * 1000 + EPOCH, f"P={P} R={R} scaled and shifted")


@pytest.mark.parametrize("P,R", [(1, 8193), (8193, 1), (64, 257), (5, 4000), (300, 100), (128, 512), (1100, 40)])
def test_multi_window_shapes(zl, oracle, P, R):
    rng = np.random.default_rng(77 * P + R)
    ts = np.stack([workloads.random_small(rng, P, R, 1, 1000, ties=(i % 2 == 0)) for i in range(3)])
    assert_same(zl, oracle, ts * 1000 + EPOCH, f"P={P} R={R}")


@pytest.mark.parametrize("P,R", [(8, 1024), (16, 4096), (600, 64)])
def test_equal_minima_far_apart(zl, oracle, P, R):
    # staggered workers of one period: d = (P-1)*g at every time once all have started;
    # worker 0 joins k periods late, so the first admissible time wins
    g, k = 7, R // 3
    T = P * g
    i = np.arange(R, dtype=np.int64)
    t = np.stack([p * g + i * T for p in range(P)])
    t[0] = (i + k) * T
    ts = np.stack([t, t + 3 + EPOCH])
    bar, it, dm, st = gpu_run(zl, ts)
    assert (st == 0).all()
    assert list(bar) == [k * T, k * T + 3 + EPOCH] and list(dm) == [(P - 1) * g] * 2
    assert_same(zl, oracle, ts, f"staggered P={P} R={R}")


def test_configs_3_to_5_samples(zl, oracle):
    assert_same(zl, oracle, workloads.make(3, instances=range(96)), "config 3 sample")
    assert_same(zl, oracle, workloads.make(4, instances=range(6)), "config 4 sample")
    assert_same(zl, oracle, workloads.make(5, instances=range(2)), "config 5 sample")
    assert_same(zl, oracle, workloads.make(4, instances=range(2)) + EPOCH, "config 4 shifted")


def test_skew_and_ties(zl, oracle):
    t = workloads.make(4, instances=range(2)).copy()
    t[:, 7, :] = t[:, 7, :1] + (t[:, 7, :] - t[:, 7, :1]) * 20        # one worker 20x slower
    assert_same(zl, oracle, t, "straggler x20")
    assert_same(zl, oracle, np.full((3, 8, 16), 42, dtype=np.int64), "all equal")
    assert_same(zl, oracle, np.full((2, 64, 512), -7, dtype=np.int64), "all equal, more than a workgroup holds")
    rng = np.random.default_rng(12)
    few = np.sort(rng.integers(0, 4, size=(2, 64, 1024)), axis=2).astype(np.int64) * 1_000_003
    assert_same(zl, oracle, few, "four distinct values")
    c = np.sort(rng.integers(0, 50_000, size=(1, 40, 1000)), axis=2).astype(np.int64)
    c[0, 0, -1] = 10 ** 9
    assert_same(zl, oracle, c, "cluster and outlier")
    row = np.cumsum(np.arange(1, 301, dtype=np.int64))
    assert_same(zl, oracle, np.tile(row, (2, 20, 1)), "identical workers")


def test_status_flags(zl, oracle):
    ts = workloads.make(2, instances=range(8)).copy()
    ts[3, 5, 10] = ts[3, 5, 9] - 1                      # one row of one instance goes backwards
    bar, it, dm, st = gpu_run(zl, ts)
    assert st[3] & zl.STATUS_UNSORTED and (np.delete(st, 3) == 0).all()
    ob, oi, od, rc, _ = oracle.zipline_range(np.delete(ts, 3, axis=0), "sweep", threads=8)
    assert np.array_equal(np.delete(bar, 3), ob) and np.array_equal(np.delete(dm, 3), od)
    # a spread of 2^32 or more is no reason for a flag
    wide = workloads.make(2, instances=range(4)).copy()
    wide[2] *= 1 << 20
    bar, it, dm, st = gpu_run(zl, wide)
    assert (st == 0).all()
    ms = workloads.make(3, instances=range(4)).copy()
    ms[1, 9, 100] = ms[1, 9, 99] - 5
    bar, it, dm, st = gpu_run(zl, ms)
    assert st[1] & zl.STATUS_UNSORTED and (np.delete(st, 1) == 0).all()


def _properties_hold(ts, bar, it, dm):
    """Checks that hold at any size (torch, on the GPU): each worker stops at its last timestamp
    <= barrier, the barrier is some worker's stop, and dmin is the barrier minus the earliest stop."""
    B, P, R = ts.shape
    assert int(it.min()) >= 1 and int(it.max()) <= R
    idx = (it.long() - 1).unsqueeze(-1)
    stop = torch.gather(ts, 2, idx).squeeze(-1)                        # [B, P]
    assert bool((stop <= bar.unsqueeze(-1)).all())
    nxt = torch.gather(ts, 2, torch.clamp(idx + 1, max=R - 1)).squeeze(-1)
    beyond = (it.long() == R) | (nxt > bar.unsqueeze(-1))
    assert bool(beyond.all())
    assert bool((stop.max(dim=1).values == bar).all())
    assert bool((bar - stop.min(dim=1).values == dm).all())
    first_all = ts[:, :, 0].max(dim=1).values
    assert bool((bar >= first_all).all())
    # never worse than the classic barrier after one iteration of every worker
    lag = torch.searchsorted(ts.contiguous(), first_all.view(B, 1, 1).expand(B, P, 1).contiguous(), right=True).squeeze(-1)
    classic = first_all - torch.gather(ts, 2, (lag - 1).unsqueeze(-1)).squeeze(-1).min(dim=1).values
    assert bool((dm <= classic).all())


@pytest.mark.parametrize("k", [3, 4, 5])
def test_full_size_configs(zl, oracle, k):
    # every instance of the 2 GiB configurations against the oracle
    host = workloads.make(k, threads=16)
    ts = torch.from_numpy(host).cuda()
    bar, it, dm, st = zl.ebsp_zipline_range_batch(ts)
    torch.cuda.synchronize()
    assert int(st.max().item()) == 0
    _properties_hold(ts, bar, it, dm)
    ob, oi, od, rc, _ = oracle.zipline_range(host, "sweep", threads=16)
    assert (rc == 0).all()
    assert np.array_equal(bar.cpu().numpy(), ob), f"barrier differs at {np.nonzero(bar.cpu().numpy() != ob)[0][:5]}"
    assert np.array_equal(dm.cpu().numpy(), od), f"dmin differs at {np.nonzero(dm.cpu().numpy() != od)[0][:5]}"
    assert np.array_equal(it.cpu().numpy(), oi)


def test_value_spread_beyond_32_bits(zl, oracle):
    # keys, successors and the distance back to a worker's previous value no longer fit 32 bits:
    # one workgroup per instance (config 2), windows (configs 3 to 5), a mix of both kinds in one batch
    assert_same(zl, oracle, workloads.make(2, instances=range(64)) * 1000 + EPOCH, "config 2 in ns")
    mixed = workloads.make(2, instances=range(16)).copy()
    mixed[::2] *= 1 << 20
    assert_same(zl, oracle, mixed, "config 2, every other instance x 2^20")
    assert_same(zl, oracle, workloads.make(3, instances=range(6)) * 1000, "config 3 in ns")
    assert_same(zl, oracle, workloads.make(4, instances=range(2)) * 1000, "config 4 in ns")
    assert_same(zl, oracle, workloads.make(5, instances=[0]) * 1000, "config 5 in ns")
    rng = np.random.default_rng(5)
    # every waiting time itself is beyond 2^32: two to five workers with iteration times near 2^33
    for P, R in ((2, 3), (3, 40), (5, 700), (2, 5000)):
        steps = rng.integers(2 ** 33, 2 ** 33 + 2 ** 31, size=(7, P, R), dtype=np.int64)
        assert_same(zl, oracle, np.cumsum(steps, axis=2), f"steps near 2^33, P={P} R={R}")
    # dense stretches far apart: most pieces of 2^32 are empty, some hold more than a workgroup takes
    for P, R in ((8, 600), (64, 512), (300, 100)):
        steps = rng.integers(1, 50, size=(3, P, R), dtype=np.int64)
        steps[:, :, R // 3] += 2 ** 40
        steps[:, :, 2 * R // 3] += 2 ** 34
        steps[:, ::3, R // 2] += 2 ** 36
        assert_same(zl, oracle, np.cumsum(steps, axis=2) - 2 ** 41, f"clusters far apart, P={P} R={R}")
    # the widest values the precondition allows for two workers
    big = np.array([[[0, 2 ** 61, 2 ** 62 - 1], [5, 2 ** 61 + 7, 2 ** 62 - 3]]], dtype=np.int64)
    assert_same(zl, oracle, big, "values up to 2^62")
    assert_same(zl, oracle, big - 2 ** 61, "values from -2^61")
