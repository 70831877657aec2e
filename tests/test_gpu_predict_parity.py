"""Parity of ``ebsp_predict_zipline_batch`` (prediction folded into the search: rows
``last_end + (i + 1) * interval`` that are never stored) with the CPU oracle run on the rows
written out, through the C ABI (needs an MI355X).  Bar: bit-exact on all three outputs.
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


def gpu_run(zl, le, iv, R):
    out = zl.ebsp_predict_zipline_batch(torch.from_numpy(np.ascontiguousarray(le)).cuda(),
                                        torch.from_numpy(np.ascontiguousarray(iv)).cuda(), R)
    torch.cuda.synchronize()
    return tuple(x.cpu().numpy() for x in out)


def assert_same(zl, oracle, le, iv, R, label=""):
    bar, it, w, st = gpu_run(zl, le, iv, R)
    ob, oi, ow, rc, _ = oracle.zipline(oracle.predicted_rows(le, iv, R), "sweep", threads=16)
    assert (rc == 0).all()
    assert (st == 0).all(), f"{label}: status {np.unique(st)}"
    assert np.array_equal(w, ow), f"{label}: wait differs at {np.nonzero(w != ow)[0][:5]}"
    assert np.array_equal(bar, ob), f"{label}: barrier differs at {np.nonzero(bar != ob)[0][:5]}"
    assert np.array_equal(it, oi), f"{label}: iters differ at {np.nonzero((it != oi).any(axis=1))[0][:5]}"


def random_inputs(rng, n, P, lo, hi, ties):
    iv = rng.integers(lo, hi + 1, size=(n, P)).astype(np.int64)
    if ties:
        iv = (iv // 10 + 1) * 10
    le = rng.integers(0, hi, size=(n, P)).astype(np.int64)
    if ties:
        le = le // 10 * 10
    return le, iv


@pytest.mark.parametrize("P,R", [(1, 1), (1, 9), (6, 1), (2, 3), (3, 5), (7, 9), (4, 16), (13, 19), (16, 64),
                                 (64, 64), (64, 256), (100, 163)])
def test_single_workgroup_shapes(zl, oracle, P, R):
    rng = np.random.default_rng(1000 * P + R)
    for ties in (False, True):
        le, iv = random_inputs(rng, 6, P, 1, 1000, ties)
        assert_same(zl, oracle, le, iv, R, f"P={P} R={R} ties={ties}")
        assert_same(zl, oracle, le + EPOCH, iv, R, f"P={P} R={R} shifted")


@pytest.mark.parametrize("P,R", [(1, 16385), (16385, 1), (64, 257), (5, 4000), (300, 100), (128, 512),
                                 (1100, 40), (1024, 64)])
def test_multi_window_shapes(zl, oracle, P, R):
    rng = np.random.default_rng(77 * P + R)
    for ties in (False, True):
        le, iv = random_inputs(rng, 3, P, 1, 1000, ties)
        assert_same(zl, oracle, le + EPOCH, iv, R, f"P={P} R={R} ties={ties}")
        assert_same(zl, oracle, le, iv, R, f"P={P} R={R} ties={ties}, small epoch")
        assert_same(zl, oracle, le - EPOCH, iv, R, f"P={P} R={R} ties={ties}, negative epoch")


def test_all_configurations(zl, oracle):
    for k, ids in ((1, None), (2, range(256)), (3, range(64)), (4, range(6)), (5, range(2))):
        le, iv = workloads.make_predicted(k, instances=ids, shift=EPOCH)
        assert_same(zl, oracle, le, iv, workloads.CONFIGS[k].R, f"config {k}")


def test_same_as_the_stored_path(zl, oracle):
    # the stored-rows entry point on the rows written out must give the very same outputs
    for k, ids in ((2, range(128)), (4, range(4))):
        le, iv = workloads.make_predicted(k, instances=ids)
        R = workloads.CONFIGS[k].R
        bar, it, w, st = gpu_run(zl, le, iv, R)
        ts = torch.from_numpy(oracle.predicted_rows(le, iv, R)).cuda()
        sb, si, sw, ss = zl.ebsp_zipline_batch(ts)
        torch.cuda.synchronize()
        assert np.array_equal(bar, sb.cpu().numpy()) and np.array_equal(w, sw.cpu().numpy())
        assert np.array_equal(it, si.cpu().numpy()) and (st == 0).all()


def test_degenerate_and_wide_inputs(zl, oracle):
    rng = np.random.default_rng(5)
    # zero intervals (all timestamps of a worker equal), identical workers, one very slow worker
    le, iv = random_inputs(rng, 4, 20, 1, 500, False)
    iv[:, ::3] = 0
    assert_same(zl, oracle, le, iv, 40, "zero intervals")
    assert_same(zl, oracle, np.full((2, 64), 7, dtype=np.int64), np.full((2, 64), 13, dtype=np.int64), 512, "identical workers")
    le, iv = random_inputs(rng, 2, 300, 100, 1000, False)
    iv[:, 5] *= 1000
    assert_same(zl, oracle, le, iv, 100, "one worker 1000x slower")
    # spreads of 2^32 and more (nanosecond units): the general search
    le, iv = random_inputs(rng, 3, 16, 1, 1000, True)
    assert_same(zl, oracle, le * 100_000_007, iv * 100_000_007, 64, "wide, single workgroup")
    le, iv = random_inputs(rng, 2, 128, 1, 1000, False)
    assert_same(zl, oracle, le * 100_000_007 + EPOCH, iv * 100_000_007, 512, "wide, multi-window")


def test_negative_interval_is_flagged(zl, oracle):
    for P, R in ((16, 64), (128, 512)):
        rng = np.random.default_rng(P)
        le, iv = random_inputs(rng, 6, P, 1, 1000, False)
        iv[2, 3] = -5
        bar, it, w, st = gpu_run(zl, le, iv, R)
        assert st[2] & zl.STATUS_UNSORTED and (np.delete(st, 2) == 0).all()
        keep = np.delete(np.arange(6), 2)
        ob, oi, ow, rc, _ = oracle.zipline(oracle.predicted_rows(le[keep], iv[keep], R), "sweep", threads=8)
        assert np.array_equal(bar[keep], ob) and np.array_equal(w[keep], ow) and np.array_equal(it[keep], oi)


@pytest.mark.parametrize("k", [3, 4, 5])
def test_full_size_configs(zl, oracle, k):
    # every instance of the 2 GiB shapes against the oracle on the written-out rows (a quarter of the batch at a time)
    cfg = workloads.CONFIGS[k]
    le, iv = workloads.make_predicted(k, shift=EPOCH)
    bar, it, w, st = gpu_run(zl, le, iv, cfg.R)
    assert (st == 0).all()
    for part in np.array_split(np.arange(cfg.B), 4):
        ob, oi, ow, rc, _ = oracle.zipline(oracle.predicted_rows(le[part], iv[part], cfg.R), "sweep", threads=16)
        assert (rc == 0).all()
        assert np.array_equal(bar[part], ob), f"barrier differs at {part[np.nonzero(bar[part] != ob)[0][:5]]}"
        assert np.array_equal(w[part], ow) and np.array_equal(it[part], oi)
    # properties that hold for every instance: each worker stops at its last predicted timestamp <= barrier,
    # the stops sum to the reported wait, some worker stops exactly at the barrier
    stop = le + it.astype(np.int64) * iv
    assert (it >= 1).all() and (it <= cfg.R).all()
    assert (stop <= bar[:, None]).all()
    assert ((it == cfg.R) | (stop + iv > bar[:, None])).all()
    assert (stop.max(axis=1) == bar).all()
    assert ((bar[:, None] - stop).sum(axis=1) == w).all()
