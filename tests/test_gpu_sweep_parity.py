"""The frontier sweep (``zl_sweep_kernel``: stored rows searched in one pass, chosen with
``ebsp_zipline_tune_sweep``) against the CPU oracle, bit for bit, and against the window kernels at full
size.  Needs an MI355X."""
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
    yield zipline
    zipline.ebsp_zipline_tune_sweep(0, 0)


def gpu_run(zl, ts):
    d = torch.from_numpy(np.ascontiguousarray(ts)).cuda()
    out = zl.ebsp_zipline_batch(d)
    torch.cuda.synchronize()
    return [x.cpu().numpy() for x in out]


def assert_same(zl, oracle, ts, label):
    bar, it, w, st = gpu_run(zl, ts)
    ob, oi, ow, rc, _ = oracle.zipline(ts, "sweep", threads=16)
    assert (rc == 0).all() and (st == 0).all(), f"{label}: status {np.unique(st)}"
    assert np.array_equal(bar, ob), f"{label}: barrier differs at {np.nonzero(bar != ob)[0][:5]}"
    assert np.array_equal(w, ow), f"{label}: wait differs at {np.nonzero(w != ow)[0][:5]}"
    assert np.array_equal(it, oi), f"{label}: iters differ at {np.nonzero((it != oi).any(axis=1))[0][:5]}"


@pytest.mark.parametrize("P,R", [(1, 1), (1, 9), (6, 1), (2, 3), (7, 9), (13, 19), (16, 64), (33, 31), (64, 64), (17, 241),
                                 (64, 256), (100, 163), (2048, 1), (1, 20000), (64, 257), (5, 4000), (300, 100), (128, 512),
                                 (1000, 150), (37, 2999), (2048, 16), (3, 70001)])
def test_shapes(zl, oracle, P, R):
    zl.ebsp_zipline_tune_sweep(1, 0)            # every shape through the sweep
    rng = np.random.default_rng(1000 * P + R)
    ts = np.stack([workloads.random_small(rng, P, R, 1, 1000, ties=(i % 2 == 0)) for i in range(4)])
    assert_same(zl, oracle, ts, f"P={P} R={R}")
    assert_same(zl, oracle, ts + EPOCH, f"P={P} R={R} shifted")


def test_degenerate_values(zl, oracle):
    zl.ebsp_zipline_tune_sweep(1, 0)
    assert_same(zl, oracle, np.full((3, 8, 16), 42, dtype=np.int64), "all equal")
    assert_same(zl, oracle, np.full((2, 64, 512), -7, dtype=np.int64), "all equal, larger")
    row = np.cumsum(np.arange(1, 301, dtype=np.int64))
    assert_same(zl, oracle, np.tile(row, (2, 100, 1)), "identical workers")
    rng = np.random.default_rng(5)
    ts = np.stack([workloads.random_small(rng, 40, 300, 1, 1000, ties=True) for _ in range(3)])
    assert_same(zl, oracle, ts * 1_000_003, "steps near 2^30")
    assert_same(zl, oracle, ts * 100_000_007, "steps beyond 2^32")
    c = np.sort(rng.integers(0, 50, size=(2, 30, 400)), axis=2) + (np.arange(400) // 100) * (1 << 40)
    assert_same(zl, oracle, c.astype(np.int64), "dense clusters 2^40 apart")
    c = np.sort(rng.integers(0, 3, size=(2, 200, 300)), axis=2)
    assert_same(zl, oracle, c.astype(np.int64), "three distinct values")


@pytest.mark.parametrize("slice_keys", [256, 1000, 5000, 40000])
def test_results_do_not_depend_on_the_slices(zl, oracle, slice_keys):
    zl.ebsp_zipline_tune_sweep(1, slice_keys)
    rng = np.random.default_rng(slice_keys)
    ts = np.stack([workloads.random_small(rng, 24, 900, 1, 1000, ties=(i == 0)) for i in range(3)])
    assert_same(zl, oracle, ts, f"slice_keys={slice_keys}")
    assert_same(zl, oracle, workloads.make(3, instances=range(8)), f"config 3, slice_keys={slice_keys}")
    assert_same(zl, oracle, workloads.make(4, instances=range(2)), f"config 4, slice_keys={slice_keys}")


def test_unsorted_row_is_flagged(zl):
    zl.ebsp_zipline_tune_sweep(1, 0)
    rng = np.random.default_rng(6)
    ts = np.stack([workloads.random_small(rng, 30, 700, 1, 1000) for _ in range(4)])
    ts[2, 7, 300] = ts[2, 7, 299] - 1
    st = gpu_run(zl, ts)[3]
    assert st[2] & zl.STATUS_UNSORTED and (np.delete(st, 2) == 0).all()


@pytest.mark.parametrize("k", [3, 4, 5])
def test_full_size_configs(zl, oracle, k):
    zl.ebsp_zipline_tune_sweep(8192, 0)
    host = workloads.make(k, threads=16)
    ts = torch.from_numpy(host).cuda()
    bar, it, w, st = zl.ebsp_zipline_batch(ts)
    torch.cuda.synchronize()
    assert int(st.max().item()) == 0
    ob, oi, ow, rc, _ = oracle.zipline(host, "sweep", threads=16)
    assert (rc == 0).all()
    assert np.array_equal(bar.cpu().numpy(), ob) and np.array_equal(w.cpu().numpy(), ow) and np.array_equal(it.cpu().numpy(), oi)
