"""Seeded random shapes and value distributions: all three entry points against the oracle, bit for bit."""
import numpy as np
import pytest

from paper_2001_01347_amd import workloads

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def zl():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    from paper_2001_01347_amd import zipline
    zipline.load()
    return zipline


@pytest.fixture(scope="module")
def oracle():
    import oracle as o
    return o


def _instances(rng):
    P = int(rng.choice([1, 2, 3, 5, 8, 16, 33, 64, 100, 256, 300, 512, 1000, 1024, 1500, 2048]))
    R = int(rng.choice([1, 2, 7, 16, 64, 100, 256, 1000, 1024, 4096, 5000]))
    n = P * R
    if n > 2_000_000:
        return None
    B = int(rng.integers(1, 4)) if n > 100_000 else int(rng.integers(1, 30))
    kind = int(rng.integers(0, 5))
    lo, hi = (1, 1000) if kind < 2 else ((0, 3) if kind == 2 else ((1, 50_000) if kind == 3 else (1, 5)))
    steps = rng.integers(lo, hi + 1, size=(B, P, R)).astype(np.int64)
    if kind == 1:                                   # workers of very different speed
        steps *= rng.integers(1, 2000, size=(B, P, 1))
    if kind == 4:                                   # long pauses now and then
        every = max(1, R // 3)
        steps[:, :, ::every] += rng.integers(0, 10_000_000, size=steps[:, :, ::every].shape)
    epoch = int(rng.choice([0, 1_700_000_000_000_000]))
    return np.cumsum(steps, axis=2) + rng.integers(-10 ** 6, 10 ** 6, size=(B, P, 1)) + epoch


@pytest.mark.parametrize("seed", [101, 102, 103])
def test_random_stored_rows_both_objectives(zl, oracle, seed):
    rng = np.random.default_rng(seed)
    done = 0
    while done < 40:
        ts = _instances(rng)
        if ts is None:
            continue
        done += 1
        label = f"seed {seed} case {done} shape {ts.shape}"
        t = torch.from_numpy(ts).cuda()
        bar, it, w, st = (x.cpu().numpy() for x in zl.ebsp_zipline_batch(t))
        ob, oi, ow, rc, _ = oracle.zipline(ts, "sweep", threads=16)
        assert (rc == 0).all() and (st == 0).all(), label
        assert np.array_equal(bar, ob) and np.array_equal(w, ow) and np.array_equal(it, oi), label
        rbar, rit, rd, rst = (x.cpu().numpy() for x in zl.ebsp_zipline_range_batch(t))
        assert (rst == 0).all(), label
        qb, qi, qd, _, _ = oracle.zipline_range(ts, "sweep", threads=16)
        ok = rst == 0
        assert np.array_equal(rbar[ok], qb[ok]) and np.array_equal(rd[ok], qd[ok]) and np.array_equal(rit[ok], qi[ok]), label


@pytest.mark.parametrize("seed", [201, 202])
def test_random_predicted_rows(zl, oracle, seed):
    rng = np.random.default_rng(seed)
    for case in range(40):
        P = int(rng.choice([1, 2, 7, 16, 64, 256, 600, 1024, 2048]))
        R = int(rng.choice([1, 3, 16, 64, 256, 1000, 4096]))
        if P * R > 2_000_000:
            continue
        B = int(rng.integers(1, 4)) if P * R > 100_000 else int(rng.integers(1, 30))
        iv = rng.integers(0 if case % 7 == 0 else 1, int(rng.choice([5, 1000, 300_000])), size=(B, P)).astype(np.int64)
        le = rng.integers(-10 ** 6, 10 ** 7, size=(B, P)).astype(np.int64) + int(rng.choice([0, 1_700_000_000_000_000]))
        label = f"seed {seed} case {case} B={B} P={P} R={R}"
        bar, it, w, st = (x.cpu().numpy() for x in zl.ebsp_predict_zipline_batch(torch.from_numpy(le).cuda(),
                                                                                 torch.from_numpy(iv).cuda(), R))
        ob, oi, ow, rc, _ = oracle.zipline(oracle.predicted_rows(le, iv, R), "sweep", threads=16)
        assert (rc == 0).all() and (st == 0).all(), label
        assert np.array_equal(bar, ob) and np.array_equal(w, ow) and np.array_equal(it, oi), label


@pytest.mark.parametrize("P,R", [(2, 4096), (3, 2731), (5, 1000), (8, 1024), (64, 128), (100, 80), (1000, 8), (4100, 1), (4097, 2), (1, 8192), (1, 4097),
                                 (2, 8192), (3, 5461), (16, 1000), (64, 256), (100, 163), (2000, 8), (8193, 1), (8200, 2), (1, 16384), (1, 8193),
                                 (2, 1024), (3, 700), (64, 32), (33, 100), (1025, 1), (1, 2048), (2, 600), (5, 819), (4096, 1), (1, 1025),
                                 (2, 512), (3, 300), (16, 64), (1000, 1), (1, 1024), (257, 1), (1, 257), (5, 60)])
def test_instances_of_257_to_16384_entries(zl, oracle, P, R):
    """One workgroup each, keys in registers and deltas taken from the neighbouring lane's key (128 threads up to 1024
    entries, 256 up to 4096, 512 up to 8192, 1024 above): the short list of surviving entries is filled in one round where
    most buckets are dropped (many workers) and in several where few are (few workers), stored and predicted rows;
    equal values, a spread above 2^32 and unsorted rows take the exits to the general search."""
    rng = np.random.default_rng(P * 10007 + R)
    B = 12
    steps = rng.integers(1, 2000, size=(B, P, R)).astype(np.int64)
    steps[1] = rng.integers(0, 2, size=(P, R))                       # many equal values
    steps[2] *= 40                                                    # wide
    steps[3, :, R // 2] += 1 << 33                                    # spread above 2^32
    steps[4] = 7                                                      # all rows alike
    ts = np.cumsum(steps, axis=2) + rng.integers(0, 5000, size=(B, P, 1)) + 1_700_000_000_000_000
    if R > 2:
        ts[5, P // 2, 1], ts[5, P // 2, 2] = ts[5, P // 2, 2] + 5, ts[5, P // 2, 1]      # one row out of order
    t = torch.from_numpy(ts).cuda()
    bar, it, w, st = (x.cpu().numpy() for x in zl.ebsp_zipline_batch(t))
    ob, oi, ow, rc, _ = oracle.zipline(ts, "sweep", threads=16)
    ok = rc == 0
    assert np.array_equal(st != 0, rc != 0) and ok.sum() >= B - 1
    assert np.array_equal(bar[ok], ob[ok]) and np.array_equal(w[ok], ow[ok]) and np.array_equal(it[ok], oi[ok])
    iv = rng.integers(1, 3000, size=(B, P)).astype(np.int64)
    iv[1] = 0
    iv[2] = 1 << 22
    le = rng.integers(0, 10 ** 6, size=(B, P)).astype(np.int64)
    bar, it, w, st = (x.cpu().numpy() for x in zl.ebsp_predict_zipline_batch(torch.from_numpy(le).cuda(), torch.from_numpy(iv).cuda(), R))
    ob, oi, ow, rc, _ = oracle.zipline(oracle.predicted_rows(le, iv, R), "sweep", threads=16)
    assert (rc == 0).all() and (st == 0).all()
    assert np.array_equal(bar, ob) and np.array_equal(w, ow) and np.array_equal(it, oi)


@pytest.mark.parametrize("P,R", [(1, 50000), (2, 20000), (3, 30000), (7, 9000), (40, 3000)])
def test_windows_whose_survivors_outnumber_the_list(zl, oracle, P, R):
    """Few workers in the multi-window path: the bounds drop little, so more entries of a window survive than its
    compact list holds (half a window with stored rows) and they are listed and evaluated in rounds; both objectives,
    stored and predicted rows."""
    rng = np.random.default_rng(P * 7919 + R)
    B = 5
    steps = rng.integers(1, 3000, size=(B, P, R)).astype(np.int64)
    steps[1] = 1000                                                    # every worker alike: all candidates tie
    ts = np.cumsum(steps, axis=2) + rng.integers(0, 4000, size=(B, P, 1))
    t = torch.from_numpy(ts).cuda()
    bar, it, w, st = (x.cpu().numpy() for x in zl.ebsp_zipline_batch(t))
    ob, oi, ow, rc, _ = oracle.zipline(ts, "sweep", threads=16)
    assert (rc == 0).all() and (st == 0).all()
    assert np.array_equal(bar, ob) and np.array_equal(w, ow) and np.array_equal(it, oi)
    rbar, rit, rd, rst = (x.cpu().numpy() for x in zl.ebsp_zipline_range_batch(t))
    qb, qi, qd, _, _ = oracle.zipline_range(ts, "sweep", threads=16)
    assert (rst == 0).all() and np.array_equal(rbar, qb) and np.array_equal(rd, qd) and np.array_equal(rit, qi)
    iv = rng.integers(1, 3000, size=(B, P)).astype(np.int64)
    le = rng.integers(0, 10 ** 6, size=(B, P)).astype(np.int64)
    bar, it, w, st = (x.cpu().numpy() for x in zl.ebsp_predict_zipline_batch(torch.from_numpy(le).cuda(), torch.from_numpy(iv).cuda(), R))
    ob, oi, ow, rc, _ = oracle.zipline(oracle.predicted_rows(le, iv, R), "sweep", threads=16)
    assert (rc == 0).all() and (st == 0).all()
    assert np.array_equal(bar, ob) and np.array_equal(w, ow) and np.array_equal(it, oi)
