"""The largest instances the ABI admits (P*R up to just below 2^31), through the C ABI (needs an MI355X).

The oracle would take minutes for one such instance, so the inputs are workers with one common
iteration time, whose answer has a closed form (``closed_forms.same_interval_workers``, itself
checked against every route of the oracle at small sizes in ``test_oracle.py``).  The rows are
built on the device.  Shapes with extreme aspect ratios (a million workers with one iteration, two
workers with a million) are small enough for the oracle and are compared with it.
Bar: bit-exact on all three outputs of all three entry points.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from closed_forms import same_interval_workers  # noqa: E402


@pytest.fixture(scope="module")
def zl():
    assert torch.cuda.is_available(), "these tests need a GPU"
    from paper_2001_01347_amd import zipline
    zipline.load()
    return zipline


def check(label, got, want):
    bar, it, val, st = got
    torch.cuda.synchronize()
    assert int(st[0].item()) == 0, label
    assert (int(bar[0].item()), int(val[0].item())) == want[:2], label
    assert np.array_equal(it[0].cpu().numpy(), want[2]), label


# (P, R): 32-bit crossing indices with byte offsets that still fit 32 bits (P*R just below 2^29);
# P*R = 2^29 exactly (the general window search takes every window); P*R just below 2^31 with many
# rows, with few long rows, and with R itself at 2^31 - 1 (a row scan that counts in steps of a
# wave's width must not wrap there)
@pytest.mark.parametrize("P,R", [(2048, 262143), (8192, 65536), (2048, 1048575), (64, 33554431), (3, 715827882),
                                 (1, 2147483647)])
def test_one_instance_at_the_size_limits(zl, P, R):
    rng = np.random.default_rng(P)
    D = 100_003
    off = rng.choice(D, size=P, replace=False).astype(np.int64)
    want = same_interval_workers(off, D, R)
    epoch = 1_700_000_000_000_000
    want = {k: (v[0] + epoch, v[1], v[2]) for k, v in want.items()}
    off_dev = torch.from_numpy(off).cuda() + epoch
    print(f"P={P} R={R}: predicted rows", flush=True)
    check(f"predicted P={P} R={R}", zl.ebsp_predict_zipline_batch((off_dev - D)[None].contiguous(),
                                                                  torch.full((1, P), D, dtype=torch.int64, device="cuda"), R),
          want["sum"])
    ts = (off_dev[:, None] + torch.arange(R, dtype=torch.int64, device="cuda")[None, :] * D)[None].contiguous()
    print(f"P={P} R={R}: stored rows, summed wait", flush=True)
    check(f"sum P={P} R={R}", zl.ebsp_zipline_batch(ts), want["sum"])
    print(f"P={P} R={R}: stored rows, max(Z) - min(Z)", flush=True)
    check(f"range P={P} R={R}", zl.ebsp_zipline_range_batch(ts), want["range"])
    del ts
    torch.cuda.empty_cache()


def test_shapes_beyond_the_limit_are_refused(zl):
    ts = torch.zeros((1, 4, 4), dtype=torch.int64, device="cuda")
    lib = zl.load()
    p = ts.data_ptr()
    # P*R = 2^31: refused on the host, nothing runs (the pointers are never used)
    assert lib.ebsp_zipline_batch(p, 1, 1 << 16, 1 << 15, p, p, p, None, None, 0, None) == -2
    assert lib.ebsp_zipline_range_batch(p, 1, 1 << 16, 1 << 15, p, p, p, None, None, 0, None) == -2
    assert zl.ebsp_zipline_workspace_bytes(1, 1 << 16, 1 << 15) == 0


@pytest.mark.parametrize("B,P,R", [(1, 1 << 20, 1), (1, 1 << 20, 2), (2, 300000, 3), (1, 65537, 16), (3, 17, 65535),
                                   (3, 17, 65536), (3, 17, 65537), (1, 2, 1 << 20), (5, 1, 100000), (1, 40000, 40)])
def test_extreme_aspect_ratios(zl, oracle, B, P, R):
    # a million workers with one or two iterations each, two workers with a million, R on both sides of
    # the switch from 16- to 32-bit crossing indices: all three entry points against the oracle
    rng = np.random.default_rng(P + R)
    ts = np.cumsum(rng.integers(1, 1000, size=(B, P, R), dtype=np.int64), axis=2) + rng.integers(0, 1000, size=(B, P, 1))
    dev = torch.from_numpy(ts).cuda()
    ob, oi, ow, rc, _ = oracle.zipline(ts, "sweep", threads=16)
    bar, it, w, st = (x.cpu().numpy() for x in zl.ebsp_zipline_batch(dev))
    assert (st == 0).all() and np.array_equal(bar, ob) and np.array_equal(w, ow) and np.array_equal(it, oi)
    ob, oi, od, rc, _ = oracle.zipline_range(ts, "sweep", threads=16)
    bar, it, dm, st = (x.cpu().numpy() for x in zl.ebsp_zipline_range_batch(dev))
    assert (st == 0).all() and np.array_equal(bar, ob) and np.array_equal(dm, od) and np.array_equal(it, oi)
    iv = rng.integers(0, 1000, size=(B, P)).astype(np.int64)
    le = rng.integers(0, 1000, size=(B, P)).astype(np.int64)
    ob, oi, ow, rc, _ = oracle.zipline(oracle.predicted_rows(le, iv, R), "sweep", threads=16)
    bar, it, w, st = (x.cpu().numpy() for x in zl.ebsp_predict_zipline_batch(torch.from_numpy(le).cuda(), torch.from_numpy(iv).cuda(), R))
    assert (st == 0).all() and np.array_equal(bar, ob) and np.array_equal(w, ow) and np.array_equal(it, oi)
