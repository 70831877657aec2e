"""The entry point that allocates nothing (``ebsp_zipline_batch_static``) against ``ebsp_zipline_batch``:
the same kernels on the library's static scratch must give the same results, bit for bit, also when a call
follows a larger one whose contents are still in the scratch.  Called through the C ABI (needs an MI355X)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2001_01347_amd import workloads  # noqa: E402


@pytest.fixture(scope="module")
def zl():
    assert torch.cuda.is_available(), "these tests need a GPU"
    from paper_2001_01347_amd import zipline
    zipline.load()
    return zipline


def _both(zl, host):
    ts = torch.from_numpy(np.ascontiguousarray(host)).cuda()
    B, P, R = ts.shape
    assert 0 < zl.ebsp_zipline_workspace_bytes(B, P, R) <= zl.ebsp_zipline_static_scratch_bytes()   # the scratch is in use
    want = zl.ebsp_zipline_batch(ts)
    torch.cuda.synchronize()
    outs = (torch.full((B,), -1, dtype=torch.int64, device="cuda"), torch.full((B, P), -1, dtype=torch.int32, device="cuda"),
            torch.full((B,), -1, dtype=torch.int64, device="cuda"), torch.full((B,), -1, dtype=torch.int32, device="cuda"))
    before = torch.cuda.memory_allocated()
    got = zl.ebsp_zipline_batch_static(ts, *outs)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    for name, g, w in zip(("barrier", "iters", "wait", "status"), got, want):
        assert torch.equal(g, w), f"{name} differs between the static-scratch call and the workspace call"
    return [x.cpu().numpy() for x in got]


def test_two_calls_in_a_row_the_second_smaller(zl, oracle):
    first = workloads.make(4, instances=range(12))                       # 12 x 256 x 1024: multi-window, ~4 MiB of scratch
    rng = np.random.default_rng(7)
    second = np.stack([workloads.random_small(rng, 96, 300, 1, 1000, ties=(i == 1)) for i in range(3)])   # smaller, other shape
    for host in (first, second):
        bar, it, w, st = _both(zl, host)
        ob, oi, ow, rc, _ = oracle.zipline(host, "sweep", threads=16)
        assert (st == 0).all() and (rc == 0).all()
        assert np.array_equal(bar, ob) and np.array_equal(w, ow) and np.array_equal(it, oi)


def test_a_batch_beyond_the_scratch_is_refused(zl):
    B, P, R = 64, 1024, 4096
    assert zl.ebsp_zipline_workspace_bytes(B, P, R) > zl.ebsp_zipline_static_scratch_bytes()
    ts = torch.zeros((1, 1, 1), dtype=torch.int64, device="cuda")       # never read: the call is refused on its shape
    lib = zl.load()
    rc = lib.ebsp_zipline_batch_static(ts.data_ptr(), B, P, R, ts.data_ptr(), ts.data_ptr(), ts.data_ptr(), None, None)
    assert rc == -3 and "static scratch" in zl.ebsp_last_error()
