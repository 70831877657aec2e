"""Parity of the HIP path with the CPU oracle, through the C ABI (needs an MI355X).

Bar: bit-exact on barrier (int64), wait (int64) and iters (int32) -- the
search is integer work and its result is unique (first minimum, upper-bound
iteration counts), so every output is compared element by element.

Every case is compared in full, the three 2 GiB configurations included: they
are run at full size in the launch configuration the benchmark times, every
instance is compared with the oracle, and on every instance the three outputs
are also checked against properties that hold at any size (each worker stops at its last timestamp <= barrier, the stops sum
to the reported wait, some worker stops exactly at the barrier, and the wait
does not exceed the classic-BSP wait of one iteration per worker).
"""
import json
import os

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2001_01347_amd import workloads  # noqa: E402

EPOCH = 1_700_000_000_000_000   # an absolute microsecond epoch, to exercise large offsets


@pytest.fixture(scope="module")
def zl():
    assert torch.cuda.is_available(), "these tests need a GPU"
    from paper_2001_01347_amd import zipline
    zipline.load()          # raises if the HIP library has not been built
    return zipline


def gpu_run(zl, ts):
    d = torch.from_numpy(np.ascontiguousarray(ts)).cuda()
    bar, it, w, st = zl.ebsp_zipline_batch(d)
    torch.cuda.synchronize()
    return bar.cpu().numpy(), it.cpu().numpy(), w.cpu().numpy(), st.cpu().numpy()


def assert_same(zl, oracle, ts, label=""):
    bar, it, w, st = gpu_run(zl, ts)
    ob, oi, ow, rc, _ = oracle.zipline(ts, "sweep", threads=16)
    assert (rc == 0).all()
    assert (st == 0).all(), f"{label}: status {np.unique(st)}"
    assert np.array_equal(bar, ob), f"{label}: barrier differs at {np.nonzero(bar != ob)[0][:5]}"
    assert np.array_equal(w, ow), f"{label}: wait differs at {np.nonzero(w != ow)[0][:5]}"
    assert np.array_equal(it, oi), f"{label}: iters differ at {np.nonzero((it != oi).any(axis=1))[0][:5]}"


def test_hand_worked_examples(zl, oracle):
    path = os.path.join(os.path.dirname(__file__), "golden", "worked_examples.json")
    for c in json.load(open(path))["cases"]:
        bar, it, w, st = gpu_run(zl, np.array([c["t"]], dtype=np.int64))
        assert (int(bar[0]), int(w[0]), list(it[0]), int(st[0])) == (c["barrier"], c["wait"], c["iters"], 0)


def test_config1_and_config2_full(zl, oracle):
    assert_same(zl, oracle, workloads.make(1), "config 1")
    assert_same(zl, oracle, workloads.make(2), "config 2")
    assert_same(zl, oracle, workloads.make(2, instances=range(512), shift=EPOCH), "config 2 shifted")


@pytest.mark.parametrize("P,R", [(1, 1), (1, 9), (6, 1), (2, 3), (3, 5), (7, 9), (4, 16), (13, 19),
                                 (16, 64), (33, 31), (64, 64), (50, 81), (17, 241), (64, 256),
                                 (100, 163), (128, 128), (16384, 1), (1, 16384)])
def test_single_workgroup_shapes(zl, oracle, P, R):
    rng = np.random.default_rng(1000 * P + R)
    ts = np.stack([workloads.random_small(rng, P, R, 1, 1000, ties=(i % 2 == 0)) for i in range(6)])
    assert_same(zl, oracle, ts, f"P={P} R={R}")
    assert_same(zl, oracle, ts + EPOCH, f"P={P} R={R} shifted")
    assert_same(zl, oracle, ts - 5_000_000, f"P={P} R={R} negative")


@pytest.mark.parametrize("P,R", [(1, 16385), (16385, 1), (64, 257), (5, 4000), (300, 100), (128, 512),
                                 (1000, 150), (37, 2999), (2048, 16), (3, 70001)])
def test_multi_window_shapes(zl, oracle, P, R):
    rng = np.random.default_rng(77 * P + R)
    ts = np.stack([workloads.random_small(rng, P, R, 1, 1000, ties=(i % 2 == 0)) for i in range(3)])
    assert_same(zl, oracle, ts, f"P={P} R={R}")
    assert_same(zl, oracle, ts + EPOCH, f"P={P} R={R} shifted")


@pytest.mark.parametrize("P,R", [(40, 60000), (600, 7100), (64, 70000)])
def test_more_fine_bins_than_the_plan_holds_in_lds(zl, oracle, P, R):
    # above 4096 fine bins per instance the windows are packed by the sequential walk; above 8200
    # (the last shape, which also needs 32-bit crossing indices) the bins are counted from the whole table
    assert zl.ebsp_zipline_shape_info(2, P, R)["bins"] > (8200 if R > 65535 else 4096)
    rng = np.random.default_rng(P + R)
    ts = np.stack([workloads.random_small(rng, P, R, 1, 1000, ties=(i == 1)) for i in range(2)])
    assert_same(zl, oracle, ts, f"P={P} R={R}")


def test_results_do_not_depend_on_the_tuning_knobs(zl, oracle):
    ts = workloads.make(4, instances=range(4))
    try:
        for cap, single, fill in [(0, 0, 0), (0, 0, 700), (8192, 0, 5000), (16384, 0, 0), (4096, 4096, 3000)]:
            zl.ebsp_zipline_tune(cap, single, fill)
            assert_same(zl, oracle, ts, f"tune {cap} {single} {fill}")
            small = workloads.make(3, instances=range(8))
            assert_same(zl, oracle, small, f"tune {cap} {single} {fill} config 3")
    finally:
        zl.ebsp_zipline_tune(0, 0, 0)


def test_degenerate_values(zl, oracle):
    # all timestamps equal; all workers identical; one giant tie at the optimum
    assert_same(zl, oracle, np.full((3, 8, 16), 42, dtype=np.int64), "all equal")
    assert_same(zl, oracle, np.full((2, 64, 512), -7, dtype=np.int64), "all equal, multi-window")
    row = np.cumsum(np.arange(1, 301, dtype=np.int64))
    assert_same(zl, oracle, np.tile(row, (2, 100, 1)), "identical workers")
    t = np.tile(np.arange(1, 65, dtype=np.int64) * 10, (1, 40, 1))
    t[0, :, 63] = 1000
    assert_same(zl, oracle, t, "tie at the end")


@pytest.mark.parametrize("P,R", [(8, 2048), (4, 1024), (16, 4096), (600, 64)])
def test_equal_minima_far_apart(zl, oracle, P, R):
    # workers of one period T, evenly staggered: after the first period every arrival gives
    # the same wait g*P*(P-1)/2, so the minimum is attained in every bucket and every window;
    # worker 0 joins k periods late, which makes all earlier candidates inadmissible.
    # The earliest admissible minimum must win: the barrier is worker 0's first timestamp.
    g, k = 7, R // 3
    T = P * g
    i = np.arange(R, dtype=np.int64)
    t = np.stack([p * g + i * T for p in range(P)])
    t[0] = (i + k) * T
    ts = np.stack([t, t + 3, t * 1000 + EPOCH])          # the last one: spread >= 2^32 for the larger shapes
    bar, it, w, st = gpu_run(zl, ts)
    assert (st == 0).all()
    assert list(bar) == [k * T, k * T + 3, k * T * 1000 + EPOCH]
    assert list(w[:2]) == [g * P * (P - 1) // 2] * 2 and int(w[2]) == 1000 * g * P * (P - 1) // 2
    assert_same(zl, oracle, ts, f"staggered P={P} R={R}")


def test_wide_value_ranges(zl, oracle):
    # per-instance spread of 2^32 units or more (e.g. nanosecond timestamps): deltas need 64 bits
    rng = np.random.default_rng(8)
    for P, R in [(3, 5), (16, 64), (64, 256), (50, 81)]:
        ts = np.stack([workloads.random_small(rng, P, R, 1, 1000, ties=(i % 2 == 0)) for i in range(4)])
        assert_same(zl, oracle, ts * 100_000_007, f"wide P={P} R={R}")
        assert_same(zl, oracle, ts * (1 << 36) - EPOCH, f"very wide P={P} R={R}")
    assert_same(zl, oracle, workloads.make(3, instances=range(8)) * 1000, "config 3 in ns")
    for P, R in [(64, 257), (128, 512), (5, 4000)]:
        ts = np.stack([workloads.random_small(rng, P, R, 1, 1000, ties=(i % 2 == 0)) for i in range(2)])
        assert_same(zl, oracle, ts * 100_000_007 + EPOCH, f"wide multi-window P={P} R={R}")
    assert_same(zl, oracle, workloads.make(4, instances=range(2)) * 1000, "config 4 in ns")
    # mixed batch: narrow and wide instances side by side
    m = workloads.make(2, instances=range(6)).copy()
    m[1] *= 5000
    m[4] *= 1 << 30
    assert_same(zl, oracle, m, "mixed widths")


def test_skewed_and_clustered_values(zl, oracle):
    # one worker 1000x slower stretches the value range: nearly all keys share a few fine bins
    t = workloads.make(4, instances=range(2)).copy()
    t[:, 7, :] = t[:, 7, :1] + (t[:, 7, :] - t[:, 7, :1]) * 1000
    assert_same(zl, oracle, t, "straggler x1000")
    # a handful of distinct values, each far more frequent than one window can hold
    rng = np.random.default_rng(12)
    few = np.sort(rng.integers(0, 4, size=(2, 64, 1024)), axis=2).astype(np.int64) * 1_000_003
    assert_same(zl, oracle, few, "four distinct values")
    # dense cluster + sparse tail: 40000 keys within 50000 units, then one far outlier row end
    c = np.sort(rng.integers(0, 50_000, size=(1, 40, 1000)), axis=2).astype(np.int64)
    c[0, 0, -1] = 10 ** 12
    assert_same(zl, oracle, c, "cluster and outlier")


def test_rows_far_from_evenly_spaced(zl, oracle):
    # the fine bins are laid out as if every row were evenly spaced between its first and last value:
    # rows that are not only make the bins uneven (oversize windows go to the general search)
    rng = np.random.default_rng(5)
    t = workloads.make(4, instances=range(2)).copy()
    t[:, :, 512:] += 3_000_000_000                          # every worker pauses for 50 minutes half way
    assert_same(zl, oracle, t, "a long pause")
    u = workloads.make(4, instances=range(2)).copy()
    u[:, ::2, 100:] += 500_000_000                          # half of the workers pause early
    u[:, 1::2, 900:] += 900_000_000                         # the others late
    assert_same(zl, oracle, u, "staggered pauses")
    # quadratic rows: iterations slow down steadily
    i = np.arange(700, dtype=np.int64)
    q = (rng.integers(0, 1000, size=(2, 300, 1)) + i * 1000 + (i * i) * rng.integers(1, 40, size=(2, 300, 1))).astype(np.int64)
    assert_same(zl, oracle, q, "slowing workers")


def test_status_flags(zl, oracle):
    ts = workloads.make(2, instances=range(8)).copy()
    ts[3, 5, 10] = ts[3, 5, 9] - 1                      # one row of one instance goes backwards
    bar, it, w, st = gpu_run(zl, ts)
    assert st[3] & zl.STATUS_UNSORTED and (np.delete(st, 3) == 0).all()
    ob, oi, ow, rc, _ = oracle.zipline(ts)
    keep = rc == 0
    assert rc[3] == 1 and keep.sum() == 7
    assert np.array_equal(bar[keep], ob[keep]) and np.array_equal(w[keep], ow[keep])
    assert np.array_equal(it[keep], oi[keep])
    # P * range beyond int64: flagged, no fault
    big = np.zeros((1, 4, 4), dtype=np.int64)
    big[0, :, :] = np.array([0, 1, 2, 2 ** 62], dtype=np.int64)
    _, _, _, st = gpu_run(zl, big)
    assert st[0] & zl.STATUS_OVERFLOW
    # same in the multi-window path
    m = workloads.make(4, instances=range(3)).copy()
    m[1, 200, 500] = m[1, 200, 400]
    bar, it, w, st = gpu_run(zl, m)
    assert st[1] & zl.STATUS_UNSORTED and st[0] == 0 and st[2] == 0
    ob, oi, ow, rc, _ = oracle.zipline(m)
    for b in (0, 2):
        assert (bar[b], w[b]) == (ob[b], ow[b]) and np.array_equal(it[b], oi[b])


def test_empty_batch_and_reuse_of_buffers(zl, oracle):
    d = torch.zeros((0, 4, 8), dtype=torch.int64, device="cuda")
    bar, it, w, st = zl.ebsp_zipline_batch(d)
    assert bar.numel() == 0 and it.shape == (0, 4)
    # caller-owned outputs and workspace, two different batches through the same buffers
    a = workloads.make(4, instances=range(4))
    b = workloads.make(4, instances=range(4, 8))
    outs = None
    ws = torch.empty(zl.ebsp_zipline_workspace_bytes(4, 256, 1024), dtype=torch.uint8, device="cuda")
    for ts in (a, b, a):
        d = torch.from_numpy(ts).cuda()
        outs = zl.ebsp_zipline_batch(d, *(outs or (None, None, None, None)), workspace=ws)
        torch.cuda.synchronize()
        ob, oi, ow, _, _ = oracle.zipline(ts)
        assert np.array_equal(outs[0].cpu().numpy(), ob) and np.array_equal(outs[2].cpu().numpy(), ow)
        assert np.array_equal(outs[1].cpu().numpy(), oi)


def test_deterministic_and_stream(zl):
    ts = torch.from_numpy(workloads.make(4, instances=range(6))).cuda()
    first = [x.clone() for x in zl.ebsp_zipline_batch(ts)]
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        second = zl.ebsp_zipline_batch(ts)
    s.synchronize()
    torch.cuda.synchronize()
    for x, y in zip(first, second):
        assert torch.equal(x, y)


def _properties_hold(ts_dev, bar, it, w):
    B, P, R = ts_dev.shape
    idx = (it.long() - 1).clamp(0, R - 1).unsqueeze(2)
    stop = torch.gather(ts_dev, 2, idx).squeeze(2)                       # t[p][iters-1]
    nxt_idx = it.long().clamp(0, R - 1).unsqueeze(2)
    nxt = torch.gather(ts_dev, 2, nxt_idx).squeeze(2)
    assert bool(((it >= 1) & (it <= R)).all())
    assert bool((stop <= bar[:, None]).all())
    assert bool(((nxt > bar[:, None]) | (it == R)).all())
    assert bool(((bar[:, None] - stop).sum(dim=1) == w).all())
    assert bool((stop.max(dim=1).values == bar).all())                   # the barrier is a timestamp
    first = ts_dev[:, :, 0]
    assert bool((bar >= first.max(dim=1).values).all())
    assert bool((w <= (first.max(dim=1, keepdim=True).values - first).sum(dim=1)).all())
    assert bool((w >= 0).all())


@pytest.mark.parametrize("k", [3, 4, 5])
def test_full_size_configs(zl, oracle, k):
    # every instance of the 2 GiB configurations against the oracle, in the launch configuration the benchmark times
    host = workloads.make(k, threads=16)
    ts = torch.from_numpy(host).cuda()
    bar, it, w, st = zl.ebsp_zipline_batch(ts)
    torch.cuda.synchronize()
    assert int(st.max().item()) == 0
    _properties_hold(ts, bar, it, w)
    ob, oi, ow, rc, _ = oracle.zipline(host, "sweep", threads=16)
    assert (rc == 0).all()
    assert np.array_equal(bar.cpu().numpy(), ob), f"barrier differs at {np.nonzero(bar.cpu().numpy() != ob)[0][:5]}"
    assert np.array_equal(w.cpu().numpy(), ow), f"wait differs at {np.nonzero(w.cpu().numpy() != ow)[0][:5]}"
    assert np.array_equal(it.cpu().numpy(), oi)


def test_shifted_epoch_multi_window(zl, oracle):
    assert_same(zl, oracle, workloads.make(5, instances=[0, 63], shift=EPOCH), "config 5 shifted")
    assert_same(zl, oracle, workloads.make(4, instances=range(16), shift=EPOCH), "config 4 shifted")
    assert_same(zl, oracle, workloads.make(3, instances=range(64), shift=-EPOCH), "config 3 shifted")


def all_three(zl, oracle, ts, label):
    """Summed wait and max(Z) - min(Z) on stored rows against their oracles."""
    assert_same(zl, oracle, ts, label)
    d = torch.from_numpy(np.ascontiguousarray(ts)).cuda()
    bar, it, dm, st = (x.cpu().numpy() for x in zl.ebsp_zipline_range_batch(d))
    ob, oi, od, rc, _ = oracle.zipline_range(ts, "sweep", threads=16)
    assert (rc == 0).all() and (st == 0).all(), label
    assert np.array_equal(bar, ob) and np.array_equal(dm, od) and np.array_equal(it, oi), f"{label}: range objective"


def test_values_at_the_ends_of_int64(zl, oracle):
    # all arithmetic is relative to the instance's smallest value, modulo 2^64: the epoch may sit anywhere
    rng = np.random.default_rng(64)
    lo, hi = np.iinfo(np.int64).min, np.iinfo(np.int64).max
    for P, R in [(3, 5), (16, 64), (100, 163), (64, 257), (300, 100)]:
        ts = np.stack([workloads.random_small(rng, P, R, 1, 1000, ties=(i % 2 == 0)) for i in range(3)])
        ts -= ts.min()
        all_three(zl, oracle, ts + lo, f"from INT64_MIN, P={P} R={R}")
        all_three(zl, oracle, ts + (hi - ts.max()), f"up to INT64_MAX, P={P} R={R}")
        all_three(zl, oracle, ts - ts.max() // 2, f"around zero, P={P} R={R}")
        # predicted rows ending exactly at INT64_MAX
        iv = rng.integers(1, 1000, size=(3, P)).astype(np.int64)
        le = hi - R * iv - rng.integers(0, 3, size=(3, P)) * (iv != iv.max(axis=1, keepdims=True))
        got = tuple(x.cpu().numpy() for x in zl.ebsp_predict_zipline_batch(torch.from_numpy(le).cuda(), torch.from_numpy(iv).cuda(), R))
        ob, oi, ow, rc, _ = oracle.zipline(oracle.predicted_rows(le, iv, R), "sweep", threads=8)
        assert (got[3] == 0).all() and (rc == 0).all()
        assert np.array_equal(got[0], ob) and np.array_equal(got[2], ow) and np.array_equal(got[1], oi), f"predicted up to INT64_MAX, P={P} R={R}"


def test_very_many_instances(zl, oracle):
    # a million tiny instances (one workgroup each) and twelve thousand that are cut into windows
    rng = np.random.default_rng(1_000_000)
    steps = rng.integers(1, 50, size=(1_000_000, 3, 5), dtype=np.int64)
    all_three(zl, oracle, np.cumsum(steps, axis=2) + rng.integers(0, 50, size=(1_000_000, 3, 1)), "B = 10^6, P=3 R=5")
    steps = rng.integers(1, 2000, size=(12_000, 300, 100), dtype=np.int64)
    all_three(zl, oracle, np.cumsum(steps, axis=2) + rng.integers(0, 2000, size=(12_000, 300, 1)), "B = 12000, P=300 R=100")


@pytest.mark.parametrize("k,n", [(4, 64), (5, 4)])
def test_the_fast_kernels_take_the_configurations(zl, k, n):
    # On the synthetic configurations next to nothing is left to the general (sort-based) kernels.
    # They are correct too, so only their share of the time shows whether the windows are planned
    # as intended: a plan with surplus or oversize windows would still pass every parity test.
    ts = torch.from_numpy(workloads.make(k, instances=range(n))).cuda()
    for call, fast, general in ((zl.ebsp_zipline_batch, "zl_window_kernel", "zl_window_general_kernel"),
                                (zl.ebsp_zipline_range_batch, "zl_range_fast_kernel", "zl_range_window_kernel")):
        call(ts)
        torch.cuda.synchronize()
        zl.ebsp_zipline_profile_begin(3)
        for _ in range(3):
            out = call(ts)
        ms, calls = zl.ebsp_zipline_profile_end()
        assert calls == 3 and int(out[3].max().item()) == 0
        assert ms[general] < 0.5 * ms[fast], f"config {k}: {general} {ms[general]:.3f} ms against {fast} {ms[fast]:.3f} ms"


def test_host_threads_with_their_own_streams_and_workspaces(zl, oracle):
    # the header's promise: calls on different streams may overlap if they use different workspaces.
    # Four host threads, each with a stream, a workspace and a workload of its own (two of them
    # multi-window), call all three entry points twenty times over while the others do the same.
    import threading
    jobs = []
    for k, n in ((2, 256), (3, 24), (4, 6), (5, 1)):
        cfg = workloads.CONFIGS[k]
        ts = workloads.make(k, instances=range(n))
        le, iv = workloads.make_predicted(k, instances=range(n))
        want = (oracle.zipline(ts, "sweep", threads=16)[:3], oracle.zipline_range(ts, "sweep", threads=16)[:3],
                oracle.zipline(oracle.predicted_rows(le, iv, cfg.R), "sweep", threads=16)[:3])
        jobs.append((cfg, torch.from_numpy(ts).cuda(), torch.from_numpy(le).cuda(), torch.from_numpy(iv).cuda(), want))
    torch.cuda.synchronize()
    errors = []

    def work(job):
        cfg, ts, le, iv, want = job
        try:
            stream = torch.cuda.Stream()
            with torch.cuda.stream(stream):
                for rep in range(20):
                    got = (zl.ebsp_zipline_batch(ts), zl.ebsp_zipline_range_batch(ts), zl.ebsp_predict_zipline_batch(le, iv, cfg.R))
                    stream.synchronize()
                    for (bar, it, val, st), (ob, oi, ov) in zip(got, want):
                        if not ((st == 0).all().item() and np.array_equal(bar.cpu().numpy(), ob)
                                and np.array_equal(val.cpu().numpy(), ov) and np.array_equal(it.cpu().numpy(), oi)):
                            errors.append(f"config {cfg.k}, repetition {rep}")
        except Exception as e:          # noqa: BLE001
            errors.append(f"config {cfg.k}: {e!r}")

    threads = [threading.Thread(target=work, args=(j,)) for j in jobs]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors[:5]


def test_status_may_be_null(zl, oracle):
    # the C ABI takes NULL for status on every entry point (the binding always passes an array)
    lib = zl.load()
    for k, n in ((2, 64), (4, 3)):                       # one workgroup per instance; windows
        cfg = workloads.CONFIGS[k]
        host = workloads.make(k, instances=range(n))
        le_h, iv_h = workloads.make_predicted(k, instances=range(n))
        ts, le, iv = (torch.from_numpy(x).cuda() for x in (host, le_h, iv_h))
        bar = torch.empty(n, dtype=torch.int64, device="cuda")
        it = torch.empty((n, cfg.P), dtype=torch.int32, device="cuda")
        val = torch.empty(n, dtype=torch.int64, device="cuda")
        need = max(zl.ebsp_zipline_workspace_bytes(n, cfg.P, cfg.R), zl.ebsp_zipline_range_workspace_bytes(n, cfg.P, cfg.R),
                   zl.ebsp_simulate_workspace_bytes(n, cfg.P, cfg.R))
        ws = torch.empty(need, dtype=torch.uint8, device="cuda")
        stream = torch.cuda.current_stream().cuda_stream

        def same(want):
            torch.cuda.synchronize()
            return (np.array_equal(bar.cpu().numpy(), want[0]) and np.array_equal(it.cpu().numpy(), want[1])
                    and np.array_equal(val.cpu().numpy(), want[2]))

        assert lib.ebsp_zipline_batch(ts.data_ptr(), n, cfg.P, cfg.R, bar.data_ptr(), it.data_ptr(), val.data_ptr(), None,
                                      ws.data_ptr(), need, stream) == 0
        assert same(oracle.zipline(host, "sweep", threads=8))
        assert lib.ebsp_zipline_range_batch(ts.data_ptr(), n, cfg.P, cfg.R, bar.data_ptr(), it.data_ptr(), val.data_ptr(), None,
                                            ws.data_ptr(), need, stream) == 0
        assert same(oracle.zipline_range(host, "sweep", threads=8))
        assert lib.ebsp_predict_zipline_batch(le.data_ptr(), iv.data_ptr(), n, cfg.P, cfg.R, bar.data_ptr(), it.data_ptr(),
                                              val.data_ptr(), None, ws.data_ptr(), need, stream) == 0
        want = oracle.zipline(oracle.predicted_rows(le_h, iv_h, cfg.R), "sweep", threads=8)
        assert same(want)
        assert lib.ebsp_simulate_supersteps(le.data_ptr(), iv.data_ptr(), 0, 1, n, cfg.P, cfg.R, bar.data_ptr(), it.data_ptr(),
                                            val.data_ptr(), None, ws.data_ptr(), need, stream) == 0
        assert same(want)                                  # one superstep is one predicted search


@pytest.mark.parametrize("P,R", [(256, 240), (1024, 240)])
def test_nanosecond_timestamps_at_the_papers_scales(zl, oracle, P, R):
    # iteration times of 80-120 ms in nanoseconds: the instance's spread passes 2^32, its windows and the
    # steps of its rows do not, so the fast window search takes all but the last windows, where only the
    # slowest workers are left and a window is itself wider than 2^32 ns
    rng = np.random.default_rng(P)
    B = 6
    mean = rng.integers(80_000_000, 120_000_000, size=(B, P, 1))
    steps = (mean * (1.0 + 0.05 * rng.standard_normal((B, P, R)))).astype(np.int64)
    ts = np.cumsum(steps, axis=2) + rng.integers(0, 100_000_000, size=(B, P, 1)) + EPOCH * 1000
    assert ((ts.max(axis=(1, 2)) - ts.min(axis=(1, 2))) >> 32).all()
    assert_same(zl, oracle, ts, f"ns, P={P} R={R}")
    all_three(zl, oracle, ts[:2], f"ns, P={P} R={R}, both objectives")


@pytest.mark.parametrize("pauses", [1, 3, 15, 16, 40])
def test_a_few_long_pauses_in_nanosecond_rows(zl, oracle, pauses):
    # an instance in nanoseconds whose rows step by less than 2^32 except for a few pauses of 2^33 and more:
    # only the windows such a step ends in are left to the general search (up to 15 of them are remembered
    # per instance; with more the whole instance is), and the result must not change either way
    rng = np.random.default_rng(pauses)
    B, P, R = 3, 600, 400
    steps = rng.integers(80_000_000, 120_000_000, size=(B, P, R)).astype(np.int64)
    for b in range(B):
        for _ in range(pauses):
            steps[b, rng.integers(0, P), rng.integers(1, R)] += int(rng.integers(2 ** 33, 2 ** 34))
    ts = np.cumsum(steps, axis=2) + rng.integers(0, 100_000_000, size=(B, P, 1))
    all_three(zl, oracle, ts, f"{pauses} pauses")
    # the same pauses at the very first step of a row (its first entry stays early, the second comes late)
    steps[:, :4, 1] += 2 ** 35
    all_three(zl, oracle, np.cumsum(steps, axis=2), f"{pauses} pauses and four early ones")


@pytest.mark.parametrize("nbytes", [16, 4096 + 16, 16 * 1024 * 3 + 48, 8 * 1024 * 1024, 64 * 1024 * 1024 + 16 * 7])
def test_the_yardstick_kernels_copy_and_read_everything(zl, nbytes):
    # the copy probe copies every byte, the read probe sums every 32-bit word (pieces per workgroup, ragged ends)
    g = torch.Generator(device="cuda").manual_seed(nbytes)
    src = torch.randint(0, 1 << 31, (nbytes // 4,), dtype=torch.int32, device="cuda", generator=g)
    dst = torch.zeros_like(src)
    sink = torch.zeros(zl.READ_SINK_WORDS, dtype=torch.int64, device="cuda")
    zl.ebsp_zipline_copy_probe(src, dst)
    zl.ebsp_zipline_read_probe(src, sink)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)
    assert int(sink.sum().item()) == int(src.to(torch.int64).sum().item())
    with pytest.raises(ValueError):
        zl.ebsp_zipline_read_probe(src, sink[:1])
