"""The synthetic input generator: shapes, determinism and the structure each configuration promises."""
import numpy as np

from paper_2001_01347_amd import workloads


def test_shapes_and_monotone_rows():
    for k, n in [(1, 1), (2, 8), (3, 4), (4, 2), (5, 1)]:
        cfg = workloads.CONFIGS[k]
        ts = workloads.make(k, instances=range(n))
        assert ts.shape == (n, cfg.P, cfg.R) and ts.dtype == np.int64
        assert (np.diff(ts, axis=2) >= 0).all()
        assert ts.min() >= 0


def test_subset_matches_full_and_is_reproducible():
    full = workloads.make(2, instances=range(32))
    again = workloads.make(2, instances=[5, 31, 0], threads=1)
    assert np.array_equal(again[0], full[5]) and np.array_equal(again[1], full[31])
    assert np.array_equal(again[2], full[0])
    assert not np.array_equal(full[0], full[1])


def test_shift_is_added():
    a = workloads.make(1)
    b = workloads.make(1, shift=1_700_000_000_000_000)
    assert np.array_equal(a + 1_700_000_000_000_000, b)


def test_config2_has_two_stragglers_and_config4_has_ties():
    ts = workloads.make(2, instances=range(16))
    mean_iter = np.diff(ts, axis=2).mean(axis=2)          # [n, P] in us
    assert ((mean_iter > 1.35 * 120_000).sum(axis=1) <= 2).all()
    assert ((mean_iter > 125_000).sum(axis=1) >= 1).all()
    t4 = workloads.make(4, instances=[0])[0]
    assert (t4 % 1000 == 0).all()
    assert np.unique(t4).size < 0.9 * t4.size             # rounding to 1 ms forces exact ties


def test_key_ranges_fit_the_documented_bit_budget():
    # per-instance spread (max - min) stays below 2^32 us on every configuration
    for k, n in [(2, 4), (3, 2), (4, 1), (5, 1)]:
        ts = workloads.make(k, instances=range(n))
        spread = ts.reshape(n, -1).max(axis=1) - ts.reshape(n, -1).min(axis=1)
        assert (spread < 2 ** 32).all()


def test_predicted_inputs_are_reproducible():
    le, iv = workloads.make_predicted(3, instances=[5, 9])
    le2, iv2 = workloads.make_predicted(3, instances=[9])
    assert le.shape == iv.shape == (2, 64) and le.dtype == iv.dtype == np.int64
    assert np.array_equal(le[1], le2[0]) and np.array_equal(iv[1], iv2[0])
    assert (iv >= 1).all() and (le >= 0).all()
    shifted, _ = workloads.make_predicted(3, instances=[5], shift=10**15)
    assert np.array_equal(shifted[0], le[0] + 10**15)
    le4, iv4 = workloads.make_predicted(4, instances=[0])
    assert (le4 % 1000 == 0).all() and (iv4 % 1000 == 0).all()      # config 4 rounds to 1 ms


def test_superstep_inputs_are_reproducible_and_stay_near_the_workers_means():
    le, iv = workloads.make_supersteps(3, 6, instances=[5, 9])
    le2, iv2 = workloads.make_supersteps(3, 6, instances=[9])
    base_le, mean = workloads.make_predicted(3, instances=[5, 9])
    assert le.shape == (2, 64) and iv.shape == (6, 2, 64) and iv.dtype == np.int64
    assert np.array_equal(le, base_le)
    assert np.array_equal(le[1], le2[0]) and np.array_equal(iv[:, 1], iv2[:, 0])
    assert (iv >= 1).all()
    assert (np.abs(iv - mean[None]) <= 0.12 * mean[None] + 1).all()          # 2 % jitter: six sigma
    assert not np.array_equal(iv[0], iv[1])                                   # a fresh draw per superstep
    _, flat = workloads.make_supersteps(3, 3, instances=[5], jitter=0.0)
    assert np.array_equal(flat, np.broadcast_to(mean[None, :1], (3, 1, 64)))
