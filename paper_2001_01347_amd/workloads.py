"""Seeded synthetic inputs for the ZipLine barrier search.

This module only draws random worker timelines; it contains none of the
search's arithmetic and is used by the tests, the smoke check and the
benchmark to feed identical inputs to whatever is being run.

The paper generates its timing data "based on realistic scenarios" without
giving the generator (Section V, "Dataset"), so five synthetic configurations
stand in for it.  One instance is a P x R matrix of predicted iteration end
timestamps in integer microseconds (Section III: the sets S^p of R end
timestamps, Section IV: the n x R matrix M), built as

    t[p][i] = offset_p + sum_{j<=i} d[p][j]

with per-worker mean iteration time mu_p, per-iteration durations d drawn
around mu_p, and a start offset.  All floating-point draws are float64 in
milliseconds, converted with rint(x * 1000) to microseconds; durations are
clamped to >= 1 us so rows are strictly increasing before any rounding.

Every instance b of configuration k has its own generator
``numpy.random.Generator(PCG64(SeedSequence([200101347 * 10 + k, b])))`` so
any subset of instances can be produced without producing the rest.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass
from typing import Iterable, Optional

import numpy as np

SEED_BASE = 200101347 * 10


@dataclass(frozen=True)
class Config:
    """Shape and distribution parameters of one synthetic configuration."""
    k: int
    B: int
    P: int
    R: int
    mu_lo: float            # ms
    mu_hi: float            # ms
    jitter: str             # "lognormal" | "pareto"
    sigma: float            # lognormal sigma, or Pareto jitter scale
    stragglers: int         # number of workers whose mu is scaled by U[1.5, 3]
    bimodal: bool = False   # 80 % U[90,110] ms, 20 % U[200,300] ms
    offset_hi_ms: Optional[float] = None   # None: U[0, mu_p); else U[0, offset_hi_ms)
    round_to_us: int = 1    # every timestamp rounded to a multiple of this

    @property
    def n_keys(self) -> int:
        return self.B * self.P * self.R


CONFIGS = {
    1: Config(1, 1, 4, 8, 80.0, 120.0, "lognormal", 0.1, 0),
    2: Config(2, 4096, 16, 64, 80.0, 120.0, "lognormal", 0.1, 2),
    3: Config(3, 16384, 64, 256, 50.0, 150.0, "lognormal", 0.2, 6),
    4: Config(4, 1024, 256, 1024, 90.0, 110.0, "lognormal", 0.15, 0, bimodal=True,
              round_to_us=1000),
    5: Config(5, 64, 1024, 4096, 20.0, 200.0, "pareto", 0.1, 0, offset_hi_ms=1000.0),
}


def _instance(cfg: Config, b: int) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([SEED_BASE + cfg.k, b])))
    P, R = cfg.P, cfg.R
    if cfg.bimodal:
        slow = rng.random(P) >= 0.8
        mu = np.where(slow, rng.uniform(200.0, 300.0, P), rng.uniform(90.0, 110.0, P))
    else:
        mu = rng.uniform(cfg.mu_lo, cfg.mu_hi, P)
    if cfg.stragglers:
        who = rng.choice(P, size=cfg.stragglers, replace=False)
        mu[who] *= rng.uniform(1.5, 3.0, cfg.stragglers)
    if cfg.jitter == "lognormal":
        d = mu[:, None] * rng.lognormal(0.0, cfg.sigma, (P, R))
    else:  # Pareto type I, alpha = 3, x_m = 1:  X = U^(-1/3), U in (0, 1]
        x = (1.0 - rng.random((P, R))) ** (-1.0 / 3.0)
        d = mu[:, None] * (1.0 + cfg.sigma * x)
    if cfg.offset_hi_ms is None:
        off = rng.random(P) * mu
    else:
        off = rng.random(P) * cfg.offset_hi_ms
    d_us = np.maximum(np.rint(d * 1000.0), 1.0).astype(np.int64)
    t = np.rint(off * 1000.0).astype(np.int64)[:, None] + np.cumsum(d_us, axis=1)
    if cfg.round_to_us > 1:
        q = cfg.round_to_us
        t = ((t + q // 2) // q) * q
    return t


def make(k: int, instances: Optional[Iterable[int]] = None, shift: int = 0,
         threads: int = 8) -> np.ndarray:
    """Timestamps of configuration ``k`` as an int64 array [n, P, R].

    ``instances`` selects instance numbers (default: all B of them, in order);
    ``shift`` is added to every timestamp (e.g. an absolute epoch).
    """
    cfg = CONFIGS[k]
    ids = list(range(cfg.B)) if instances is None else [int(b) for b in instances]
    for b in ids:
        if not 0 <= b < cfg.B:
            raise ValueError(f"instance {b} outside [0, {cfg.B})")
    out = np.empty((len(ids), cfg.P, cfg.R), dtype=np.int64)

    def fill(j: int) -> None:
        out[j] = _instance(cfg, ids[j])
        if shift:
            out[j] += shift

    if threads > 1 and len(ids) > 1:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(fill, range(len(ids)), chunksize=max(1, len(ids) // (threads * 8))))
    else:
        for j in range(len(ids)):
            fill(j)
    return out


def make_predicted(k: int, instances: Optional[Iterable[int]] = None, shift: int = 0):
    """Inputs of the fused prediction for configuration ``k``: ``(last_end[n, P], interval[n, P])`` int64.

    Worker p's interval is its mean iteration time of the configuration (the same
    distribution of means, stragglers and rounding as :func:`make`), its last end
    timestamp the configuration's random offset; the predicted rows are
    ``last_end + (i + 1) * interval``.  Instance ``b`` uses its own seeded stream.
    """
    cfg = CONFIGS[k]
    ids = list(range(cfg.B)) if instances is None else [int(b) for b in instances]
    le = np.empty((len(ids), cfg.P), dtype=np.int64)
    iv = np.empty((len(ids), cfg.P), dtype=np.int64)
    for j, b in enumerate(ids):
        if not 0 <= b < cfg.B:
            raise ValueError(f"instance {b} outside [0, {cfg.B})")
        rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([SEED_BASE + 100 + cfg.k, b])))
        P = cfg.P
        if cfg.bimodal:
            slow = rng.random(P) >= 0.8
            mu = np.where(slow, rng.uniform(200.0, 300.0, P), rng.uniform(90.0, 110.0, P))
        else:
            mu = rng.uniform(cfg.mu_lo, cfg.mu_hi, P)
        if cfg.stragglers:
            who = rng.choice(P, size=cfg.stragglers, replace=False)
            mu[who] *= rng.uniform(1.5, 3.0, cfg.stragglers)
        off = rng.random(P) * (mu if cfg.offset_hi_ms is None else cfg.offset_hi_ms)
        q = max(1, cfg.round_to_us)
        iv[j] = np.maximum((np.rint(mu * 1000.0).astype(np.int64) + q // 2) // q * q, 1)
        le[j] = (np.rint(off * 1000.0).astype(np.int64) + q // 2) // q * q + shift
    return le, iv


def make_supersteps(k: int, S: int, instances: Optional[Iterable[int]] = None, jitter: float = 0.02,
                    shift: int = 0):
    """Inputs of a run of ``S`` supersteps for configuration ``k``: ``(last_end0[n, P], interval[S, n, P])`` int64.

    The workers start at the configuration's random offsets and have its mean iteration times (as
    :func:`make_predicted`); in superstep s a worker's iteration time is its mean times
    ``1 + jitter * N(0, 1)`` (at least 1), drawn per (superstep, worker) from the instance's own
    seeded stream: iteration times of one worker stay similar from one superstep to the next.
    """
    cfg = CONFIGS[k]
    ids = list(range(cfg.B)) if instances is None else [int(b) for b in instances]
    le, mean = make_predicted(k, ids, shift)
    iv = np.empty((int(S), len(ids), cfg.P), dtype=np.int64)
    for j, b in enumerate(ids):
        rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([SEED_BASE + 200 + cfg.k, b])))
        f = 1.0 + float(jitter) * rng.standard_normal((int(S), cfg.P))
        iv[:, j, :] = np.maximum(np.rint(mean[j][None, :] * f).astype(np.int64), 1)
    return le, iv


def make_workers(P: int, R: int, n: int, tag: int = 0) -> np.ndarray:
    """``n`` instances [n, P, R] of any shape, workers as in configuration 2 without its stragglers (mean iteration
    time U[80, 120] ms, durations mu * LogNormal(0, 0.1), start offset U[0, mu)): the shapes of the paper's Table II
    (10 to 1000 workers, 15 and 150 predicted iterations).  Instance b draws from
    ``SeedSequence([SEED_BASE + 300 + tag, P, R, b])``."""
    cfg = Config(0, int(n), int(P), int(R), 80.0, 120.0, "lognormal", 0.1, 0)
    out = np.empty((int(n), int(P), int(R)), dtype=np.int64)
    for b in range(int(n)):
        rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([SEED_BASE + 300 + int(tag), int(P), int(R), b])))
        mu = rng.uniform(cfg.mu_lo, cfg.mu_hi, cfg.P)
        d = mu[:, None] * rng.lognormal(0.0, cfg.sigma, (cfg.P, cfg.R))
        off = rng.random(cfg.P) * mu
        d_us = np.maximum(np.rint(d * 1000.0), 1.0).astype(np.int64)
        out[b] = np.rint(off * 1000.0).astype(np.int64)[:, None] + np.cumsum(d_us, axis=1)
    return out


def random_small(rng: np.random.Generator, P: int, R: int, lo: int = 1, hi: int = 20,
                 ties: bool = False) -> np.ndarray:
    """A small random instance [P, R]: cumulative sums of integer steps in [lo, hi].

    With ``ties`` the steps come from a two-value set, which forces many equal
    timestamps across and within workers.
    """
    if ties:
        steps = rng.choice(np.array([0, lo, hi], dtype=np.int64), size=(P, R))
    else:
        steps = rng.integers(lo, hi + 1, size=(P, R), dtype=np.int64)
    return np.cumsum(steps, axis=1) + rng.integers(0, hi + 1, size=(P, 1), dtype=np.int64)
