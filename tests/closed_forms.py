"""Closed forms used by the tests: instances whose answer follows from arithmetic alone."""
import numpy as np


def same_interval_workers(off, D, R):
    """Workers with one common iteration time: t[p][i] = off[p] + i * D, 0 <= off[p] < D, i < R, R >= 3.

    At a candidate c = off[q] + i * D every worker p has waited (off[q] - off[p]) mod D as long as no
    row has ended, whatever i is, so both objectives depend on q alone and the first minimum lies at
    the earliest admissible time of the best q: off[q] itself if it is the largest offset (the
    threshold max_p t[p][0]), else off[q] + D.  With x = off[q]:

        summed wait  = sum_p (x - off[p]) mod D = P * x - sum(off) + D * #{p : off[p] > x}
        max(Z)-min(Z) = max_p (x - off[p]) mod D = x - (smallest off[p] > x) + D, or x - min(off) if none

    Returns {"sum": (barrier, wait, iters[P]), "range": (barrier, dmin, iters[P])}.
    """
    off = np.asarray(off, dtype=np.int64)
    P = off.shape[0]
    assert R >= 3 and off.min() >= 0 and off.max() < D
    srt = np.sort(off)
    above = P - np.searchsorted(srt, off, side="right")                   # workers with a larger offset
    wait = P * off - off.sum() + D * above
    nxt = np.searchsorted(srt, off, side="right")
    dz = np.where(nxt < P, off - srt[np.minimum(nxt, P - 1)] + D, off - srt[0])
    when = np.where(off == off.max(), off, off + D)                       # earliest candidate of each q
    out = {}
    for name, val in (("sum", wait), ("range", dz)):
        best = val.min()
        barrier = when[val == best].min()
        iters = np.minimum((barrier - off) // D + 1, R).astype(np.int32)
        out[name] = (int(barrier), int(best), iters)
    return out
