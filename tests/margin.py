"""Test-side construction of a top-k margin (uses the CPU oracle; never the HIP path).

Natural gaps between the k-th and (k+1)-th largest s_j at D_ff ~ 1e4 are 1e-6..1e-4 relative,
below what fp32-vs-fp64 rounding can resolve, so bit-exact index parity is asserted on inputs
whose boundary gap has been opened to > 2e-3: the W1 rows of the losers just below each
boundary are scaled by 0.98 (and rounded to the storage type again) until every boundary of
every sequence is clear.  The list of (row, factor) pairs is plain data that the input
generator can replay.
"""
from __future__ import annotations

from typing import List, Sequence, Tuple

import numpy as np

import oracle
import synth


def boundary_report(s: np.ndarray, k: int) -> Tuple[float, float]:
    """(relative gap at the k boundary, s_(k))."""
    o = np.sort(s)[::-1]
    if k >= o.shape[0]:
        return float("inf"), float(o[-1])
    return float((o[k - 1] - o[k]) / o[k - 1]), float(o[k - 1])


def open_margin(Xs: Sequence[np.ndarray], Wg, W1: np.ndarray, act: int, dtype: int, ks: Sequence[int],
                bg=None, b1=None, target: float = 2e-3, band: float = 4e-3, factor: float = 0.98,
                max_iter: int = 64, Zs: List[np.ndarray] = None, verbose: bool = False, combine=None):
    """Nudge W1 in place until every (sequence, k) boundary has a relative gap >= target.

    Returns (nudges, s_list): the (row, factor) pairs in application order and the final
    statistic of every sequence.  `Zs` may pass precomputed oracle activations per sequence.
    `combine` maps the list of per-sequence statistics to the list of score vectors whose
    top-k boundaries must be clear (default: the statistics themselves); it is how a batch
    that shares one set (Eq. 7) gets its margin on the shared score.
    """
    F = W1.shape[0]
    if Zs is None:
        Zs = [oracle.ff1(X, Wg, W1, act, bg, b1) for X in Xs]
    nudges: List[Tuple[int, float]] = []
    for it in range(max_iter):
        s_list = [oracle.stat(Z) for Z in Zs]
        rows = set()
        worst = float("inf")
        for s in (combine(s_list) if combine else s_list):
            order = np.argsort(-s, kind="stable")
            for k in ks:
                if k >= F:
                    continue
                sk = s[order[k - 1]]
                gap = (sk - s[order[k]]) / sk
                worst = min(worst, gap)
                if gap < target:
                    t = k
                    while t < F and s[order[t]] > sk * (1.0 - band):
                        rows.add(int(order[t]))
                        t += 1
        if verbose:
            print("  margin iter %d: worst gap %.3e, nudging %d rows" % (it, worst, len(rows)), flush=True)
        if not rows:
            return nudges, s_list
        rows_l = sorted(rows)
        step = [(j, factor) for j in rows_l]
        synth.apply_nudges(W1, step, dtype)
        nudges.extend(step)
        Wg_r = None if Wg is None else Wg[rows_l]
        bg_r = None if bg is None else np.asarray(bg)[rows_l]
        b1_r = None if b1 is None else np.asarray(b1)[rows_l]
        for X, Z in zip(Xs, Zs):
            Z[:, rows_l] = oracle.ff1(X, Wg_r, W1[rows_l], act, bg_r, b1_r)
    raise RuntimeError("top-k margin did not open in %d iterations" % max_iter)
