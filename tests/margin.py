"""Test-side construction of a top-k margin (uses the CPU oracle; never the HIP path).

Natural gaps between the k-th and (k+1)-th largest s_j at D_ff ~ 1e4 are 1e-6..1e-4 relative,
below what fp32-vs-fp64 rounding can resolve, so bit-exact index parity is asserted on inputs
whose boundary gap has been opened to > 2e-3.  For every boundary that is too tight a window of
that relative width is laid over it where it holds the fewest neurons; the W1 rows of the neurons
inside are scaled (winners up, losers down, re-rounded to the storage type) by the smallest factor
of a ladder that is predicted to carry them clear of the window AND clear of every other boundary
of every other sequence that shares the weights (s_j is close to linear in the scale of row j and
independent of the other rows), so that opening one boundary does not close another.  What the
rounding to bf16 makes of a factor is only roughly the factor, so the statistic is recomputed by
the oracle and the step repeated until every boundary is clear.  The list of (row, factor) pairs is
plain data that the input generator replays.
"""
from __future__ import annotations

from typing import List, Sequence, Tuple

import numpy as np

import oracle
import synth

# scale factors tried in this order, winners (up) and losers (down); the first whose predicted
# position is clear of every boundary is taken
_UP = (1.006, 1.01, 1.015, 1.02, 1.03, 1.04, 1.06)
_DOWN = (0.994, 0.99, 0.985, 0.98, 0.97, 0.96, 0.94)


def boundary_report(s: np.ndarray, k: int) -> Tuple[float, float]:
    """(relative gap at the k boundary, s_(k))."""
    o = np.sort(s)[::-1]
    if k >= o.shape[0]:
        return float("inf"), float(o[-1])
    return float((o[k - 1] - o[k]) / o[k - 1]), float(o[k - 1])


def _window(desc: np.ndarray, k: int, width: float) -> Tuple[float, float]:
    """Interval (lo, hi) with hi = lo / (1 - width) that separates rank k from rank k+1 of the
    descending scores and holds as few other scores as possible."""
    a, b = desc[k - 1], desc[k]              # k-th and (k+1)-th largest
    asc = desc[::-1]
    best = None
    for lo in np.linspace(a * (1.0 - width), min(b, a * (1.0 - width * 1e-3)), 9):
        hi = lo / (1.0 - width)
        inside = np.searchsorted(asc, hi, side="left") - np.searchsorted(asc, lo, side="right")
        if best is None or inside < best[0]:
            best = (inside, lo, hi)
    return best[1], best[2]


def open_margin(Xs: Sequence[np.ndarray], Wg, W1: np.ndarray, act: int, dtype: int, ks: Sequence[int],
                bg=None, b1=None, target: float = 2e-3, max_iter: int = 64, Zs: List[np.ndarray] = None,
                verbose: bool = False, combine=None):
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
    width = 1.2 * target                     # what a step aims for; the loop ends on the real gap
    pad = 1.5 * target                       # distance kept from boundaries, beyond the window
    for it in range(max_iter):
        s_list = [oracle.stat(Z) for Z in Zs]
        scores = [np.asarray(s, dtype=np.float64) for s in (combine(s_list) if combine else s_list)]
        worst = float("inf")
        zones = []                           # (score index, lo, hi): where no score may end up
        todo = []                            # (score index, k, lo, hi) of the boundaries still too tight
        for c, s in enumerate(scores):
            desc = np.sort(s)[::-1]
            for k in ks:
                if k >= F or not desc[k - 1] > 0.0:
                    continue
                a, b = desc[k - 1], desc[k]
                gap = (a - b) / a
                worst = min(worst, gap)
                if gap >= target:
                    zones.append((c, b, a))
                else:
                    lo, hi = _window(desc, k, width)
                    zones.append((c, lo, hi))
                    todo.append((c, k, lo, hi))
        if verbose:
            print("  margin iter %d: worst gap %.3e, %d boundaries to open" % (it, worst, len(todo)), flush=True)
        if not todo:
            return nudges, s_list
        moves = {}                           # row -> +1 (up) / -1 (down); a row asked both ways goes down
        for c, k, lo, hi in todo:
            s = scores[c]
            winner = np.zeros(F, dtype=bool)
            winner[np.argsort(-s, kind="stable")[:k]] = True
            # winners below the upper edge go up, losers above the lower edge go down
            for j in np.nonzero((s > lo) & (s < hi))[0]:
                want = 1 if winner[j] else -1
                moves[int(j)] = min(moves.get(int(j), want), want)
        step = []
        for j, way in sorted(moves.items()):
            chosen = None
            for allow_cross in (False, True):
                for f in (_UP if way > 0 else _DOWN):
                    ok = True
                    for c, lo, hi in zones:
                        v0, v1 = scores[c][j], scores[c][j] * f
                        if lo * (1.0 - pad) < v1 < hi * (1.0 + pad):
                            ok = False           # would end inside (or too close to) a boundary
                        elif not allow_cross and (v0 <= lo) != (v1 <= lo) and not (lo * (1.0 - 1e-12) < v0 < hi * (1.0 + 1e-12)):
                            ok = False           # would change the set of a sequence it has nothing to do with
                        if not ok:
                            break
                    if ok:
                        chosen = f
                        break
                if chosen is not None:
                    break
            step.append((j, chosen if chosen is not None else (_UP if way > 0 else _DOWN)[3]))
        rows_l = [j for j, _ in step]
        synth.apply_nudges(W1, step, dtype)
        nudges.extend(step)
        Wg_r = None if Wg is None else Wg[rows_l]
        bg_r = None if bg is None else np.asarray(bg)[rows_l]
        b1_r = None if b1 is None else np.asarray(b1)[rows_l]
        for X, Z in zip(Xs, Zs):
            Z[:, rows_l] = oracle.ff1(X, Wg_r, W1[rows_l], act, bg_r, b1_r)
    raise RuntimeError("top-k margin did not open in %d iterations" % max_iter)
