"""Choosing the staleness threshold T on a sample of the inputs (section 3.3).

The arithmetic runs in the library: ss_detect_stale writes the drift of every
hot row once, ss_sample_drop counts the droppable sampled inputs for a ladder
of up to 32 candidate thresholds in one pass, ss_drop_stats turns a count into
the estimate and confidence interval of Eq. 2-4.  This module only drives those
calls and holds the search over T, which is host control flow.

The paper searches T by bisection over the sampled drop estimates and does not
say when the search stops or what it aims at.  The rule taken here: the caller
names the largest share of inputs it is willing to drop, and the search returns
the largest T it has tried whose interval's upper end stays within that share.
Because one pass prices 32 thresholds, each pass splits the bracket into 33
parts instead of 2; two passes resolve T to about 1/1000 of the starting
bracket (in the logarithm).
"""
from __future__ import annotations

import math
from typing import Callable, List, Optional, Sequence, Tuple

T_CRIT_999 = 3.340        # critical value the paper uses for 99.9 % (section 3.3.3)


def geometric_ladder(lo: float, hi: float, n: int) -> List[float]:
    """n thresholds strictly inside (lo, hi), evenly spaced in the logarithm."""
    if not (0.0 < lo < hi) or n < 1:
        raise ValueError("need 0 < lo < hi and n >= 1")
    step = (math.log(hi) - math.log(lo)) / (n + 1)
    return [math.exp(math.log(lo) + step * (k + 1)) for k in range(n)]


def ladder_search(upper_bounds: Callable[[Sequence[float]], Sequence[float]],
                  lo: float, hi: float, budget: float, passes: int = 2,
                  width: int = 32) -> Tuple[Optional[float], List[Tuple[float, float]]]:
    """Largest tried T in [lo, hi] whose upper bound on the dropped share is
    within `budget`, assuming the bound does not decrease with T.

    upper_bounds(thresholds) returns one bound per threshold.  Returns
    (T or None if even `lo` is over budget, every (T, bound) pair evaluated).
    """
    tried: List[Tuple[float, float]] = []
    ends = list(upper_bounds([lo, hi]))
    tried += [(lo, ends[0]), (hi, ends[1])]
    if ends[0] > budget:
        return None, tried
    if ends[1] <= budget:
        return hi, tried
    good, bad = lo, hi
    for _ in range(passes):
        ladder = geometric_ladder(good, bad, width)
        ladder = [t for t in ladder if good < t < bad]      # rounding at a tiny bracket
        if not ladder:
            break
        bounds = list(upper_bounds(ladder))
        tried += list(zip(ladder, bounds))
        for t, b in zip(ladder, bounds):
            if b <= budget:
                good = t
            else:
                bad = t
                break
    return good, tried


class SamplingBlock:
    """Drop estimates for candidate thresholds on a fixed sample of inputs.

    hot: the HotState of the running step (its snapshot is the reference the
    drift is measured against); sidx: int32 [T, S, L] lookups of the sampled
    inputs, on the device; population: number of inputs the sample was drawn
    from; n_hot_inputs: scale of the count-valued interval.
    """

    def __init__(self, tables, hot, sidx, alpha: int, population: int,
                 n_hot_inputs: Optional[int] = None, t_crit: float = T_CRIT_999):
        import torch
        from . import binding as B
        self._B = B
        self.tables, self.hot, self.sidx = tables, hot, sidx
        self.alpha, self.population = int(alpha), int(population)
        self.n_hot_inputs = self.population if n_hot_inputs is None else int(n_hot_inputs)
        self.t_crit = float(t_crit)
        self.n_samples = int(sidx.shape[1])
        self.counts = torch.zeros(B.MAX_THRESHOLDS, dtype=torch.int32, device=sidx.device)

    def refresh_drift(self) -> None:
        """Drift of every hot row against the stored snapshot; changes nothing else."""
        self._B.ss_detect_stale(self.tables, self.hot, 0.0, refresh_snapshot=False)

    def counts_for(self, thresholds: Sequence[float]) -> List[int]:
        """Droppable sampled inputs per threshold (waits for the GPU)."""
        out: List[int] = []
        for i in range(0, len(thresholds), self._B.MAX_THRESHOLDS):
            chunk = list(thresholds[i:i + self._B.MAX_THRESHOLDS])
            self._B.ss_sample_drop(self.hot, self.sidx, self.alpha, chunk, self.counts)
            got = self.counts[:len(chunk)].cpu().numpy().view("uint32")
            out += [int(c) for c in got]
        return out

    def estimate(self, thresholds: Sequence[float]) -> List[dict]:
        return [self._B.ss_drop_stats(c, self.n_samples, self.population,
                                      self.n_hot_inputs, self.t_crit)
                for c in self.counts_for(thresholds)]

    def find_threshold(self, budget: float, lo: float, hi: float, passes: int = 2):
        """See ladder_search; call refresh_drift() first."""
        return ladder_search(lambda ts: [e["hi"] for e in self.estimate(ts)],
                             lo, hi, budget, passes, self._B.MAX_THRESHOLDS)
