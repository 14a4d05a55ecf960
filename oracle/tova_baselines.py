"""fp64 oracles of the baseline compression policies the paper compares TOVA with (TEST
INFRASTRUCTURE ONLY): Window, Window+i and H2O (Sec. 4.1, "Baseline Compression Policies").

They plug into the same place as TOVA (Sec. 3.3: a policy turns a multi-state of k+1 rows into one
of k rows) and share everything before it with the TOVA oracle: the incoming token's row is appended,
the query attends over all k+1 rows (Sec. 3.2, Sec. 2.2), and the output still sees the row that is
about to leave.  Only the choice of the row differs:

  * Window (Sec. 4.1): first in, first out -- the oldest row leaves.
  * Window+i (Sec. 4.1): the same, but the first i tokens are never dropped; the oldest row that is
    not one of them leaves.  i = 0 is Window.
  * H2O (Sec. 4.1): a window of the most recent tokens is always kept; the other rows are the ones
    with the highest attention scores AGGREGATED over the sequence so far.  The number of non-window
    rows is "typically half of the multi-state size".  Layer-wise here (the head-averaged weights
    are aggregated and all heads share the victim); the head-wise variant the paper reports is this
    oracle per head, exactly as TovaHeadOracle is TovaOracle per head.

Readings of what the section leaves open (listed in the design notes):
  * Window+i / Window: the incoming token is always stored (it is the most recent one).
  * H2O: the multi-state of k rows holds `heavy` non-window rows and k - heavy window rows, heavy =
    floor(k / 2) unless given; the k - heavy most recent tokens, the incoming one included, are the
    window and cannot leave; every row carries the sum, over all steps since its token came in (that
    step included), of its head-averaged attention weight; at a step with k+1 rows the weights of that
    step are added first and then, among the rows outside the window, the one with the lowest sum
    leaves; ties go to the lowest slot index (as everywhere in this library).  While the multi-state
    has room the sums are aggregated all the same ("throughout the sequence").
"""
from __future__ import annotations

from typing import Optional

import numpy as np

from .tova_oracle import StepResult, TovaOracle


class WindowOracle(TovaOracle):
    """Window+i (Sec. 4.1); pinned = i, 0 for plain Window.  Slots as in TovaOracle: the victim's
    slot is overwritten by the incoming row."""

    def select_oldest(self):
        """Slot of the oldest token that is not one of the first `pinned`."""
        tok = self.slot_token.astype(np.float64)
        tok[self.slot_token < self.pinned] = np.inf          # the first i tokens stay
        return int(np.argmin(tok))

    def step(self, q, k_new, v_new, force_victim: Optional[int] = None) -> StepResult:
        out, _ = self.attend(q, k_new, v_new)
        if self.n + 1 <= self.k:
            self.update(-1, k_new, v_new)
            return StepResult(out, -1, float("inf"), None)
        j = self.select_oldest()
        self.update(j if force_victim is None else int(force_victim), k_new, v_new)
        return StepResult(out, j, float("inf"), None)


class H2OOracle(TovaOracle):
    """H2O, layer-wise (Sec. 4.1).  heavy = number of non-window rows (default floor(k / 2))."""

    def __init__(self, k: int, H: int, H_kv: int, d: int, scale: Optional[float] = None,
                 heavy: Optional[int] = None):
        super().__init__(k, H, H_kv, d, scale, pinned=0)
        self.heavy = k // 2 if heavy is None else int(heavy)
        assert 0 <= self.heavy < k
        self.recent = k - self.heavy                          # window size, the incoming token included
        self.acc = np.zeros(k, dtype=np.float64)              # aggregated head-mean weight per slot

    def eligible(self):
        """Candidates (slots 0..n-1, then the incoming token) that are outside the recent window."""
        newest_protected = self.t - self.recent + 1           # tokens >= this are in the window
        el = np.zeros(self.n + 1, dtype=bool)
        el[: self.n] = self.slot_token[: self.n] < newest_protected
        return el                                             # (the incoming token, index n, never is)

    def step(self, q, k_new, v_new, force_victim: Optional[int] = None) -> StepResult:
        out, p = self.attend(q, k_new, v_new)
        s = self.scores(p)                                    # head-mean weights of this step, [n+1]
        n = self.n
        total = np.concatenate([self.acc[:n] + s[:n], [s[n]]])   # aggregate first ...
        self.acc[:n] = total[:n]
        if n + 1 <= self.k:
            self.update(-1, k_new, v_new)
            self.acc[n] = total[n]
            return StepResult(out, -1, float("inf"), None)
        el = self.eligible()
        cand = np.where(el, total, np.inf)                    # ... then the lowest outside the window leaves
        j = int(np.argmin(cand))
        rest = np.delete(cand, j)
        gap = float(np.min(rest) - cand[j]) if np.isfinite(np.min(rest)) else float("inf")
        v = j if force_victim is None else int(force_victim)
        assert v < self.k
        self.update(v, k_new, v_new)
        self.acc[v] = total[n]                                # the incoming token starts its own sum
        return StepResult(out, j, gap, total)
