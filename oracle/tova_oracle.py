"""Slot-based fp64 oracle of one TOVA decode step (TEST INFRASTRUCTURE ONLY).

State of one (layer, sequence) unit: a multi-state of at most k rows,
H_t = (K_t, V_t) (Sec. 3.1, 3.2), kept here in k fixed slots.

One decode step, in the paper's order:
  1. the incoming token's k_t, v_t are appended to the multi-state and the
     query attends over all of it (Sec. 3.2, the two-line layer equation);
     so the softmax runs over the cached rows plus the new one, and the output
     still sees the row that is about to be dropped;
  2. attention is Softmax(q K^T) V per head (Sec. 2.2); the usual 1/sqrt(d)
     scaling, which that section leaves out "for brevity", is applied;
  3. once the multi-state would exceed k rows (t > k, Sec. 3.3), the TOVA
     policy (Sec. 4 "TOVA", and the appendix algorithm) averages the last
     query's attention weights over the heads of the layer, takes the argmin
     and removes that row from K and V; below capacity it does nothing.

Readings the paper leaves open (all listed in the design notes):
  * removal is done by overwriting the victim's slot with the new token
    instead of compacting; single-query attention does not depend on row
    order, so the retained set and every output are the same;
  * candidate index n (= k when full) is the incoming token; if it has the
    lowest score it is simply not stored;
  * ties go to the lowest candidate index;
  * with grouped-query attention the mean runs over all H query heads and the
    one victim is shared by every KV head.

Two variants from the paper's policy ablation (App. A) are covered as well:
  * TOVA+i: the first i tokens are additionally never dropped (`pinned=i`); they
    occupy slots 0..i-1 from the fill phase on, so the argmin simply skips those
    candidates;
  * TOVA-head: every head keeps its own set of tokens (TovaHeadOracle); with
    grouped-query attention a "head" is a KV head with the G query heads it serves,
    averaged as in the layer variant.

Everything is float64; inputs are whatever the caller rounded them to
(bf16 / fp32 values convert to float64 exactly).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np


@dataclass
class StepResult:
    out: np.ndarray        # [H, d] attention output of this step
    evicted: int           # -1 below capacity; 0..k-1 slot; k = incoming token dropped
    gap: float             # second-lowest minus lowest head-mean score (inf below capacity)
    s: Optional[np.ndarray]  # [k+1] head-mean scores (None below capacity)


class TovaOracle:
    def __init__(self, k: int, H: int, H_kv: int, d: int, scale: Optional[float] = None, pinned: int = 0):
        assert k >= 1 and H >= 1 and H_kv >= 1 and H % H_kv == 0 and d >= 1
        assert 0 <= pinned < k
        self.k, self.H, self.H_kv, self.d = k, H, H_kv, d
        self.pinned = pinned                         # TOVA+i: tokens 0..i-1 (= slots 0..i-1) are kept
        self.G = H // H_kv
        self.scale = (1.0 / np.sqrt(float(d))) if scale is None or scale <= 0 else float(scale)
        self.K = np.zeros((H_kv, k, d), dtype=np.float64)
        self.V = np.zeros((H_kv, k, d), dtype=np.float64)
        self.n = 0                                   # occupied slots, g(t) = min(t, k)
        self.slot_token = np.full(k, -1, dtype=np.int64)
        self.t = 0                                   # index of the next token

    # -- step 1 + 2: append, then attend (Sec. 3.2; Sec. 2.2) ------------------
    def attend(self, q, k_new, v_new):
        q = np.asarray(q, dtype=np.float64).reshape(self.H, self.d)
        k_new = np.asarray(k_new, dtype=np.float64).reshape(self.H_kv, self.d)
        v_new = np.asarray(v_new, dtype=np.float64).reshape(self.H_kv, self.d)
        n = self.n
        out = np.empty((self.H, self.d), dtype=np.float64)
        p = np.empty((self.H, n + 1), dtype=np.float64)
        for g in range(self.H_kv):
            # the multi-state of KV head g with the incoming row appended
            Kc = np.concatenate([self.K[g, :n], k_new[g][None, :]], axis=0)   # [n+1, d]
            Vc = np.concatenate([self.V[g, :n], v_new[g][None, :]], axis=0)
            for h in range(g * self.G, (g + 1) * self.G):             # query heads it serves: h // G == g
                l = self.scale * (Kc @ q[h])                          # logits over the n+1 candidates
                w = np.exp(l - np.max(l))
                p[h] = w / np.sum(w)                                  # softmax
                out[h] = p[h] @ Vc
        return out, p

    # -- step 3a: head-averaged score of the last (only) query -----------------
    def scores(self, p):
        s = np.zeros(p.shape[1], dtype=np.float64)
        for h in range(self.H):                                   # fixed head order
            s = s + p[h]
        return s / self.H

    # -- step 3b: victim = argmin, lowest index on ties -------------------------
    @staticmethod
    def select(s, pinned: int = 0):
        """Victim among the candidates pinned..len(s)-1 (pinned = 0: all of them)."""
        cand = s[pinned:]
        j = int(np.argmin(cand))                                  # first occurrence of the minimum
        rest = np.delete(cand, j)
        gap = float(np.min(rest) - cand[j]) if rest.size else float("inf")
        return j + pinned, gap

    # -- step 3c: state update ---------------------------------------------------
    def update(self, evicted: int, k_new, v_new):
        k_new = np.asarray(k_new, dtype=np.float64).reshape(self.H_kv, self.d)
        v_new = np.asarray(v_new, dtype=np.float64).reshape(self.H_kv, self.d)
        if evicted < 0:                     # below capacity: the new row takes the next free slot
            assert self.n < self.k
            slot = self.n
            self.n += 1
        elif evicted < self.k:              # a cached row leaves; the new row takes its slot
            slot = evicted
        else:                               # the incoming token itself scored lowest
            slot = None
        if slot is not None:
            self.K[:, slot, :] = k_new
            self.V[:, slot, :] = v_new
            self.slot_token[slot] = self.t
        self.t += 1

    def step(self, q, k_new, v_new, force_victim: Optional[int] = None) -> StepResult:
        """One decode step.  force_victim lets a test make the oracle follow a
        different, equally-scored choice after a counted near-tie."""
        out, p = self.attend(q, k_new, v_new)
        if self.n + 1 <= self.k:            # num_kv <= cache_max_size: nothing to drop
            self.update(-1, k_new, v_new)
            return StepResult(out, -1, float("inf"), None)
        s = self.scores(p)
        j, gap = self.select(s, self.pinned)
        self.update(j if force_victim is None else int(force_victim), k_new, v_new)
        return StepResult(out, j, gap, s)


class TovaHeadOracle:
    """TOVA-head (App. A): every KV head keeps its own multi-state and drops its own row.
    KV head g with its G query heads is an independent TovaOracle(k, G, 1, d)."""

    def __init__(self, k: int, H: int, H_kv: int, d: int, scale: Optional[float] = None, pinned: int = 0):
        assert H % H_kv == 0
        self.k, self.H, self.H_kv, self.d, self.G = k, H, H_kv, d, H // H_kv
        self.heads = [TovaOracle(k, self.G, 1, d, scale, pinned) for _ in range(H_kv)]

    def step(self, q, k_new, v_new):
        """q [H, d], k_new / v_new [H_kv, d] -> list of StepResult, one per KV head."""
        q = np.asarray(q, dtype=np.float64).reshape(self.H_kv, self.G, self.d)
        k_new = np.asarray(k_new, dtype=np.float64).reshape(self.H_kv, 1, self.d)
        v_new = np.asarray(v_new, dtype=np.float64).reshape(self.H_kv, 1, self.d)
        return [self.heads[g].step(q[g], k_new[g], v_new[g]) for g in range(self.H_kv)]


def run_stream(k: int, q, k_new, v_new, scale: Optional[float] = None):
    """Run one unit over a whole stream.

    q [T, H, d], k_new / v_new [T, H_kv, d] (any real dtype).  Returns
    (out [T, H, d], evicted [T], gap [T], oracle) with the oracle holding the
    final state.
    """
    q = np.asarray(q, dtype=np.float64)
    k_new = np.asarray(k_new, dtype=np.float64)
    v_new = np.asarray(v_new, dtype=np.float64)
    T, H, d = q.shape
    H_kv = k_new.shape[1]
    orc = TovaOracle(k, H, H_kv, d, scale)
    out = np.empty((T, H, d), dtype=np.float64)
    evicted = np.empty(T, dtype=np.int64)
    gap = np.empty(T, dtype=np.float64)
    for t in range(T):
        r = orc.step(q[t], k_new[t], v_new[t])
        out[t], evicted[t], gap[t] = r.out, r.evicted, r.gap
    return out, evicted, gap, orc
