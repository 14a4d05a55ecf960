"""Mask formulation of TOVA over a whole prompt (TEST INFRASTRUCTURE ONLY).

For language modelling the paper scores all positions of a text at once and
folds the policy into the attention mask: row t of the mask is what the bounded
multi-state holds when token t is processed, and it is derived from the
attention weights of the layer itself, one row after the other (appendix on the
language-modelling experiments; Sec. 3.3 for the bounded multi-state, Sec. 4 and
App. B Alg. 1 for the rule that removes a token).  Nothing is ever compacted or
moved here: K and V stay the full [T] arrays and only the mask changes.

This is the definition of what processing a prompt of m tokens in one call must
produce (num_q > 1): exactly what m single-token steps produce.  It pins the
slot-based oracle from a third side (same outputs, same retained tokens), and
the multi-token entry point of the library is checked against the slot-based
oracle on the strength of that.

Ties: a removed token is the one with the lowest mean weight; among exactly
tied ones this formulation drops the oldest (first occurrence, as an argmin over
the temporally ordered row does), the slot-based oracle the lowest slot.  On
continuous data they agree.
"""
from __future__ import annotations

from typing import Optional, Tuple

import numpy as np


def tova_masked_prompt(q, k, v, capacity: int, scale: Optional[float] = None,
                       pinned: int = 0) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """q [T, H, d]; k, v [T, H_kv, d].  Returns (out [T, H, d], mask [T, T] bool with
    mask[t, j] = position t attends to token j, dropped [T] = token removed after
    position t or -1)."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    T, H, d = q.shape
    H_kv = k.shape[1]
    G = H // H_kv
    sc = (1.0 / np.sqrt(float(d))) if scale is None or scale <= 0 else float(scale)
    mask = np.zeros((T, T), dtype=bool)
    out = np.zeros((T, H, d))
    dropped = np.full(T, -1, dtype=np.int64)
    state = np.zeros(T, dtype=bool)          # tokens currently in the multi-state
    for t in range(T):
        state[t] = True                      # the incoming token joins before it attends (Sec. 3.2)
        mask[t] = state
        cols = np.flatnonzero(state)         # temporal order
        mean_w = np.zeros(len(cols))
        for h in range(H):
            logits = sc * (k[cols, h // G, :] @ q[t, h])
            w = np.exp(logits - logits.max())
            p = w / w.sum()
            out[t, h] = p @ v[cols, h // G, :]
            mean_w += p
        mean_w /= H
        if len(cols) > capacity:             # (App. B: nothing happens while num_kv <= cache_max_size)
            cand = mean_w.copy()
            cand[cols < pinned] = np.inf     # TOVA+i keeps the first i tokens (App. A)
            j = int(np.argmin(cand))
            dropped[t] = cols[j]
            state[cols[j]] = False
    return out, mask, dropped
