"""Ordered-list formulation of TOVA (TEST INFRASTRUCTURE ONLY).

This is the policy as the paper's appendix states it (App. B, Alg. 1): the
cache is a list of rows in temporal order with shape [heads, num_kv, dim]; the
policy receives the attention weights [heads, num_q, num_kv] that were already
computed over the cache *including* the newest row, does nothing while
num_kv <= cache_max_size, and otherwise averages the last query's weights
over heads, takes the argmin and closes the gap left by that row (Sec. 4, the
equation that stacks the rows before and after j).

It exists to pin the slot-based oracle: both must retain the same set of
tokens at every step (they differ only in where a row is stored, and in which
of several exactly tied rows leaves: here the oldest, there the lowest slot).
Written for MHA and GQA alike; the caches hold one row per KV head.
"""
from __future__ import annotations

from typing import List, Optional, Tuple

import numpy as np


def tova_policy(attn_weights: np.ndarray, k_cache: np.ndarray, v_cache: np.ndarray,
                cache_max_size: int) -> Tuple[np.ndarray, np.ndarray, Optional[int]]:
    """attn_weights [heads, num_q, num_kv]; k_cache, v_cache [kv_heads, num_kv, dim].
    Returns the (possibly shortened) caches and the dropped position or None."""
    num_kv = attn_weights.shape[2]
    assert k_cache.shape[1] == num_kv and v_cache.shape[1] == num_kv
    if num_kv <= cache_max_size:
        return k_cache, v_cache, None
    last_query = attn_weights[:, -1, :]                 # [heads, num_kv]
    mean_w = last_query.mean(axis=0)
    drop = int(np.argmin(mean_w))
    keep = [c for c in range(num_kv) if c != drop]
    return k_cache[:, keep, :], v_cache[:, keep, :], drop


class LiteralTova:
    """Decoder-layer view: append the new row, attend, then apply the policy."""

    def __init__(self, k: int, H: int, H_kv: int, d: int, scale: Optional[float] = None):
        self.k, self.H, self.H_kv, self.d = k, H, H_kv, d
        self.scale = (1.0 / np.sqrt(float(d))) if scale is None or scale <= 0 else float(scale)
        self.k_cache = np.zeros((H_kv, 0, d))
        self.v_cache = np.zeros((H_kv, 0, d))
        self.tokens: List[int] = []       # token id of every cached row, temporal order
        self.t = 0

    def step(self, q, k_new, v_new):
        q = np.asarray(q, dtype=np.float64).reshape(self.H, self.d)
        k_new = np.asarray(k_new, dtype=np.float64).reshape(self.H_kv, 1, self.d)
        v_new = np.asarray(v_new, dtype=np.float64).reshape(self.H_kv, 1, self.d)
        # (K_t, V_t) = ((K_{t-1}; k_t), (V_{t-1}; v_t))         (Sec. 3.2)
        self.k_cache = np.concatenate([self.k_cache, k_new], axis=1)
        self.v_cache = np.concatenate([self.v_cache, v_new], axis=1)
        self.tokens.append(self.t)
        G = self.H // self.H_kv
        k_rep = np.repeat(self.k_cache, G, axis=0)              # [H, num_kv, d]
        v_rep = np.repeat(self.v_cache, G, axis=0)
        logits = self.scale * np.einsum("hd,hnd->hn", q, k_rep)
        logits = logits - logits.max(axis=1, keepdims=True)
        w = np.exp(logits)
        attn = w / w.sum(axis=1, keepdims=True)                 # [H, num_kv]
        out = np.einsum("hn,hnd->hd", attn, v_rep)
        self.k_cache, self.v_cache, drop = tova_policy(attn[:, None, :], self.k_cache,
                                                       self.v_cache, self.k)
        dropped_token = None
        if drop is not None:
            dropped_token = self.tokens.pop(drop)
        self.t += 1
        return out, dropped_token
