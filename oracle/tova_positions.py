"""fp64 oracle of TOVA decoding beyond the training length (TEST INFRASTRUCTURE ONLY).

Sec. 7.2 ("Extrapolation with TOVA"): with a bounded multi-state the retained tokens end up
far apart, so before each attention the positions of the cached tokens are re-assigned: the
gap g between two tokens that are adjacent in the multi-state becomes ln(ln(g)), except that
gaps of at most 10 are kept as they are.  The positional encoding is then applied with those
positions, which is only possible if the cache holds the keys WITHOUT positional encoding.

Per decode step, for one (layer, sequence) unit:
  1. the candidates are the cached tokens and the incoming one (as in the plain step);
  2. sorted by token index, consecutive candidates get the compressed gaps; a candidate's
     position is the running sum of the gaps before it (the first candidate keeps its own
     index -- the paper's example maps (i, i+g) to (i, i+ln ln g); only differences of
     positions ever reach the logits, so that origin has no effect);
  3. rotary position embedding with those (real-valued) positions on the cached keys, the
     incoming key and the query; the query's position is the incoming token's;
  4. from there on the plain TOVA step: softmax, outputs, head-mean scores, argmin.
The cache keeps the un-rotated keys, and values are never rotated.

Readings (all listed in the design notes): natural logarithms; the rule is applied at every
step to the set the query attends over; the rotary embedding is the standard one of the model
family the paper uses, pairing element i with element i + d/2 and using the angles
p * base^(-2i/d), base 10000 unless given.  The paper does not define it (it belongs to the
models); it is restated here from its published definition.
"""
from __future__ import annotations

from typing import Optional

import numpy as np

from .tova_oracle import TovaOracle

GAP_KEPT = 10          # gaps up to this many tokens keep their length (Sec. 7.2)


def compress_gap(g: float) -> float:
    """New distance between two adjacent tokens whose indices differ by g >= 1."""
    g = float(g)
    assert g >= 1.0
    return g if g <= GAP_KEPT else float(np.log(np.log(g)))


def compressed_positions(tokens) -> np.ndarray:
    """tokens: strictly increasing token indices.  Returns their re-assigned positions."""
    tokens = np.asarray(tokens, dtype=np.int64)
    assert tokens.ndim == 1 and tokens.size >= 1 and np.all(np.diff(tokens) > 0)
    pos = np.empty(tokens.size, dtype=np.float64)
    pos[0] = float(tokens[0])
    for m in range(1, tokens.size):
        pos[m] = pos[m - 1] + compress_gap(tokens[m] - tokens[m - 1])
    return pos


def rope(x, pos, base: float = 10000.0) -> np.ndarray:
    """Rotary embedding of x[..., d] at position(s) pos (broadcast over the leading axes):
    the pair (x[i], x[i + d/2]) is rotated by the angle pos * base**(-2 i / d)."""
    x = np.asarray(x, dtype=np.float64)
    d = x.shape[-1]
    assert d % 2 == 0
    half = d // 2
    theta = float(base) ** (-2.0 * np.arange(half, dtype=np.float64) / d)
    ang = np.asarray(pos, dtype=np.float64)[..., None] * theta
    c, s = np.cos(ang), np.sin(ang)
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


class TovaPositionsOracle(TovaOracle):
    """TovaOracle whose q / k_new arrive without positional encoding and whose attention
    re-assigns the positions of everything it attends over first (steps 1-3 above)."""

    def __init__(self, k: int, H: int, H_kv: int, d: int, scale: Optional[float] = None, pinned: int = 0,
                 base: float = 10000.0, t0: int = 0):
        super().__init__(k, H, H_kv, d, scale, pinned)
        assert d % 2 == 0
        self.base = float(base)
        self.t = int(t0)                          # index of the first token (any origin gives the same results)

    # (as attributes, so that a test can plant a mistake in either and show that the pins notice)
    positions_of = staticmethod(compressed_positions)
    rotary = staticmethod(rope)

    def candidate_positions(self) -> np.ndarray:
        """Positions of the n cached slots (slot order) followed by the incoming token's."""
        n = self.n
        tokens = np.concatenate([self.slot_token[:n], [self.t]])
        order = np.argsort(tokens, kind="stable")                 # temporal order
        pos = np.empty(n + 1, dtype=np.float64)
        pos[order] = self.positions_of(tokens[order])
        return pos

    def attend(self, q, k_new, v_new):
        q = np.asarray(q, dtype=np.float64).reshape(self.H, self.d)
        k_new = np.asarray(k_new, dtype=np.float64).reshape(self.H_kv, self.d)
        v_new = np.asarray(v_new, dtype=np.float64).reshape(self.H_kv, self.d)
        n = self.n
        pos = self.candidate_positions()
        out = np.empty((self.H, self.d), dtype=np.float64)
        p = np.empty((self.H, n + 1), dtype=np.float64)
        for g in range(self.H_kv):
            Kc = np.concatenate([self.K[g, :n], k_new[g][None, :]], axis=0)   # [n+1, d], no positions in them
            Vc = np.concatenate([self.V[g, :n], v_new[g][None, :]], axis=0)
            Kr = self.rotary(Kc, pos, self.base)                                     # each row at its own position
            for h in range(g * self.G, (g + 1) * self.G):
                qr = self.rotary(q[h], pos[n], self.base)                            # the query sits at the incoming token
                l = self.scale * (Kr @ qr)
                w = np.exp(l - np.max(l))
                p[h] = w / np.sum(w)
                out[h] = p[h] @ Vc
        return out, p
