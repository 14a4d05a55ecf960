"""Ordered-list formulation of TOVA (TEST INFRASTRUCTURE ONLY).

A second, differently organised statement of the same policy, kept to pin the slot-based oracle:
the multi-state is a list of token ids in temporal order, each token's key / value rows are looked
up in a dictionary, and a dropped token is simply taken out of the list, which closes the gap
(Sec. 4: the rows before and after j stay, in their order).  Per step (Sec. 3.2, then Sec. 4 and
App. B): the incoming token joins the list, the query attends over every listed token, and if
the list is now longer than the multi-state size the token whose attention weight, averaged over
the heads of the layer, is lowest leaves.  Weights come from torch's softmax, not from the
slot-based oracle's own exponentials.

Both formulations must hold the same set of tokens after every step.  They differ only in where a
row is stored and in which of several exactly tied tokens leaves: here the oldest one (first in
temporal order), there the one in the lowest slot.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Tuple

import numpy as np
import torch


class OrderedTova:
    def __init__(self, k: int, H: int, H_kv: int, d: int, scale: Optional[float] = None):
        assert H % H_kv == 0
        self.size, self.H, self.H_kv, self.d = k, H, H_kv, d
        self.scale = (1.0 / np.sqrt(float(d))) if scale is None or scale <= 0 else float(scale)
        self.tokens: List[int] = []                                       # temporal order
        self.rows: Dict[int, Tuple[torch.Tensor, torch.Tensor]] = {}      # token -> (key [H_kv, d], value [H_kv, d])
        self.t = 0

    def step(self, q, k_new, v_new):
        """Returns (attention output [H, d], id of the token that left or None)."""
        me = self.t
        self.t += 1
        self.tokens.append(me)
        self.rows[me] = (torch.as_tensor(np.asarray(k_new, dtype=np.float64)).reshape(self.H_kv, self.d),
                         torch.as_tensor(np.asarray(v_new, dtype=np.float64)).reshape(self.H_kv, self.d))
        G = self.H // self.H_kv
        query = torch.as_tensor(np.asarray(q, dtype=np.float64)).reshape(self.H_kv, G, self.d)
        keys = torch.stack([self.rows[tok][0] for tok in self.tokens], dim=1)      # [H_kv, n, d]
        vals = torch.stack([self.rows[tok][1] for tok in self.tokens], dim=1)
        weights = torch.softmax(self.scale * torch.einsum("cgd,cnd->cgn", query, keys), dim=-1)   # [H_kv, G, n]
        out = torch.einsum("cgn,cnd->cgd", weights, vals).reshape(self.H, self.d).numpy()
        gone = None
        if len(self.tokens) > self.size:
            per_token = weights.reshape(self.H, -1).mean(dim=0)            # averaged over the layer's heads
            gone = self.tokens[int(torch.argmin(per_token))]               # (the first of equal minima: the oldest)
            self.tokens.remove(gone)
            del self.rows[gone]
        return out, gone
