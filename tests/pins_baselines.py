"""Pins for the baseline-policy oracles (Window, Window+i, H2O: Sec. 4.1), written as functions of the
oracle classes so that the same checks run on deliberately broken variants.

None of them re-types the oracle's formulae through the same calls: closed forms of the retained
sets, torch's attention over the tokens a closed form names, a hand-computed four-step example,
and a brute-force recomputation from the raw stream with python floats / math.fsum and
accumulators kept per TOKEN in a dictionary (the oracle keeps them per slot in an array)."""
from __future__ import annotations

import math

import numpy as np
import torch

from pins import _brute_scores, _stream


def _sdpa(q_t, K_rows, V_rows, G):
    """torch attention (1/sqrt(d) scale) of one query [H, d] over rows [n, H_kv, d]."""
    Kt = torch.from_numpy(np.asarray(K_rows)).permute(1, 0, 2).repeat_interleave(G, dim=0)
    Vt = torch.from_numpy(np.asarray(V_rows)).permute(1, 0, 2).repeat_interleave(G, dim=0)
    return torch.nn.functional.scaled_dot_product_attention(torch.from_numpy(q_t).unsqueeze(1), Kt, Vt)[:, 0].numpy()


# W1 -- Window+i keeps the first i tokens and the k - i most recent ones, nothing else (Sec. 4.1), and
# the output of step t is plain attention over exactly those of step t-1 plus token t
def pin_window_closed_form(Window):
    rng = np.random.default_rng(31)
    for (k, i, H, H_kv, d) in [(1, 0, 2, 1, 4), (4, 0, 4, 2, 8), (5, 1, 4, 4, 4), (8, 4, 6, 2, 8), (6, 5, 2, 2, 2)]:
        T = 3 * k + 9
        q, kk, vv = _stream(rng, T, H, H_kv, d)
        orc = Window(k, H, H_kv, d, pinned=i)
        held = []
        for t in range(T):
            r = orc.step(q[t], kk[t], vv[t])
            attended = held + [t]
            np.testing.assert_allclose(r.out, _sdpa(q[t], kk[attended], vv[attended], H // H_kv), rtol=1e-12, atol=1e-13)
            held = sorted(set(range(min(i, t + 1))) | set(range(max(0, t - (k - i) + 1), t + 1)))
            assert sorted(int(x) for x in orc.slot_token if x >= 0) == held, (k, i, t)
            assert orc.n == min(t + 1, k)
            if t >= k:
                assert r.evicted == i + (t - k) % (k - i)        # the slots behind the first i are a ring
            else:
                assert r.evicted == -1


# H1 -- H2O on identical keys: every weight is 1/(n+1), so an older token's aggregate is strictly larger
# than a younger one's and the token that has just left the window is always the one to go: the
# multi-state holds the first `heavy` tokens and the k - heavy most recent ones (the bias towards
# initial tokens that the footnote of Sec. 4.1 describes), and with heavy = 0 it is Window
def pin_h2o_identical_keys(H2O):
    rng = np.random.default_rng(32)
    for (k, heavy, H, H_kv, d) in [(2, None, 2, 1, 4), (6, None, 4, 2, 8), (7, 2, 4, 4, 4), (5, 0, 2, 2, 4), (8, 7, 2, 1, 2)]:
        T = 3 * k + 5
        q, _, vv = _stream(rng, T, H, H_kv, d)
        key = rng.standard_normal((1, H_kv, d)).repeat(T, axis=0)
        orc = H2O(k, H, H_kv, d, heavy=heavy)
        hv = k // 2 if heavy is None else heavy
        rec = k - hv
        for t in range(T):
            r = orc.step(q[t], key[t], vv[t])
            held = sorted(set(range(min(hv, t + 1))) | set(range(max(0, t - rec + 1), t + 1)))
            assert sorted(int(x) for x in orc.slot_token if x >= 0) == held, (k, heavy, t, orc.slot_token)
            if t >= k:
                assert r.evicted == hv + (t - k) % rec
        # the aggregate of token 0: sum over the steps of 1 / (rows attended over)
        want = math.fsum(1.0 / (min(t, k) + 1) for t in range(T)) if hv > 0 else None
        if want is not None:
            assert abs(orc.acc[list(orc.slot_token).index(0)] - want) < 1e-12


# H2 -- a hand-computed example (one head, d = 1, scale 1, k = 3, one window row): the weights of the
# step are added BEFORE the lowest aggregate is looked for.  Tokens 0..2 fill the cache under
# uniform attention (aggregates 11/6, 5/6, 1/3).  At step 3 the query picks out token 2 (logit 20
# against 0): token 2 ends at 1/3 + ~1 and token 1, at 5/6 + ~0, is the one to go -- although it
# was ahead of token 2 before this step.  Then a uniform step: the window is token 4 alone, token 3
# (aggregate ~0 + 1/4) is the lowest outside it.
def pin_h2o_worked_example(H2O):
    orc = H2O(3, 1, 1, 1, scale=1.0, heavy=2)
    keys = [0.0, 0.0, 5.0, 0.0, 0.0]
    qs = [0.0, 0.0, 0.0, 4.0, 0.0]
    ev = [orc.step(np.array([[qs[t]]]), np.array([[keys[t]]]), np.array([[float(t)]])).evicted for t in range(5)]
    assert ev[:3] == [-1, -1, -1]
    assert ev[3] == 1, ev                     # not 2: its weight of this step counts
    assert ev[4] == 1, ev                     # token 3 sits in token 1's slot and is the lowest again
    e20 = math.exp(20.0)
    tok2 = 1.0 / 3 + e20 / (e20 + 3) + 0.25
    assert abs(orc.acc[2] - tok2) < 1e-12 and abs(orc.acc[0] - (1 + 0.5 + 1.0 / 3 + 1 / (e20 + 3) + 0.25)) < 1e-12
    assert abs(orc.acc[1] - 0.25) < 1e-12     # token 4 came in with its own weight of that step


# H3 -- brute force from the raw stream: aggregates per token in a dictionary, weights through python
# floats and math.fsum, the window taken from token indices; victim token and retained set must agree
def pin_h2o_brute_force(H2O):
    rng = np.random.default_rng(33)
    for (k, heavy, H, H_kv, d) in [(2, None, 1, 1, 1), (3, None, 2, 2, 3), (5, 1, 3, 1, 2), (6, None, 4, 2, 4), (4, 3, 2, 1, 4)]:
        T = 4 * k + 6
        q, kk, vv = _stream(rng, T, H, H_kv, d)
        G, scale = H // H_kv, 1.0 / math.sqrt(d)
        hv = k // 2 if heavy is None else heavy
        rec = k - hv
        orc = H2O(k, H, H_kv, d, heavy=heavy)
        agg = {}                                              # token -> aggregated head-mean weight
        held = []                                             # tokens in the multi-state
        for t in range(T):
            cand = held + [t]
            s = _brute_scores(q[t], [kk[c] for c in cand], G, scale)
            for c, w in zip(cand, s):
                agg[c] = agg.get(c, 0.0) + w
            r = orc.step(q[t], kk[t], vv[t])
            if len(cand) <= k:
                held = cand
                assert r.evicted == -1
            else:
                outside = [c for c in cand if c <= t - rec]
                assert len(outside) == hv + 1
                lo = min(agg[c] for c in outside)
                near = [c for c in outside if agg[c] - lo < 1e-9]
                assert len(near) == 1, "the random stream produced a near tie; pick another seed"
                held = [c for c in cand if c != near[0]]
                assert r.evicted < k and sorted(int(x) for x in orc.slot_token) == sorted(held), (k, heavy, t)
            for slot in range(orc.n):
                assert abs(orc.acc[slot] - agg[int(orc.slot_token[slot])]) < 1e-12
            assert set(range(max(0, t - rec + 1), t + 1)) <= set(held)      # the window is always there


# H4 -- shared with TOVA: outputs are plain attention over what the multi-state held (torch), and
# while it has room nothing leaves (every policy equals the full model then: App. A, last column)
def pin_baselines_attend_over_their_state(Policy, **kw):
    rng = np.random.default_rng(34)
    k, H, H_kv, d, T = 6, 4, 2, 8, 25
    q, kk, vv = _stream(rng, T, H, H_kv, d)
    orc = Policy(k, H, H_kv, d, **kw)
    for t in range(T):
        held = [int(x) for x in orc.slot_token[: orc.n]]
        r = orc.step(q[t], kk[t], vv[t])
        np.testing.assert_allclose(r.out, _sdpa(q[t], kk[held + [t]], vv[held + [t]], H // H_kv), rtol=1e-12, atol=1e-13)
        assert (r.evicted == -1) == (t < k) and orc.n == min(t + 1, k)
    big = Policy(T, H, H_kv, d, **kw)
    for t in range(T):
        r = big.step(q[t], kk[t], vv[t])
        np.testing.assert_allclose(r.out, _sdpa(q[t], kk[: t + 1], vv[: t + 1], H // H_kv), rtol=1e-12, atol=1e-13)
        assert r.evicted == -1


def run_all(Window, H2O):
    pin_window_closed_form(Window)
    pin_baselines_attend_over_their_state(Window, pinned=2)
    pin_h2o_identical_keys(H2O)
    pin_h2o_worked_example(H2O)
    pin_h2o_brute_force(H2O)
    pin_baselines_attend_over_their_state(H2O)
