"""Pins for the fp64 oracle, written as functions of an oracle class so that the
same checks can be run on deliberately broken variants (test_oracle_mutants).

Each pin raises AssertionError on failure.  None of them re-types the oracle's
formulae through the same library calls: they use torch's softmax / SDPA, pure
Python loops with math.fsum over the raw stream, closed forms, or invariants.
"""
from __future__ import annotations

import math

import numpy as np
import torch

from oracle.tova_literal import OrderedTova


def _stream(rng, T, H, H_kv, d, scale=1.0):
    return (rng.standard_normal((T, H, d)) * scale,
            rng.standard_normal((T, H_kv, d)) * scale,
            rng.standard_normal((T, H_kv, d)) * scale)


# P1 -- the multi-state never fills => plain full attention (App. B: the policy returns
# early while num_kv <= cache_max_size; App. A: every policy equals the full model at 4096)
def pin_full_attention(Oracle):
    rng = np.random.default_rng(11)
    for (T, H, H_kv, d) in [(9, 4, 4, 8), (12, 6, 2, 16), (7, 8, 1, 4)]:
        q, kk, vv = _stream(rng, T, H, H_kv, d)
        for k in (T, T + 5):
            orc = Oracle(k, H, H_kv, d)
            for t in range(T):
                r = orc.step(q[t], kk[t], vv[t])
                assert r.evicted == -1
                G = H // H_kv
                Kt = torch.from_numpy(kk[: t + 1]).permute(1, 0, 2).repeat_interleave(G, dim=0)
                Vt = torch.from_numpy(vv[: t + 1]).permute(1, 0, 2).repeat_interleave(G, dim=0)
                qt = torch.from_numpy(q[t]).unsqueeze(1)                       # [H,1,d]
                ref = torch.nn.functional.scaled_dot_product_attention(qt, Kt, Vt)  # 1/sqrt(d) scale
                np.testing.assert_allclose(r.out, ref[:, 0, :].numpy(), rtol=1e-12, atol=1e-13)


# P2 -- g(t) = min(t, k) (Sec. 3.3)
def pin_occupancy(Oracle):
    rng = np.random.default_rng(5)
    for k in (1, 3, 8):
        T, H, H_kv, d = 30, 4, 2, 8
        q, kk, vv = _stream(rng, T, H, H_kv, d)
        orc = Oracle(k, H, H_kv, d)
        for t in range(T):
            orc.step(q[t], kk[t], vv[t])
            assert orc.n == min(t + 1, k) and orc.n <= k
            assert int((orc.slot_token >= 0).sum()) == orc.n


def _brute_scores(q_t, keys, G, scale):
    """Head-mean softmax weights of one query over a list of key rows, computed with
    python floats, loops ordered candidate-major, and math.fsum."""
    H = len(q_t)
    n = len(keys)
    logits = [[scale * math.fsum(float(q_t[h][i]) * float(keys[c][h // G][i]) for i in range(len(q_t[h])))
               for h in range(H)] for c in range(n)]
    s = []
    Z = [math.fsum(math.exp(logits[c][h]) for c in range(n)) for h in range(H)]
    for c in range(n):
        s.append(math.fsum(math.exp(logits[c][h]) / Z[h] for h in range(H)) / H)
    return s


# P3 -- brute force on tiny inputs from the raw stream + ordered-list formulation
def pin_brute_force(Oracle):
    rng = np.random.default_rng(2024)
    cases = [(1, 1, 1, 1), (2, 1, 1, 4), (3, 3, 3, 4), (5, 3, 1, 2), (4, 4, 2, 3), (5, 6, 3, 4)]
    for (k, H, H_kv, d) in cases:
        T = 4 * k + 7
        q, kk, vv = _stream(rng, T, H, H_kv, d)
        G = H // H_kv
        scale = 1.0 / math.sqrt(d)
        orc = Oracle(k, H, H_kv, d)
        lit = OrderedTova(k, H, H_kv, d)
        retained = []                       # token ids, maintained by brute force
        for t in range(T):
            slot_token_before = orc.slot_token.copy()
            n_before = orc.n
            r = orc.step(q[t], kk[t], vv[t])
            out_lit, dropped_lit = lit.step(q[t], kk[t], vv[t])
            np.testing.assert_allclose(r.out, out_lit, rtol=1e-11, atol=1e-12)
            cand_tokens = retained + [t]
            if len(cand_tokens) <= k:
                assert r.evicted == -1 and dropped_lit is None
                retained = cand_tokens
            else:
                s = _brute_scores(q[t], [kk[c] for c in cand_tokens], G, scale)
                victim_token = cand_tokens[min(range(len(s)), key=lambda c: (s[c], 0))]
                srt = sorted(s)
                assert srt[1] - srt[0] > 1e-9, "test stream has a near-tie; change the seed"
                # the oracle's victim, translated from slot index to token id
                tok = t if r.evicted == k else int(slot_token_before[r.evicted])
                assert n_before == k and 0 <= r.evicted <= k
                assert tok == victim_token, (k, H, H_kv, d, t, tok, victim_token)
                assert dropped_lit == victim_token
                assert abs(r.gap - (srt[1] - srt[0])) < 1e-12
                np.testing.assert_allclose(sorted(r.s), srt, rtol=0, atol=1e-13)
                retained = [c for c in cand_tokens if c != victim_token]
            assert sorted(int(x) for x in orc.slot_token if x >= 0) == sorted(retained)
            assert sorted(lit.tokens) == sorted(retained)
            # cached rows really are the raw rows of the retained tokens
            for slot in range(orc.n):
                tk = int(orc.slot_token[slot])
                np.testing.assert_array_equal(orc.K[:, slot, :], kk[tk])
                np.testing.assert_array_equal(orc.V[:, slot, :], vv[tk])


# P4 -- after capacity is reached exactly one of the k+1 candidates leaves per step (Sec. 4)
def pin_one_leaves(Oracle):
    rng = np.random.default_rng(3)
    k, T, H, H_kv, d = 6, 40, 4, 2, 8
    q, kk, vv = _stream(rng, T, H, H_kv, d)
    orc = Oracle(k, H, H_kv, d)
    prev = set()
    for t in range(T):
        r = orc.step(q[t], kk[t], vv[t])
        cur = set(int(x) for x in orc.slot_token if x >= 0)
        if t >= k:
            assert 0 <= r.evicted <= k
            assert len((prev | {t}) - cur) == 1 and cur <= (prev | {t})
        else:
            assert r.evicted == -1 and cur == prev | {t}
        prev = cur


# P5 -- softmax rows and the head-mean sum to one; outputs lie in the hull of the V rows
def pin_simplex_hull(Oracle):
    rng = np.random.default_rng(8)
    k, T, H, H_kv, d = 5, 25, 6, 3, 4
    q, kk, vv = _stream(rng, T, H, H_kv, d, scale=2.0)
    orc = Oracle(k, H, H_kv, d)
    for t in range(T):
        n = orc.n
        Vc = np.concatenate([orc.V[:, :n], vv[t][:, None, :]], axis=1)
        out, p = orc.attend(q[t], kk[t], vv[t])
        assert p.shape == (H, n + 1) and np.all(p >= 0)
        np.testing.assert_allclose(p.sum(axis=1), 1.0, rtol=0, atol=1e-14)
        G = H // H_kv
        for h in range(H):
            lo, hi = Vc[h // G].min(axis=0), Vc[h // G].max(axis=0)
            assert np.all(out[h] >= lo - 1e-12) and np.all(out[h] <= hi + 1e-12)
        r = orc.step(q[t], kk[t], vv[t])
        if r.s is not None:
            assert abs(r.s.sum() - 1.0) < 1e-14 and r.s.shape == (k + 1,)


# P6 -- the victim does not depend on V; permuting the slots permutes the victim index
# and changes neither the output nor the evicted token
def pin_v_independence_and_permutation(Oracle):
    rng = np.random.default_rng(21)
    k, T, H, H_kv, d = 7, 30, 4, 2, 8
    q, kk, vv = _stream(rng, T, H, H_kv, d)
    a, b = Oracle(k, H, H_kv, d), Oracle(k, H, H_kv, d)
    vv2 = rng.standard_normal(vv.shape) * 3.0
    for t in range(T):
        ra, rb = a.step(q[t], kk[t], vv[t]), b.step(q[t], kk[t], vv2[t])
        assert ra.evicted == rb.evicted
    # permutation
    a, b = Oracle(k, H, H_kv, d), Oracle(k, H, H_kv, d)
    for t in range(k):
        a.step(q[t], kk[t], vv[t]); b.step(q[t], kk[t], vv[t])
    perm = rng.permutation(k)
    b.K, b.V, b.slot_token = b.K[:, perm].copy(), b.V[:, perm].copy(), b.slot_token[perm].copy()
    for t in range(k, T):
        tok_a, tok_b = a.slot_token.copy(), b.slot_token.copy()
        ra, rb = a.step(q[t], kk[t], vv[t]), b.step(q[t], kk[t], vv[t])
        np.testing.assert_allclose(ra.out, rb.out, rtol=1e-12, atol=1e-13)
        ta = t if ra.evicted == k else tok_a[ra.evicted]
        tb = t if rb.evicted == k else tok_b[rb.evicted]
        assert ta == tb


# P7 -- closed forms
def pin_closed_forms(Oracle):
    rng = np.random.default_rng(4)
    # (a) k = 1, one head: of {cached, incoming} the row with the larger logit q.k survives
    d, T = 6, 40
    q, kk, vv = _stream(rng, T, 1, 1, d)
    orc = Oracle(1, 1, 1, d)
    kept = None
    for t in range(T):
        r = orc.step(q[t], kk[t], vv[t])
        if t == 0:
            kept = 0
            continue
        l_old, l_new = float(q[t, 0] @ kk[kept, 0]), float(q[t, 0] @ kk[t, 0])
        assert r.evicted == (0 if l_old < l_new else 1)
        kept = t if l_old < l_new else kept
        assert int(orc.slot_token[0]) == kept
    # (b) all keys identical => every candidate has the same score exactly => slot 0 leaves
    k, H, H_kv = 4, 4, 2
    key = rng.standard_normal((H_kv, d))
    orc = Oracle(k, H, H_kv, d)
    for t in range(20):
        r = orc.step(rng.standard_normal((H, d)), key, rng.standard_normal((H_kv, d)))
        assert r.evicted == (-1 if t < k else 0)
        if t >= k:
            assert r.gap == 0.0
    # (c) softmax of equal logits is uniform: output is the plain mean of the V rows
    orc = Oracle(8, 2, 2, d)
    vs = rng.standard_normal((5, 2, d))
    for t in range(5):
        r = orc.step(rng.standard_normal((2, d)), key[:2], vs[t])
        np.testing.assert_allclose(r.out, vs[: t + 1].mean(axis=0), rtol=1e-12, atol=1e-13)
    # (d) a key strongly aligned with every query is never evicted;
    #     a key strongly anti-aligned is evicted as soon as the cache is full
    k, H, H_kv, d = 5, 4, 4, 8
    u = np.ones(d) / math.sqrt(d)
    orc = Oracle(k, H, H_kv, d)
    for t in range(60):
        qq = rng.standard_normal((H, d)) * 0.1 + 4.0 * u
        kn = rng.standard_normal((H_kv, d)) * 0.1
        if t == 2:
            kn = kn + 6.0 * u
        if t == 20:
            kn = kn - 6.0 * u
        r = orc.step(qq, kn, rng.standard_normal((H_kv, d)))
        assert 2 in orc.slot_token or t < 2
        if t == 20:
            assert r.evicted == k          # the anti-aligned incoming token is dropped at once
    # (e) scale: with d = 4 and q = k = (2,0,0,0) vs a zero key the logits are 2 and 0
    #     (1/sqrt(d) = 1/2), so the weights are e^2/(1+e^2) and 1/(1+e^2)
    orc = Oracle(4, 1, 1, 4)
    orc.step(np.zeros((1, 4)), np.zeros((1, 4)), np.array([[1.0, 0, 0, 0]]))
    out, p = orc.attend(np.array([[2.0, 0, 0, 0]]), np.array([[2.0, 0, 0, 0]]), np.array([[0, 1.0, 0, 0]]))
    e2 = math.exp(2.0)
    np.testing.assert_allclose(p[0], [1 / (1 + e2), e2 / (1 + e2)], rtol=1e-14)
    np.testing.assert_allclose(out[0], [1 / (1 + e2), e2 / (1 + e2), 0, 0], rtol=1e-14)


# GQA head grouping: query head h reads KV head h // G.  With one-hot structure the
# answer is known in closed form.
def pin_gqa_grouping(Oracle):
    H, H_kv, d = 6, 3, 4
    orc = Oracle(8, H, H_kv, d)
    # KV head g stores value rows equal to (g+1) * ones, keys zero => uniform weights
    for t in range(3):
        vn = np.stack([(g + 1.0) * np.ones(d) for g in range(H_kv)])
        r = orc.step(np.ones((H, d)), np.zeros((H_kv, d)), vn)
    for h in range(H):
        np.testing.assert_allclose(r.out[h], (h // 2 + 1.0) * np.ones(d), rtol=1e-14)
    # mean over *query* heads: make only query head 4 (KV head 2) attend sharply to token 0
    k, d = 3, 2
    orc = Oracle(k, H, H_kv, d)
    keys = np.zeros((4, H_kv, d))
    keys[0, 2] = [10.0, 0.0]                      # token 0 attractive for KV head 2 only
    keys[1, 0] = [10.0, 0.0]                      # token 1 attractive for KV head 0 only
    qs = np.zeros((H, d))
    qs[4] = [10.0, 0.0]                           # query head 4 -> KV head 4 // 2 = 2
    ev = [orc.step(qs, keys[t], np.zeros((H_kv, d))).evicted for t in range(4)]
    # at t=3 candidates are tokens 0,1,2 and 3; head 4 puts ~all mass on token 0, the other
    # five heads are uniform, so tokens 1,2,3 tie exactly (their keys are invisible to the
    # zero queries of KV head 0) and the lowest index among them, slot 1, leaves.
    assert ev == [-1, -1, -1, 1]


# P10 -- a whole prompt under the mask formulation (appendix on the language-modelling runs: the
# policy folded into the attention mask, K and V never moved) gives what the single-token steps
# give: same outputs, same token removed at every position, same final multi-state.  It is also
# the definition of what a multi-token call must produce.
def pin_mask_formulation(Oracle):
    from oracle.tova_masked import tova_masked_prompt
    rng = np.random.default_rng(23)
    for (T, H, H_kv, d, k) in [(40, 4, 4, 8, 5), (60, 8, 2, 16, 12), (25, 6, 1, 4, 1), (30, 4, 2, 8, 40)]:
        q, kk, vv = _stream(rng, T, H, H_kv, d)
        out_m, mask, dropped = tova_masked_prompt(q, kk, vv, k)
        orc = Oracle(k, H, H_kv, d)
        for t in range(T):
            held_before = set(int(x) for x in orc.slot_token[: orc.n])
            r = orc.step(q[t], kk[t], vv[t])
            assert set(np.flatnonzero(mask[t])) == held_before | {t}
            np.testing.assert_allclose(r.out, out_m[t], rtol=1e-11, atol=1e-13)
            if r.evicted < 0:
                assert dropped[t] == -1
            elif r.evicted == k:
                assert dropped[t] == t
            else:
                assert dropped[t] in held_before and dropped[t] not in set(int(x) for x in orc.slot_token[: orc.n])
        assert int(mask.sum(axis=1).max()) <= k + 1          # never more than the multi-state plus the newcomer


ALL_PINS = [pin_full_attention, pin_occupancy, pin_brute_force, pin_one_leaves, pin_simplex_hull,
            pin_v_independence_and_permutation, pin_closed_forms, pin_gqa_grouping, pin_mask_formulation]
