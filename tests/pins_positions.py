"""Pins for the oracle of TOVA with re-assigned positions (Sec. 7.2), written as functions of
the oracle class so that the same checks run on deliberately broken variants.

None of them re-types the oracle's formulae through the same calls: the rotary embedding is
checked against complex multiplication, the positions against closed forms of the rule, the
whole step against torch's attention at ordinary positions (nothing ever dropped), against a
scalar simulation of a two-dimensional case with closed-form logits, and against a
recomputation from the raw stream with python loops and cmath.
"""
from __future__ import annotations

import cmath
import math

import numpy as np
import torch


def _stream(rng, T, H, H_kv, d):
    return (rng.standard_normal((T, H, d)), rng.standard_normal((T, H_kv, d)), rng.standard_normal((T, H_kv, d)))


def _complex_rope(x, pos, base):
    """(x[i] + 1j x[i + d/2]) * exp(1j pos base^(-2i/d)), python scalars."""
    d = len(x)
    h = d // 2
    out = [0.0] * d
    for i in range(h):
        z = complex(x[i], x[i + h]) * cmath.exp(1j * pos * base ** (-2.0 * i / d))
        out[i], out[i + h] = z.real, z.imag
    return out


# the rule itself: gaps of at most 10 are kept, longer ones become ln ln g (Sec. 7.2)
def pin_gap_rule(Oracle):
    pos = Oracle.positions_of
    for g in range(1, 11):
        p = pos([7, 7 + g])
        assert p[0] == 7.0 and p[1] == 7.0 + g                      # the paper's (i, i+g) -> (i, i+g) for g <= 10
    for g, want in [(11, math.log(math.log(11.0))), (16, math.log(math.log(16.0))), (70000, math.log(math.log(70000.0)))]:
        p = pos([3, 3 + g])
        assert abs((p[1] - p[0]) - want) < 1e-15                    # (i, i+g) -> (i, i + ln ln g)
    # closed forms of ln ln: g = round(e^e) is about 1, g = round(e^(e^2)) about 2
    assert abs(pos([0, 15])[1] - 1.0) < 0.01 and abs(pos([0, 1618])[1] - 2.0) < 1e-3
    # positions chain over adjacent pairs; contiguous tokens keep theirs
    np.testing.assert_array_equal(pos(list(range(5, 40))), np.arange(5, 40, dtype=np.float64))
    p = pos([2, 4, 30, 31, 1000])
    want = [2.0, 4.0, 4.0 + math.log(math.log(26.0)), 5.0 + math.log(math.log(26.0)),
            5.0 + math.log(math.log(26.0)) + math.log(math.log(969.0))]
    np.testing.assert_allclose(p, want, rtol=0, atol=1e-14)


# the rotary embedding against complex multiplication, and its group properties
def pin_rotary(Oracle):
    rng = np.random.default_rng(3)
    rot = Oracle.rotary
    for d in (2, 8, 32):
        for base in (10000.0, 50.0):
            x = rng.standard_normal(d)
            for p in (0.0, 1.0, 17.25, -3.5, 4097.874):
                np.testing.assert_allclose(rot(x, p, base), _complex_rope(list(x), p, base), rtol=0, atol=1e-12)
            np.testing.assert_array_equal(rot(x, 0.0, base), x)
            np.testing.assert_allclose(rot(rot(x, 2.5, base), 4.0, base), rot(x, 6.5, base), atol=1e-12)
            y = rng.standard_normal(d)
            a = float(rot(x, 11.0, base) @ rot(y, 4.0, base))
            b = float(rot(x, 107.0, base) @ rot(y, 100.0, base))
            assert abs(a - b) < 1e-11                                # only the difference of positions counts
    # the first pair turns by the position itself (angle p * base^0): (1, 0) at p = pi/2 becomes (0, 1)
    x = np.zeros(8)
    x[0] = 1.0
    r = rot(x, math.pi / 2, 10000.0)
    assert abs(r[0]) < 1e-15 and abs(r[4] - 1.0) < 1e-15


# nothing is ever dropped => all gaps are 1 => ordinary rotary attention over the whole prefix
def pin_full_attention_with_ordinary_positions(Oracle):
    rng = np.random.default_rng(21)
    for (T, H, H_kv, d, base) in [(9, 4, 4, 8, 10000.0), (14, 6, 2, 16, 100.0)]:
        q, kk, vv = _stream(rng, T, H, H_kv, d)
        G = H // H_kv
        for t0 in (0, 5):
            orc = Oracle(T + 2, H, H_kv, d, base=base, t0=t0)
            for t in range(T):
                r = orc.step(q[t], kk[t], vv[t])
                assert r.evicted == -1
                Kr = np.array([[_complex_rope(list(kk[u, g]), t0 + u, base) for u in range(t + 1)] for g in range(H_kv)])
                qr = np.array([_complex_rope(list(q[t, h]), t0 + t, base) for h in range(H)])
                Kt = torch.from_numpy(Kr).repeat_interleave(G, dim=0)
                Vt = torch.from_numpy(vv[: t + 1]).permute(1, 0, 2).repeat_interleave(G, dim=0)
                ref = torch.nn.functional.scaled_dot_product_attention(torch.from_numpy(qr).unsqueeze(1), Kt, Vt)
                np.testing.assert_allclose(r.out, ref[:, 0, :].numpy(), rtol=1e-10, atol=1e-12)


# where the stream starts does not matter
def pin_origin_invariance(Oracle):
    rng = np.random.default_rng(8)
    T, H, H_kv, d, k = 60, 4, 2, 8, 5
    q, kk, vv = _stream(rng, T, H, H_kv, d)
    runs = []
    for t0 in (0, 123456):
        orc = Oracle(k, H, H_kv, d, t0=t0)
        runs.append([orc.step(q[t], kk[t], vv[t]) for t in range(T)])
    for a, b in zip(*runs):
        assert a.evicted == b.evicted
        np.testing.assert_allclose(a.out, b.out, rtol=0, atol=1e-9)


# capacity 1, one head, d = 2, base-independent (the only pair has angle = position), scale 1:
# every key is (kappa, 0) un-rotated and every query (1, 0), so the cached token's logit is
# kappa_old * cos(c(t - tau)) and the incoming token's is kappa_new: a scalar simulation.
def pin_two_dimensional_closed_form(Oracle):
    T = 90
    kappa = [1.0] + [-1.5] * (T - 1)       # weak incoming keys: the cached token survives long gaps ...
    for t in (30, 60):
        kappa[t] = 2.0                     # ... until a strong one arrives
    orc = Oracle(1, 1, 1, 2, scale=1.0)
    tau, seen_long_gap, seen_drop_new, seen_drop_old = None, False, False, False
    for t in range(T):
        r = orc.step(np.array([[1.0, 0.0]]), np.array([[kappa[t], 0.0]]), np.array([[float(t), 1.0]]))
        if tau is None:
            assert r.evicted == -1
            tau = 0
            continue
        g = t - tau
        c = float(g) if g <= 10 else math.log(math.log(float(g)))
        l_old, l_new = kappa[tau] * math.cos(c), kappa[t]
        want = 0 if l_old < l_new else (1 if l_new < l_old else 0)
        assert r.evicted == want, (t, tau, g, l_old, l_new)
        p_old = math.exp(l_old) / (math.exp(l_old) + math.exp(l_new))
        assert abs(r.out[0, 0] - (p_old * tau + (1 - p_old) * t)) < 1e-9
        seen_long_gap |= g > 10
        seen_drop_new |= want == 1
        seen_drop_old |= want == 0
        if want == 0:
            tau = t
    assert seen_long_gap and seen_drop_new and seen_drop_old      # the case walks through all three


# brute force on tiny inputs: from the raw stream and the retained token ids only
def pin_brute_force_from_the_stream(Oracle):
    rng = np.random.default_rng(17)
    checked = 0
    for (k, H, H_kv, d, T, base) in [(3, 2, 1, 4, 70, 10000.0), (5, 3, 3, 2, 60, 10.0), (2, 4, 2, 8, 50, 10000.0)]:
        q, kk, vv = _stream(rng, T, H, H_kv, d)
        G = H // H_kv
        scale = 1.0 / math.sqrt(d)
        orc = Oracle(k, H, H_kv, d, base=base)
        for t in range(T):
            held = sorted(int(x) for x in orc.slot_token[: orc.n])      # before the step
            r = orc.step(q[t], kk[t], vv[t])
            cand = held + [t]
            pos = [float(cand[0])]
            for a, b in zip(cand[:-1], cand[1:]):
                gap = b - a
                pos.append(pos[-1] + (gap if gap <= 10 else math.log(math.log(gap))))
            s = [0.0] * len(cand)
            for h in range(H):
                qr = _complex_rope(list(q[t, h]), pos[-1], base)
                ls = []
                for u, tok in enumerate(cand):
                    kr = _complex_rope(list(kk[tok, h // G]), pos[u], base)
                    ls.append(scale * math.fsum(a * b for a, b in zip(qr, kr)))
                m = max(ls)
                w = [math.exp(x - m) for x in ls]
                z = math.fsum(w)
                for u in range(len(cand)):
                    s[u] += w[u] / z / H
            if len(cand) <= k:
                assert r.evicted == -1
                continue
            srt = sorted(s)
            if srt[1] - srt[0] < 1e-9:
                continue
            victim_token = cand[int(np.argmin(s))]
            # (the oracle reports a slot; what must agree is the set of tokens it holds afterwards)
            after = sorted(int(x) for x in orc.slot_token[: orc.n])
            assert sorted(set(cand) - {victim_token}) == after, (t, cand, victim_token, after)
            checked += 1
    assert checked > 100
