"""The oracle of TOVA with re-assigned positions (Sec. 7.2) against its pins, and planted
mistakes (on the CPU) that the pins must catch."""
import math

import numpy as np
import pytest

from oracle.tova_positions import TovaPositionsOracle, compressed_positions, rope

import pins_positions as pp

PINS = [pp.pin_gap_rule, pp.pin_rotary, pp.pin_full_attention_with_ordinary_positions, pp.pin_origin_invariance,
        pp.pin_two_dimensional_closed_form, pp.pin_brute_force_from_the_stream]


@pytest.mark.parametrize("pin", PINS, ids=lambda f: f.__name__)
def test_pin(pin):
    pin(TovaPositionsOracle)


def _chain(tokens, gap):
    tokens = np.asarray(tokens, dtype=np.int64)
    pos = np.empty(tokens.size)
    pos[0] = float(tokens[0])
    for m in range(1, tokens.size):
        pos[m] = pos[m - 1] + gap(float(tokens[m] - tokens[m - 1]))
    return pos


class SingleLog(TovaPositionsOracle):            # ln g instead of ln ln g
    positions_of = staticmethod(lambda tok: _chain(tok, lambda g: g if g <= 10 else math.log(g)))


class ThresholdOffByOne(TovaPositionsOracle):    # a gap of exactly 10 is compressed too
    positions_of = staticmethod(lambda tok: _chain(tok, lambda g: g if g < 10 else math.log(math.log(g))))


class EveryGapCompressed(TovaPositionsOracle):   # local gaps not kept
    positions_of = staticmethod(lambda tok: _chain(tok, lambda g: math.log(math.log(max(g, 3.0)))))


class OriginalPositions(TovaPositionsOracle):    # no re-assignment at all
    positions_of = staticmethod(lambda tok: np.asarray(tok, dtype=np.float64))


class GapsFromTheStart(TovaPositionsOracle):     # each token's own distance to the first one compressed, not adjacent gaps
    positions_of = staticmethod(lambda tok: np.array([float(tok[0])] + [
        tok[0] + (float(x - tok[0]) if x - tok[0] <= 10 else math.log(math.log(float(x - tok[0])))) for x in tok[1:]]))


class SlotOrder(TovaPositionsOracle):            # chain over the slots as they lie, not in temporal order
    def candidate_positions(self):
        tokens = np.concatenate([self.slot_token[: self.n], [self.t]])
        pos = np.empty(tokens.size)
        pos[0] = float(tokens[0])
        for m in range(1, tokens.size):
            g = abs(float(tokens[m] - tokens[m - 1]))
            pos[m] = pos[m - 1] + (g if g <= 10 else math.log(math.log(g)))
        return pos


class InterleavedPairs(TovaPositionsOracle):     # pairs (2i, 2i+1) instead of (i, i + d/2)
    @staticmethod
    def rotary(x, pos, base=10000.0):
        x = np.asarray(x, dtype=np.float64)
        d = x.shape[-1]
        perm = np.concatenate([np.arange(0, d, 2), np.arange(1, d, 2)])
        out = np.empty_like(rope(x[..., perm], pos, base))
        out[..., perm] = rope(x[..., perm], pos, base)
        return out


class BackwardsRotation(TovaPositionsOracle):    # wrong sign of the angle
    rotary = staticmethod(lambda x, pos, base=10000.0: rope(x, -np.asarray(pos, dtype=np.float64), base))


class QueryNotRotated(TovaPositionsOracle):      # keys get positions, the query does not
    def attend(self, q, k_new, v_new):
        real = self.rotary
        calls = {"n": 0}

        def rot(x, pos, base=10000.0):
            calls["n"] += 1
            return real(x, pos, base) if np.ndim(pos) else np.asarray(x, dtype=np.float64)
        self.rotary = rot
        try:
            return super().attend(q, k_new, v_new)
        finally:
            del self.rotary


class ValuesRotated(TovaPositionsOracle):        # positions applied to the values as well
    def attend(self, q, k_new, v_new):
        out, p = super().attend(q, k_new, v_new)
        pos = self.candidate_positions()
        v_new = np.asarray(v_new, dtype=np.float64).reshape(self.H_kv, self.d)
        for g in range(self.H_kv):
            Vc = rope(np.concatenate([self.V[g, : self.n], v_new[g][None, :]], axis=0), pos, self.base)
            for h in range(g * self.G, (g + 1) * self.G):
                out[h] = p[h] @ Vc
        return out, p


class WrongBaseExponent(TovaPositionsOracle):    # base^(-i/d) instead of base^(-2i/d)
    rotary = staticmethod(lambda x, pos, base=10000.0: rope(x, pos, math.sqrt(base)))


MUTANTS = [SingleLog, ThresholdOffByOne, EveryGapCompressed, OriginalPositions, GapsFromTheStart, SlotOrder,
           InterleavedPairs, BackwardsRotation, QueryNotRotated, ValuesRotated, WrongBaseExponent]


@pytest.mark.parametrize("mutant", MUTANTS, ids=lambda c: c.__name__)
def test_some_pin_catches(mutant):
    caught = []
    for pin in PINS:
        try:
            pin(mutant)
        except AssertionError:
            caught.append(pin.__name__)
    assert caught, f"no pin notices {mutant.__name__}"
    print(mutant.__name__, "caught by", caught)
