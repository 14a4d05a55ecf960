"""Plant plausible mistakes in the oracle (on the CPU) and show that the pins catch each."""
import numpy as np
import pytest

from oracle.tova_oracle import TovaOracle, StepResult

import pins


class NoScale(TovaOracle):                       # dropped 1/sqrt(d)
    def __init__(self, k, H, H_kv, d, scale=None):
        super().__init__(k, H, H_kv, d, 1.0)


class WrongGroup(TovaOracle):                    # h % H_kv instead of h // G
    def attend(self, q, k_new, v_new):
        q = np.asarray(q, dtype=np.float64).reshape(self.H, self.d)
        perm = [(h % self.H_kv) * self.G + (h // self.H_kv) for h in range(self.H)]
        out, p = super().attend(q[perm], k_new, v_new)
        inv = np.argsort(perm)
        return out[inv], p[inv]


class ArgMax(TovaOracle):                        # wrong sign in the victim rule
    @staticmethod
    def select(s, pinned=0):
        j = int(np.argmax(s))
        return j, 0.0


class LastOnTies(TovaOracle):                    # highest instead of lowest index on ties
    @staticmethod
    def select(s, pinned=0):
        j = int(len(s) - 1 - np.argmin(s[::-1]))
        rest = np.delete(s, j)
        return j, float(np.min(rest) - s[j])


class NewTokenImmune(TovaOracle):                # argmin over cached rows only
    @staticmethod
    def select(s, pinned=0):
        j = int(np.argmin(s[:-1]))
        rest = np.delete(s, j)
        return j, float(np.min(rest) - s[j])


class EvictBeforeAttend(TovaOracle):             # output does not see the victim
    def step(self, q, k_new, v_new, force_victim=None):
        r = super().step(q, k_new, v_new, force_victim)
        if r.evicted >= 0:
            out, _ = self.attend(q, k_new, v_new)   # recomputed on the post-eviction state
            return StepResult(out, r.evicted, r.gap, r.s)
        return r


class FirstHeadOnly(TovaOracle):                 # no averaging over heads
    def scores(self, p):
        return p[0].copy()


class SwappedKV(TovaOracle):                     # transposed operands in the update
    def update(self, evicted, k_new, v_new):
        super().update(evicted, v_new, k_new)


class OffByOneCapacity(TovaOracle):              # starts evicting one step late
    def step(self, q, k_new, v_new, force_victim=None):
        if self.n == self.k and self.t == self.k:
            out, _ = self.attend(q, k_new, v_new)
            self.t += 1
            return StepResult(out, self.k, 0.0, None)
        return super().step(q, k_new, v_new, force_victim)


MUTANTS = [NoScale, WrongGroup, ArgMax, LastOnTies, NewTokenImmune, EvictBeforeAttend,
           FirstHeadOnly, SwappedKV, OffByOneCapacity]


@pytest.mark.parametrize("mutant", MUTANTS, ids=lambda c: c.__name__)
def test_some_pin_catches(mutant):
    caught = []
    for pin in pins.ALL_PINS:
        try:
            pin(mutant)
        except AssertionError:
            caught.append(pin.__name__)
        except Exception:                      # a crash also counts as caught
            caught.append(pin.__name__ + "(error)")
    assert caught, f"no pin notices the planted mistake {mutant.__name__}"
