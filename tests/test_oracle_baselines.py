"""The baseline-policy oracles (Window, Window+i, H2O: Sec. 4.1) against their pins, and planted
mistakes (on the CPU) that the pins must catch."""
import numpy as np
import pytest

from oracle.tova_baselines import H2OOracle, WindowOracle
from oracle.tova_oracle import StepResult, TovaOracle

import pins_baselines as pb


def test_window_pins():
    pb.pin_window_closed_form(WindowOracle)
    pb.pin_baselines_attend_over_their_state(WindowOracle, pinned=2)
    pb.pin_baselines_attend_over_their_state(WindowOracle, pinned=0)


def test_h2o_pins():
    pb.pin_h2o_identical_keys(H2OOracle)
    pb.pin_h2o_worked_example(H2OOracle)
    pb.pin_h2o_brute_force(H2OOracle)
    pb.pin_baselines_attend_over_their_state(H2OOracle)
    pb.pin_baselines_attend_over_their_state(H2OOracle, heavy=1)


def test_h2o_without_heavy_rows_is_window():
    """heavy = 0: the window is the whole multi-state, so H2O drops the oldest token like Window."""
    rng = np.random.default_rng(3)
    k, H, H_kv, d, T = 5, 4, 2, 8, 30
    q, kk, vv = (rng.standard_normal((T, n, d)) for n in (H, H_kv, H_kv))
    a, b = H2OOracle(k, H, H_kv, d, heavy=0), WindowOracle(k, H, H_kv, d)
    for t in range(T):
        ra, rb = a.step(q[t], kk[t], vv[t]), b.step(q[t], kk[t], vv[t])
        assert ra.evicted == rb.evicted and np.array_equal(ra.out, rb.out)


def test_h2o_differs_from_tova_and_window():
    """The three policies are really different on a random stream (otherwise the pins above would
    not separate them)."""
    rng = np.random.default_rng(4)
    k, H, H_kv, d, T = 8, 4, 2, 8, 60
    q, kk, vv = (rng.standard_normal((T, n, d)) for n in (H, H_kv, H_kv))
    orcs = [H2OOracle(k, H, H_kv, d), WindowOracle(k, H, H_kv, d, pinned=1), TovaOracle(k, H, H_kv, d)]
    sets = []
    for o in orcs:
        for t in range(T):
            o.step(q[t], kk[t], vv[t])
        sets.append(sorted(int(x) for x in o.slot_token))
    assert sets[0] != sets[1] and sets[0] != sets[2] and sets[1] != sets[2]


# ---- planted mistakes ---------------------------------------------------------------------------
class WindowDropsNewest(WindowOracle):               # LIFO instead of FIFO
    def select_oldest(self):
        tok = self.slot_token.astype(np.float64)
        tok[self.slot_token < self.pinned] = -np.inf
        return int(np.argmax(tok))


class WindowForgetsPinned(WindowOracle):             # Window+i degenerates to Window
    def select_oldest(self):
        return int(np.argmin(self.slot_token))


class WindowPinsSlotsNotTokens(WindowOracle):        # off by one in what "the first i" means
    def select_oldest(self):
        tok = self.slot_token.astype(np.float64)
        tok[self.slot_token <= self.pinned] = np.inf
        return int(np.argmin(tok))


class H2OSelectBeforeAggregate(H2OOracle):           # the step's own weights come too late
    def step(self, q, k_new, v_new, force_victim=None):
        out, p = self.attend(q, k_new, v_new)
        s = self.scores(p)
        n = self.n
        if n + 1 <= self.k:
            self.acc[:n] += s[:n]
            self.update(-1, k_new, v_new)
            self.acc[n] = s[n]
            return StepResult(out, -1, float("inf"), None)
        el = self.eligible()
        cand = np.where(el, np.concatenate([self.acc, [0.0]]), np.inf)
        j = int(np.argmin(cand))
        self.acc += s[:n]
        self.update(j, k_new, v_new)
        self.acc[j] = s[n]
        return StepResult(out, j, 0.0, None)


class H2OWindowOffByOne(H2OOracle):                  # the incoming token is not counted into the window
    def eligible(self):
        el = np.zeros(self.n + 1, dtype=bool)
        el[: self.n] = self.slot_token[: self.n] < self.t - self.recent
        return el


class H2ONoWindow(H2OOracle):                        # recent tokens unprotected
    def eligible(self):
        el = np.ones(self.n + 1, dtype=bool)
        el[self.n] = False
        return el


class H2OKeepsLowest(H2OOracle):                     # wrong sign: the heaviest row leaves
    def step(self, q, k_new, v_new, force_victim=None):
        out, p = self.attend(q, k_new, v_new)
        s = self.scores(p)
        n = self.n
        total = np.concatenate([self.acc[:n] + s[:n], [s[n]]])
        self.acc[:n] = total[:n]
        if n + 1 <= self.k:
            self.update(-1, k_new, v_new)
            self.acc[n] = total[n]
            return StepResult(out, -1, float("inf"), None)
        cand = np.where(self.eligible(), total, -np.inf)
        j = int(np.argmax(cand))
        self.update(j, k_new, v_new)
        self.acc[j] = total[n]
        return StepResult(out, j, 0.0, None)


class H2OInheritsAggregate(H2OOracle):               # the new token keeps the victim's sum
    def step(self, q, k_new, v_new, force_victim=None):
        n_before = self.n
        keep = self.acc.copy()
        r = super().step(q, k_new, v_new, force_victim)
        if n_before == self.k and 0 <= r.evicted < self.k:
            self.acc[r.evicted] += keep[r.evicted]
        return r


class H2OThisStepOnly(H2OOracle):                    # no aggregation: TOVA with a window
    def step(self, q, k_new, v_new, force_victim=None):
        self.acc[:] = 0.0
        return super().step(q, k_new, v_new, force_victim)


class H2OFirstHeadOnly(H2OOracle):                   # no averaging over heads
    def scores(self, p):
        return p[0].copy()


class H2OHalfRoundedUp(H2OOracle):                   # heavy = ceil(k / 2)
    def __init__(self, k, H, H_kv, d, scale=None, heavy=None):
        super().__init__(k, H, H_kv, d, scale, heavy=(k + 1) // 2 if heavy is None else heavy)


@pytest.mark.parametrize("Mutant", [WindowDropsNewest, WindowForgetsPinned, WindowPinsSlotsNotTokens])
def test_window_mutants_are_caught(Mutant):
    with pytest.raises(AssertionError):
        pb.pin_window_closed_form(Mutant)


@pytest.mark.parametrize("Mutant", [H2OSelectBeforeAggregate, H2OWindowOffByOne, H2ONoWindow, H2OKeepsLowest,
                                    H2OInheritsAggregate, H2OThisStepOnly, H2OFirstHeadOnly, H2OHalfRoundedUp])
def test_h2o_mutants_are_caught(Mutant):
    caught = []
    for pin in (pb.pin_h2o_identical_keys, pb.pin_h2o_worked_example, pb.pin_h2o_brute_force):
        try:
            pin(Mutant)
        except AssertionError:
            caught.append(pin.__name__)
    assert caught, f"{Mutant.__name__} passes every pin"
    print(Mutant.__name__, "caught by", caught)
