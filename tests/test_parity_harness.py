"""CPU tests of the parity harness itself (tests/parity.py): the tiled whole-stream check must accept a
log that really is the oracle's and must reject a log with a single wrong victim or a wrong output
anywhere in the stream.  The "GPU" here is the oracle run sequentially from the empty cache, so these
tests say nothing about the kernels: they pin the checker."""
import numpy as np
import pytest

from oracle.tova_oracle import TovaOracle
from workloads import Stream, StreamSpec

import parity

SPEC = StreamSpec("harness", L=2, B=2, H=4, H_kv=2, d=16, dtype="f32", k=12, T=160, sink="first", n_sinks=1,
                  drift_sigma=0.01)
SEED, UNIT = 5, (1, 0)


def _sequential_log(spec, seed, unit, t_begin=0):
    st = Stream(spec, seed, device="cpu", layers=[unit[0]], seqs=[unit[1]])
    c = st.chunk(0, spec.T)
    q, kk, vv = (c[n][:, 0, 0].double().numpy() for n in "qkv")
    orc = TovaOracle(spec.k, spec.H, spec.H_kv, spec.d)
    out = np.zeros((spec.T, spec.H, spec.d), dtype=np.float32)
    ev = np.full(spec.T, -1, dtype=np.int32)
    for t in range(spec.T):
        if t < t_begin:
            orc.update(-1, kk[t], vv[t])
            continue
        r = orc.step(q[t], kk[t], vv[t])
        out[t], ev[t] = r.out, r.evicted
    return out, ev, orc


def _check(out, ev, n_windows, t_begin=0, laid_down=False):
    jobs = parity.tiled_jobs(SPEC, SEED, UNIT, out[t_begin:], ev, t_begin, SPEC.T, n_windows, out_t0=t_begin,
                             laid_down=laid_down)
    return parity.check_tiled([(UNIT, jobs, ev, SPEC.k)], workers=2)[0]


def test_tiled_check_accepts_the_sequential_run():
    out, ev, orc = _sequential_log(SPEC, SEED, UNIT)
    s = _check(out, ev, 7)
    assert s["steps"] == SPEC.T and s["windows"] == 7 and s["t_range"] == (0, SPEC.T)
    assert s["evict_steps"] == SPEC.T - SPEC.k and s["mismatches"] == 0 and s["max_rel_err"] < 1e-6
    assert np.array_equal(parity.replay_slot_tokens(ev, SPEC.k, SPEC.T), orc.slot_token)


def test_tiled_check_from_a_laid_down_state():
    out, ev, _ = _sequential_log(SPEC, SEED, UNIT, t_begin=SPEC.k)
    s = _check(out, ev, 3, t_begin=SPEC.k, laid_down=True)
    assert s["steps"] == SPEC.T - SPEC.k == s["evict_steps"] and s["mismatches"] == 0


@pytest.mark.parametrize("t_bad", [SPEC.k, 47, 101, SPEC.T - 1])
def test_tiled_check_rejects_one_wrong_victim(t_bad):
    out, ev, _ = _sequential_log(SPEC, SEED, UNIT)
    ev = ev.copy()
    ev[t_bad] = (ev[t_bad] + 1) % (SPEC.k + 1)            # a single wrong (but in-range) victim
    with pytest.raises(AssertionError):
        _check(out, ev, 7)


def test_tiled_check_rejects_one_wrong_output():
    out, ev, _ = _sequential_log(SPEC, SEED, UNIT)
    out = out.copy()
    out[77, 2, 5] += 1e-3
    with pytest.raises(AssertionError):
        _check(out, ev, 7)
