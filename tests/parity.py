"""GPU-vs-oracle parity harness.

run_gpu() drives the HIP library over a whole synthetic stream (inputs generated on the
device, chunk by chunk) and keeps the `evicted` log of every unit plus the outputs of the
sampled units.  check_unit() then re-creates one sampled (layer, sequence) unit on the CPU
from the same generator, steps the fp64 oracle through it and compares element by element.

Bars (written here, used by every parity test):
  * outputs: per output vector (one head of one step) max|gpu - ref| / max|ref| <= OUT_TOL
    (2e-2 for bf16, 1e-5 for fp32);
  * victims: identical at every step, except steps where the oracle's two lowest head-mean
    scores are closer than GAP_EXEMPT = 1e-6 *and* the GPU's choice is within that distance
    of the minimum; those are counted, reported, and the oracle then follows the GPU's
    choice so that both keep the same state;
  * final slot -> token map: identical; cached K/V rows: bit-identical to the stream rows.
"""
from __future__ import annotations

import numpy as np
import torch

from workloads import Stream, StreamSpec

OUT_TOL = {"bf16": 2e-2, "f32": 1e-5}
GAP_EXEMPT = 1e-6


def run_gpu(spec: StreamSpec, seed: int, units, n_splits: int = 0, chunk_steps: int = 256,
            single_step_calls: bool = False, device="cuda:0", prefill: bool = False, keep=None,
            progress: bool = False, n_pinned: int = 0, per_head: bool = False, use_prefill: bool = False,
            rope_base=None, keep_native: bool = False, policy="tova", h2o_heavy: int = 0):
    """units: list of (layer, seq) whose outputs are kept.  Returns a dict of CPU arrays.

    prefill=True skips the fill phase: the first k tokens are laid down directly (slot j holds
    token j, which is exactly what k fill steps produce -- App. B's no-op branch) and stepping
    starts at token k through tova_cache_set_tokens_seen.
    keep: list of (t0, t1) or (t0, t1, [indices into units]) step ranges whose outputs are kept, for
    all sampled units or for the named ones (default: all steps, all sampled units); with keep given,
    res["out"] is a dict keyed by those tuples, each [t1 - t0, n_units_kept, H, d] in the stream's dtype
    when keep_native, else float32.
    rope_base: not None -> the stream is taken as un-rotated q / k and stepped through
    tova_decode_steps_repositioned with that rotary base (Sec. 7.2).
    n_pinned / per_head: the TOVA+i / TOVA-head variants (App. A).  With per_head the results come
    back in the equivalent layer-mode view -- B * H_kv sequences of one KV head with G query heads
    each (the stream's flat element order is the same) -- and `units` are (layer, b * H_kv + kvh)."""
    from paper_2401_06104_amd import TovaCache

    dev = torch.device(device)
    cache = TovaCache(spec.L, spec.B, spec.k, spec.H, spec.H_kv, spec.d, dtype=spec.dtype,
                      n_splits=n_splits, device=dev, n_pinned=n_pinned, per_head=per_head, policy=policy,
                      h2o_heavy=h2o_heavy)
    stream = Stream(spec, seed, device=dev)
    evicted = torch.full((spec.T, *cache.state_shape), -1, dtype=torch.int32, device=dev)
    Bv = spec.B * spec.H_kv if per_head else spec.B              # sequences / heads per sequence of the view
    Hv, Hkv_v = (spec.H // spec.H_kv, 1) if per_head else (spec.H, spec.H_kv)
    ul = torch.tensor([u[0] for u in units], device=dev)
    ub = torch.tensor([u[1] for u in units], device=dev)
    t_begin = spec.k if prefill else 0
    default_keep = keep is None
    keep = [(t_begin, spec.T)] if keep is None else [tuple(r[:2]) + ((tuple(r[2]),) if len(r) > 2 else ()) for r in keep]
    outs = {r: [] for r in keep}
    sel = {r: (torch.tensor([units[i][0] for i in r[2]], device=dev), torch.tensor([units[i][1] for i in r[2]], device=dev))
           if len(r) > 2 else (ul, ub) for r in keep}
    if prefill:
        assert spec.T > spec.k
        K, V = cache.K, cache.V
        for t0 in range(0, spec.k, chunk_steps):
            t1 = min(spec.k, t0 + chunk_steps)
            c = stream.chunk(t0, t1, need_q=False)
            K[:, :, :, t0:t1, :] = c["k"].permute(1, 2, 3, 0, 4)
            V[:, :, :, t0:t1, :] = c["v"].permute(1, 2, 3, 0, 4)
            if callable(progress) and (t0 // chunk_steps) % 32 == 31:
                torch.cuda.synchronize(dev)
                progress(f"[parity]   rows of tokens 0..{t1 - 1} of {spec.k} laid down")
        cache.occupancy.fill_(spec.k)
        cache.slot_token.copy_(torch.arange(spec.k, dtype=torch.int32, device=dev).expand_as(cache.slot_token))
        cache.set_tokens_seen(spec.k)
    for t0 in range(t_begin, spec.T, chunk_steps):
        t1 = min(spec.T, t0 + chunk_steps)
        c = stream.chunk(t0, t1)
        out = torch.empty_like(c["q"])
        if single_step_calls:
            for i in range(t1 - t0):
                cache.decode_step(c["q"][i], c["k"][i], c["v"][i], out[i], evicted[t0 + i])
        elif rope_base is not None:
            cache.decode_steps_repositioned(c["q"], c["k"], c["v"], out, evicted[t0:t1], rope_base=rope_base)
        elif use_prefill:          # the tokens of a chunk handed over as a prompt (tova_prefill)
            cache.prefill(c["q"], c["k"], c["v"], out, evicted[t0:t1])
        else:
            cache.decode_steps(c["q"], c["k"], c["v"], out, evicted[t0:t1])
        for r in keep:
            lo, hi = max(r[0], t0), min(r[1], t1)
            if lo < hi:
                o = out[lo - t0:hi - t0].view(-1, spec.L, Bv, Hv, spec.d)[:, sel[r][0], sel[r][1]]
                outs[r].append((o if keep_native else o.float()).cpu())
        if progress and (t0 // chunk_steps) % 16 == 0:
            torch.cuda.synchronize(dev)
            (progress if callable(progress) else (lambda m: print(m, flush=True)))(f"[parity]   gpu at step {t1}/{spec.T}")
    torch.cuda.synchronize(dev)
    assert int(cache.error_flag.item()) == 0, "a multi-step launch gave up waiting (error flag set)"
    res = {
        "out": {r: ((torch.cat(v) if keep_native else torch.cat(v).numpy()) if v else None)
                for r, v in outs.items()},                                          # [t, n_units, H, d]
        "evicted": evicted.view(spec.T, spec.L, Bv).cpu().numpy(),                  # [T, L, B]
        "slot_token": cache.slot_token.view(spec.L, Bv, spec.k).cpu().numpy(),      # [L, B, k]
        "occupancy": cache.occupancy.view(spec.L, Bv).cpu().numpy(),
        "K": cache.K.view(spec.L, Bv, Hkv_v, spec.k, spec.d)[ul, ub].float().cpu().numpy(),   # [n_units, H_kv, k, d]
        "V": cache.V.view(spec.L, Bv, Hkv_v, spec.k, spec.d)[ul, ub].float().cpu().numpy(),
        "layout": (cache.layout.n_splits, cache.layout.rows_per_split, cache.layout.block_threads,
                   cache.layout.grid_blocks),
        "unit_workgroups": int(cache.layout.unit_workgroups),
        "prefill_group": int(cache.layout.prefill_group),
        "tokens_seen": cache.tokens_seen,
        "prefill": prefill,
    }
    if policy == "h2o":
        res["h2o_acc"] = cache.h2o_acc.view(spec.L, Bv, spec.k).cpu().numpy()
    if default_keep:
        res["out"] = res["out"][(t_begin, spec.T)]
        res["out_t0"] = t_begin
    cache.destroy()
    return res


def _compare_step(spec, unit, t, orc, q, kk, vv, gpu_out_t, ge, stats, tol):
    """One oracle step against the GPU's output / victim of the same step (bars in the header)."""
    out, p = orc.attend(q, kk, vv)
    if gpu_out_t is not None:
        g = gpu_out_t.astype(np.float64)
        err = np.abs(g - out).max(axis=1) / np.maximum(np.abs(out).max(axis=1), 1e-30)
        worst = float(err.max())
        assert worst <= tol, f"unit {unit} step {t}: output rel err {worst:.3e} > {tol}"
        stats["max_rel_err"] = max(stats["max_rel_err"], worst)
    ge = int(ge)
    if orc.n + 1 <= spec.k:
        assert ge == -1, f"unit {unit} step {t}: GPU evicted {ge} while filling"
        orc.update(-1, kk, vv)
        return
    s = orc.scores(p)
    j, gap = orc.select(s, orc.pinned)
    stats["evict_steps"] += 1
    stats["min_gap"] = min(stats["min_gap"], gap)
    if gap < GAP_EXEMPT:
        stats["near_tie_steps"] += 1
    assert 0 <= ge <= spec.k, f"unit {unit} step {t}: GPU victim {ge} out of range"
    if ge != j:
        ok = gap < GAP_EXEMPT and (s[ge] - s[j]) < GAP_EXEMPT
        assert ok, (f"unit {unit} step {t}: GPU victim {ge} != oracle {j}, "
                    f"gap {gap:.3e}, s[gpu]-min {s[ge] - s[j]:.3e}")
        stats["mismatches"] += 1
        stats["max_gap_at_mismatch"] = max(stats["max_gap_at_mismatch"], float(s[ge] - s[j]))
    orc.update(ge, kk, vv)     # == j unless a counted near-tie


def _new_stats(unit, steps):
    return dict(unit=unit, steps=steps, evict_steps=0, near_tie_steps=0, mismatches=0, max_rel_err=0.0,
                max_gap_at_mismatch=0.0, min_gap=float("inf"))


def check_unit(spec: StreamSpec, seed: int, unit, gpu_out, gpu_evicted, gpu_slot_token, gpu_K, gpu_V,
               t_stop=None, prefill=False, out_t0=0, n_pinned=0, rope_base=None):
    """Steps the oracle over unit=(layer, seq) from the start of the stream (or, with prefill,
    from the state "slot j holds token j") and compares with the GPU's log.
    gpu_out [t, H, d] holds steps out_t0.. ; gpu_evicted [T]; gpu_slot_token [k]; gpu_K / gpu_V
    [H_kv, k, d] are the final cache (compared only when the whole stream is checked).
    Returns a dict of statistics; raises AssertionError on any violation."""
    from oracle.tova_oracle import TovaOracle
    from oracle.tova_positions import TovaPositionsOracle

    l, b = unit
    T = spec.T if t_stop is None else t_stop
    tol = OUT_TOL[spec.dtype]
    st = Stream(spec, seed, device="cpu", layers=[l], seqs=[b])
    if rope_base is None:
        orc = TovaOracle(spec.k, spec.H, spec.H_kv, spec.d, pinned=n_pinned)
    else:      # (rope_base <= 0 asks the library for its default, 10000)
        orc = TovaPositionsOracle(spec.k, spec.H, spec.H_kv, spec.d, pinned=n_pinned,
                                  base=rope_base if rope_base > 0 else 10000.0)
    stats = _new_stats(unit, T)
    kk_all, vv_all = [], []
    for t0 in range(0, T, 512):
        t1 = min(T, t0 + 512)
        filling = prefill and t1 <= spec.k
        c = st.chunk(t0, t1, need_q=not filling)
        kk = c["k"][:, 0, 0].double().numpy()
        vv = c["v"][:, 0, 0].double().numpy()
        if t_stop is None:
            kk_all.append(kk); vv_all.append(vv)
        q = None if filling else c["q"][:, 0, 0].double().numpy()
        for i in range(t1 - t0):
            t = t0 + i
            if prefill and t < spec.k:
                orc.update(-1, kk[i], vv[i])         # the no-op branch: the row takes slot t
                continue
            g = gpu_out[t - out_t0] if gpu_out is not None and t >= out_t0 else None
            _compare_step(spec, unit, t, orc, q[i], kk[i], vv[i], g, gpu_evicted[t], stats, tol)
    if t_stop is None:
        assert np.array_equal(orc.slot_token, gpu_slot_token.astype(np.int64)), f"unit {unit}: slot_token differs"
        n = orc.n
        assert np.array_equal(orc.K[:, :n], gpu_K[:, :n].astype(np.float64)), f"unit {unit}: cached K differs"
        assert np.array_equal(orc.V[:, :n], gpu_V[:, :n].astype(np.float64)), f"unit {unit}: cached V differs"
        # and the cached rows are the raw stream rows of the tokens the map names
        kk_all, vv_all = np.concatenate(kk_all), np.concatenate(vv_all)
        for slot in range(n):
            tk = int(gpu_slot_token[slot])
            assert np.array_equal(gpu_K[:, slot].astype(np.float64), kk_all[tk])
            assert np.array_equal(gpu_V[:, slot].astype(np.float64), vv_all[tk])
    return stats


def check_window(spec: StreamSpec, seed: int, unit, t0, t1, slot_token_t0, gpu_out, gpu_evicted, rope_base=None):
    """PROPERTY check, not parity from the start: every step in [t0, t1) is a correct TOVA
    transition from the state the run itself was in at t0.  That state is rebuilt from the
    stream (rows) and the integer slot -> token map implied by the GPU's evicted log, so an
    earlier wrong victim would go unnoticed here; what is checked is that, far into a long
    stream, outputs and victims still follow from the cached rows.
    gpu_out [t1 - t0, H, d], gpu_evicted [T]."""
    from oracle.tova_oracle import TovaOracle

    l, b = unit
    tol = OUT_TOL[spec.dtype]
    st = Stream(spec, seed, device="cpu", layers=[l], seqs=[b])
    need = sorted(set(int(x) for x in slot_token_t0 if x >= 0))
    rows_k, rows_v = {}, {}
    if rope_base is None:
        orc = TovaOracle(spec.k, spec.H, spec.H_kv, spec.d)
    else:      # un-rotated stream, positions re-assigned before every attention (Sec. 7.2)
        from oracle.tova_positions import TovaPositionsOracle
        orc = TovaPositionsOracle(spec.k, spec.H, spec.H_kv, spec.d, base=rope_base if rope_base > 0 else 10000.0)
    stats = _new_stats(unit, t1 - t0)
    needed = set(need)
    for a in range(0, t1, 2048):
        bnd = min(t1, a + 2048)
        c = st.chunk(a, bnd, need_q=bnd > t0)
        if a < t0:
            kk = c["k"][:, 0, 0]
            vv = c["v"][:, 0, 0]
            for t in range(a, min(bnd, t0)):
                if t in needed:
                    rows_k[t] = kk[t - a].double().numpy()
                    rows_v[t] = vv[t - a].double().numpy()
        if bnd > t0:
            if orc.t == 0:       # lay the state down once, just before the first checked step
                for slot, tk in enumerate(slot_token_t0):
                    if tk >= 0:
                        orc.K[:, slot] = rows_k[int(tk)]
                        orc.V[:, slot] = rows_v[int(tk)]
                orc.slot_token[:] = slot_token_t0
                orc.n = int((slot_token_t0 >= 0).sum())
                orc.t = t0
            q = c["q"][:, 0, 0].double().numpy()
            kk = c["k"][:, 0, 0].double().numpy()
            vv = c["v"][:, 0, 0].double().numpy()
            for t in range(max(a, t0), bnd):
                _compare_step(spec, unit, t, orc, q[t - a], kk[t - a], vv[t - a], gpu_out[t - t0],
                              gpu_evicted[t], stats, tol)
    return stats


def replay_slot_tokens(evicted_unit, k, t_stop):
    """slot -> token map after t_stop steps, from one unit's evicted log alone (integers)."""
    st = np.full(k, -1, dtype=np.int64)
    for t in range(t_stop):
        if t < k:
            st[t] = t
        else:
            e = int(evicted_unit[t])
            if e < k:
                st[e] = t
    return st


def _check_unit_star(args):
    try:
        from threadpoolctl import threadpool_limits
        limiter = threadpool_limits(limits=1)            # one core per worker (the pool is the parallelism)
    except Exception:                                     # pragma: no cover
        limiter = None
    r = check_unit(*args)
    del limiter
    return r


def check_units(spec, seed, units, res, workers: int = 1, t_stop=None, out=None, out_t0=None, n_pinned=0,
                rope_base=None, progress=None):
    """Checks every sampled unit; with workers > 1 in spawned CPU-only processes.  progress: called with
    a line of text whenever a unit is done (long runs must show that they are alive)."""
    jobs = []
    out = res["out"] if out is None else out
    out_t0 = res.get("out_t0", 0) if out_t0 is None else out_t0
    for ui, (l, b) in enumerate(units):
        jobs.append((spec, seed, (l, b), out[:, ui], res["evicted"][:, l, b],
                     res["slot_token"][l, b], res["K"][ui], res["V"][ui], t_stop, res.get("prefill", False),
                     out_t0, n_pinned, rope_base))
    if workers <= 1 or len(jobs) == 1:
        return [check_unit(*j) for j in jobs]
    import multiprocessing as mp
    with mp.get_context("spawn").Pool(min(workers, len(jobs))) as pool:
        results = []
        for i, r in enumerate(pool.imap(_check_unit_star, jobs, chunksize=1)):
            results.append(r)
            if progress:
                progress(f"[parity]   unit {r['unit']} done ({i + 1}/{len(jobs)}): {r['mismatches']} mismatches, "
                         f"{r['near_tie_steps']} near-tie steps, max rel err {r['max_rel_err']:.2e}")
        return results


def check_global_invariants(spec, res):
    """Properties of the whole run that hold at any size (every unit, every step)."""
    ev = res["evicted"]
    k = spec.k
    fill = min(k, spec.T)
    assert (ev[:fill] == -1).all(), "a unit evicted before its cache was full"  # (prefill: never written)
    if spec.T > k:
        assert ((ev[k:] >= 0) & (ev[k:] <= k)).all(), "victim out of range after capacity"
    assert (res["occupancy"] == min(spec.T, k)).all()
    assert res["tokens_seen"] == spec.T
    # replay the evicted log on integers alone: it must reproduce the final slot -> token map
    st = np.full((spec.L, spec.B, k), -1, dtype=np.int64)
    li, bi = np.meshgrid(np.arange(spec.L), np.arange(spec.B), indexing="ij")
    for t in range(spec.T):
        if t < k:
            st[:, :, t] = t
        else:
            e = ev[t]
            m = e < k
            st[li[m], bi[m], e[m]] = t
    assert np.array_equal(st, res["slot_token"].astype(np.int64)), "slot_token inconsistent with the evicted log"
    # retained tokens are distinct
    for l in range(spec.L):
        for b in range(spec.B):
            row = st[l, b][st[l, b] >= 0]
            assert len(set(row.tolist())) == len(row)


# ---------------------------------------------------------------------------------------------
# Parity over a whole long stream, by tiling it with windows that are checked on separate cores.
#
# The stream [t_begin, t_end) of one unit is cut into contiguous windows.  Each window starts from
# the state the run was in there: the slot -> token map that the GPU's integer `evicted` log implies
# (replayed on integers) and, for every retained token, its K / V rows REGENERATED from the seeded
# stream -- nothing of the GPU's floating-point results enters the oracle.  Inside a window every
# step is compared as in check_unit (outputs within tolerance; victim equal, or a counted near tie
# that the oracle then follows).  The first window starts from the empty multi-state (or from
# "slot j holds token j" when the run laid the first k tokens down).  If every window passes, every
# logged victim from the first step on is the oracle's victim given the victims before it, which by
# induction is parity over the whole stream from the empty cache -- the same statement check_unit
# makes, computed in parallel.  A single wrong victim anywhere fails the window that contains it.
# ---------------------------------------------------------------------------------------------
def _window_job(job):
    """One window of one unit (runs in a spawned CPU-only process).  job: dict, see check_tiled."""
    from oracle.tova_oracle import TovaOracle
    try:
        from threadpoolctl import threadpool_limits
        limiter = threadpool_limits(limits=1)            # one core per worker
    except Exception:                                     # pragma: no cover
        limiter = None
    spec, unit, a, b = job["spec"], job["unit"], job["a"], job["b"]
    tol = OUT_TOL[spec.dtype]
    if job["rope_base"] is None:
        orc = TovaOracle(spec.k, spec.H, spec.H_kv, spec.d, pinned=job["n_pinned"])
    else:
        from oracle.tova_positions import TovaPositionsOracle
        rb = job["rope_base"]
        orc = TovaPositionsOracle(spec.k, spec.H, spec.H_kv, spec.d, pinned=job["n_pinned"],
                                  base=rb if rb > 0 else 10000.0)
    st = np.asarray(job["slot_token"], dtype=np.int64)
    held = st >= 0
    n = int(held.sum())
    assert held[:n].all(), "occupied slots must be the first ones"
    orc.K[:, :n] = np.asarray(job["rows_k"], dtype=np.float64)        # [H_kv, n, d]
    orc.V[:, :n] = np.asarray(job["rows_v"], dtype=np.float64)
    orc.slot_token[:] = st
    orc.n = n
    orc.t = a
    q = np.asarray(job["q"], dtype=np.float64)
    kk = np.asarray(job["k"], dtype=np.float64)
    vv = np.asarray(job["v"], dtype=np.float64)
    g = None if job["out"] is None else np.asarray(job["out"], dtype=np.float64)
    ev = job["evicted"]
    stats = _new_stats(unit, b - a)
    stats["window"] = (a, b)
    for i in range(b - a):
        _compare_step(spec, unit, a + i, orc, q[i], kk[i], vv[i], None if g is None else g[i], ev[i], stats, tol)
    stats["slot_token_end"] = orc.slot_token.copy()
    del limiter
    return stats


def _to_f32(x):
    return x.float().numpy() if isinstance(x, torch.Tensor) else np.asarray(x, dtype=np.float32)


def tiled_jobs(spec: StreamSpec, seed: int, unit, gpu_out, gpu_evicted, t_begin: int, t_end: int, n_windows: int,
               out_t0: int = 0, laid_down: bool = False, rope_base=None, n_pinned: int = 0):
    """The window jobs of one unit (see the comment above).  gpu_out [t_end - out_t0 or more, H, d] holds the
    unit's outputs from step out_t0 on (torch tensor or array; None: outputs are not compared);
    gpu_evicted [>= t_end] is the unit's log.  laid_down: the run put tokens 0..k-1 into slots 0..k-1
    directly and t_begin == k.  The windows tile [t_begin, t_end) without a gap (asserted)."""
    l, b = unit
    k = spec.k
    assert 0 <= t_begin < t_end <= spec.T and n_windows >= 1
    assert t_begin == (k if laid_down else 0), "the first window must start from a known state"
    st = Stream(spec, seed, device="cpu", layers=[l], seqs=[b])
    kk_all, vv_all, q_all = [], [], []
    for a in range(0, t_end, 2048):                         # (contiguous from 0: drifting streams need it)
        c = st.chunk(a, min(t_end, a + 2048), need_q=min(t_end, a + 2048) > t_begin)
        kk_all.append(c["k"][:, 0, 0]); vv_all.append(c["v"][:, 0, 0])
        if c["q"] is not None:
            q_all.append((a, c["q"][:, 0, 0]))
    kk_all, vv_all = torch.cat(kk_all), torch.cat(vv_all)              # [t_end, H_kv, d], storage dtype
    q0 = q_all[0][0]
    q_all = torch.cat([x for _, x in q_all])                           # steps q0 .. t_end
    bounds = [t_begin + (t_end - t_begin) * i // n_windows for i in range(n_windows + 1)]
    bounds = sorted(set(bounds))
    ev = np.asarray(gpu_evicted)
    slot_token = np.full(k, -1, dtype=np.int64)
    t = 0
    jobs = []
    for a, bnd in zip(bounds[:-1], bounds[1:]):
        while t < a:                                        # the integer log, replayed up to the window's start
            if t < k:
                assert laid_down or int(ev[t]) == -1, f"unit {unit} step {t}: victim logged while filling"
                slot_token[t] = t
            else:
                e = int(ev[t])
                assert 0 <= e <= k, f"unit {unit} step {t}: victim {e} out of range"
                if e < k:
                    slot_token[e] = t
            t += 1
        n = int((slot_token >= 0).sum())
        tok = torch.from_numpy(slot_token[:n].copy())
        jobs.append(dict(spec=spec, unit=unit, a=a, b=bnd, slot_token=slot_token.copy(),
                         rows_k=_to_f32(kk_all[tok].permute(1, 0, 2)), rows_v=_to_f32(vv_all[tok].permute(1, 0, 2)),
                         q=_to_f32(q_all[a - q0:bnd - q0]), k=_to_f32(kk_all[a:bnd]), v=_to_f32(vv_all[a:bnd]),
                         out=None if gpu_out is None else _to_f32(gpu_out[a - out_t0:bnd - out_t0]),
                         evicted=ev[a:bnd].copy(), rope_base=rope_base, n_pinned=n_pinned))
    assert jobs[0]["a"] == t_begin and jobs[-1]["b"] == t_end
    assert all(x["b"] == y["a"] for x, y in zip(jobs[:-1], jobs[1:])), "windows must tile the stream without a gap"
    return jobs


def merge_window_stats(unit, stats_list, gpu_evicted, k):
    """Folds the windows' statistics of one unit into one record; checks that they tile and that each
    window ended in the state the next one started from (the log's replay, again on integers)."""
    ws = sorted(stats_list, key=lambda s: s["window"][0])
    assert all(x["window"][1] == y["window"][0] for x, y in zip(ws[:-1], ws[1:])), "windows do not tile"
    tot = _new_stats(unit, sum(s["steps"] for s in ws))
    tot["windows"] = len(ws)
    tot["t_range"] = (ws[0]["window"][0], ws[-1]["window"][1])
    for s in ws:
        for key in ("evict_steps", "near_tie_steps", "mismatches"):
            tot[key] += s[key]
        for key in ("max_rel_err", "max_gap_at_mismatch"):
            tot[key] = max(tot[key], s[key])
        tot["min_gap"] = min(tot["min_gap"], s["min_gap"])
        end = s["window"][1]
        assert np.array_equal(s["slot_token_end"], replay_slot_tokens(gpu_evicted, k, end)), \
            f"unit {unit}: state after window {s['window']} is not what the log implies"
    return tot


def check_tiled(units_jobs, workers: int = 16, progress=None):
    """units_jobs: list of (unit, jobs, gpu_evicted, k).  Runs every window of every unit on a pool of
    CPU-only processes (largest first) and returns one merged statistics record per unit.  progress:
    called with a line of text whenever a window is done."""
    import multiprocessing as mp
    flat = [(ui, j) for ui, (_, jobs, _, _) in enumerate(units_jobs) for j in jobs]
    order = sorted(range(len(flat)), key=lambda i: -(flat[i][1]["b"] - flat[i][1]["a"]))
    with mp.get_context("spawn").Pool(max(1, min(workers, len(flat)))) as pool:
        results = []
        for i, r in enumerate(pool.imap(_window_job, [flat[i][1] for i in order], chunksize=1)):
            results.append(r)
            if progress:
                progress(f"[parity]   unit {r['unit']} window {r['window']} done ({i + 1}/{len(flat)})")
    per_unit = {ui: [] for ui in range(len(units_jobs))}
    for i, r in zip(order, results):
        per_unit[flat[i][0]].append(r)
    return [merge_window_stats(units_jobs[ui][0], per_unit[ui], units_jobs[ui][2], units_jobs[ui][3])
            for ui in range(len(units_jobs))]


def check_final_rows(spec: StreamSpec, seed: int, unit, gpu_slot_token, gpu_K, gpu_V):
    """The rows the GPU's cache holds at the end are, bit for bit, the stream rows of the tokens its
    slot -> token map names.  gpu_K / gpu_V [H_kv, k, d] (float32 views of the stored values)."""
    l, b = unit
    st = Stream(spec, seed, device="cpu", layers=[l], seqs=[b])
    kk, vv = [], []
    for a in range(0, spec.T, 2048):
        c = st.chunk(a, min(spec.T, a + 2048), need_q=False)
        kk.append(c["k"][:, 0, 0]); vv.append(c["v"][:, 0, 0])
    kk, vv = torch.cat(kk).float().numpy(), torch.cat(vv).float().numpy()
    tok = np.asarray(gpu_slot_token, dtype=np.int64)
    held = tok >= 0
    assert np.array_equal(np.asarray(gpu_K)[:, held], kk[tok[held]].transpose(1, 0, 2)), f"unit {unit}: cached K rows differ"
    assert np.array_equal(np.asarray(gpu_V)[:, held], vv[tok[held]].transpose(1, 0, 2)), f"unit {unit}: cached V rows differ"
