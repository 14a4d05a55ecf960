#!/usr/bin/env python3
"""Benchmark of the TOVA decode step on one MI355X.

Workload (the configuration the headline metric is quoted on): Mistral-7B-shaped GQA layer,
32 query heads / 8 KV heads, head_dim 128, bf16, batch 64, cache capacity k = 1024.  The cache
is first filled through the same API (1024 untimed steps), then `--steps` decode steps at full
occupancy are timed in one tova_decode_steps call with all inputs already resident in HBM.
One "step" = one token for each of the 64 sequences = one pass of the fused kernel over every
(sequence, KV head); the timed call runs all its steps in ONE launch of that kernel when the
device can hold all its workgroups at once (otherwise one launch per step).

Prints ONE JSON line.  `roofline` is the fused step
kernel against the HBM roofline: algorithmic bytes per launch (bytes per step x steps per launch)
/ average launch duration measured with HIP events on the launch stream over the timed region.  `cpu_baseline` is the fp64 oracle
timed on host cores on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth
# Bytes that left L2 per decode step of the step kernel on this workload, from rocprofv3 --pmc FETCH_SIZE
# and WRITE_SIZE runs of this script (256 steps per launch), each scaled by what the same counter reads
# for a 1 GiB copy kernel (summary: profiles/tova_step_kernel_c3_mistral_gqa.txt).  Not measured live.
PROFILED_TRAFFIC_BYTES_PER_STEP = 274.2e6
# ... and of the 32-layer variant (workgroup-per-unit form), profiles/tova_step_kernel_unit_c3_mistral_gqa_x32.txt
PROFILED_TRAFFIC_BYTES_PER_STEP_X32 = 8648.6e6


def algorithmic_bytes_per_step(spec) -> int:
    """What the method itself must move per decode step at full occupancy, all units:
    K and V read once, q read, out written, the new k/v read, the victim slot written,
    evicted + slot_token written."""
    e = 2 if spec.dtype == "bf16" else 4
    per_unit = (2 * spec.k * spec.H_kv * spec.d * e      # K + V stream
                + 2 * spec.H * spec.d * e                # q in, out out
                + 2 * spec.H_kv * spec.d * e             # k_new, v_new in
                + 2 * spec.H_kv * spec.d * e             # slot overwrite
                + 8)                                     # evicted, slot_token
    return per_unit * spec.L * spec.B


def gpu_leg(spec, seed, steps, warmup, device, chunk=256, prefill=False, also_prompt=False, repositioned=False,
            repeats=0):
    """Fills the cache (through the entry point, or with prefill=True by laying the first k tokens down),
    runs `warmup` untimed steps, then times ONE call of `steps` steps with HIP events on the stream the
    kernels are launched on.  repeats > 0: the same number of further steps is timed that many more
    times (fresh tokens each time) and the per-step times of all 1 + repeats calls are returned too."""
    import torch
    from paper_2401_06104_amd import TovaCache
    from workloads import Stream

    dev = torch.device(device)
    cache = TovaCache(spec.L, spec.B, spec.k, spec.H, spec.H_kv, spec.d, dtype=spec.dtype, device=dev)
    stream = Stream(spec, seed, device=dev)
    need = spec.k + warmup + steps * (1 + repeats)
    assert need <= spec.T, f"stream too short: need {need} tokens, spec has {spec.T}"

    # repositioned: the stream is taken as un-rotated q / k and stepped through
    # tova_decode_steps_repositioned (positions re-assigned and rotary embedding applied in the kernel)
    step_fn = ((lambda *a: cache.decode_steps_repositioned(*a, rope_base=10000.0)) if repositioned
               else cache.decode_steps)

    def run(t0, t1, keep=False):
        outs = []
        for a in range(t0, t1, chunk):
            b = min(t1, a + chunk)
            c = stream.chunk(a, b)
            out = torch.empty_like(c["q"])
            ev = torch.empty(b - a, spec.L, spec.B, dtype=torch.int32, device=dev)
            step_fn(c["q"], c["k"], c["v"], out, ev)
            if keep:
                outs.append(ev)
        return outs

    if prefill:
        # lay the first k tokens down directly (slot j = token j, what k fill steps produce), so that
        # every step-kernel dispatch of this process runs at full occupancy (used for profiling)
        for a in range(0, spec.k, chunk):
            b = min(spec.k, a + chunk)
            c = stream.chunk(a, b, need_q=False)
            cache.K[:, :, :, a:b, :] = c["k"].permute(1, 2, 3, 0, 4)
            cache.V[:, :, :, a:b, :] = c["v"].permute(1, 2, 3, 0, 4)
        cache.occupancy.fill_(spec.k)
        cache.slot_token.copy_(torch.arange(spec.k, dtype=torch.int32, device=dev).expand_as(cache.slot_token))
        cache.set_tokens_seen(spec.k)
    else:
        run(0, spec.k)                               # fill: untimed, same entry point
    if warmup:
        run(spec.k, spec.k + warmup)                 # untimed full-occupancy steps
    # stage every timed input in HBM first
    t0 = spec.k + warmup
    qs, ks, vs = [], [], []
    for a in range(t0, t0 + steps, chunk):
        c = stream.chunk(a, min(t0 + steps, a + chunk))
        qs.append(c["q"]); ks.append(c["k"]); vs.append(c["v"])
    q, k_new, v_new = torch.cat(qs), torch.cat(ks), torch.cat(vs)
    del qs, ks, vs
    out = torch.empty_like(q)
    evicted = torch.empty(steps, spec.L, spec.B, dtype=torch.int32, device=dev)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize(dev)
    w0 = time.perf_counter()
    e0.record()
    step_fn(q, k_new, v_new, out, evicted)
    e1.record()
    torch.cuda.synchronize(dev)
    wall = time.perf_counter() - w0
    ev_ms = e0.elapsed_time(e1)
    ev_host = evicted.cpu()
    ok = (bool(((ev_host >= 0) & (ev_host <= spec.k)).all()) and cache.tokens_seen == spec.k + warmup + steps
          and int(cache.error_flag.item()) == 0)
    rep_ms = [ev_ms / steps]
    for r in range(repeats):
        a0 = t0 + steps * (1 + r)
        qs, ks, vs = [], [], []
        for a in range(a0, a0 + steps, chunk):
            c = stream.chunk(a, min(a0 + steps, a + chunk))
            qs.append(c["q"]); ks.append(c["k"]); vs.append(c["v"])
        q, k_new, v_new = torch.cat(qs), torch.cat(ks), torch.cat(vs)
        del qs, ks, vs
        torch.cuda.synchronize(dev)
        e0.record()
        step_fn(q, k_new, v_new, out, evicted)
        e1.record()
        torch.cuda.synchronize(dev)
        rep_ms.append(e0.elapsed_time(e1) / steps)
        ok = ok and int(cache.error_flag.item()) == 0
    lay = cache.layout
    multi = cache.multi_step_blocks
    plan = dict(multi_step_blocks=multi, n_splits=lay.n_splits, rows_per_split=lay.rows_per_split, block_threads=lay.block_threads,
                grid_blocks=lay.grid_blocks, lds_bytes=lay.lds_bytes, unit_workgroups=int(lay.unit_workgroups),
                prefill_group=int(lay.prefill_group), service_wave=int(lay.service_wave))
    prompt_ms = None
    if also_prompt:
        # the same tokens once more, handed over as a prompt (tova_prefill: groups of tokens share one
        # pass over the cache); only the time is of interest here
        e0.record()
        cache.prefill(q, k_new, v_new, out, evicted)
        e1.record()
        torch.cuda.synchronize(dev)
        prompt_ms = e0.elapsed_time(e1)
        ev2 = evicted.cpu()
        ok = ok and bool(((ev2 >= 0) & (ev2 <= spec.k)).all()) and int(cache.error_flag.item()) == 0
    cache.destroy()
    return dict(wall_s=wall, event_ms=ev_ms, plan=plan, sane=ok, prompt_event_ms=prompt_ms, repeat_ms_per_step=rep_ms,
                new_token_dropped_frac=float((ev_host == spec.k).float().mean()))


def leg_record(workload, spec, g, steps, kernel):
    """One configuration's line: time per step, throughput and the fused step kernel against the HBM roofline."""
    ms = g["event_ms"] / steps
    ab = algorithmic_bytes_per_step(spec)
    spl = steps if g["plan"]["multi_step_blocks"] else 1
    rec = {"workload": workload, "steps": steps, "ms_per_step": ms, "decode_steps_per_s": 1e3 / ms,
           "sequence_steps_per_s": 1e3 / ms * spec.L * spec.B,
           "roofline": {"bound": "hbm", "achieved": ab / (ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": ab / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "kernel": kernel, "steps_per_launch": spl,
                        "algorithmic_bytes_per_step": ab, "avg_launch_us": ms * 1e3 * spl},
           "plan": g["plan"], "sane": g["sane"]}
    if len(g["repeat_ms_per_step"]) > 1:
        r = sorted(g["repeat_ms_per_step"])
        rec["repeat_ms_per_step"] = {"n": len(r), "median": r[len(r) // 2], "min": r[0], "max": r[-1]}
    return rec


def _oracle_worker(args):
    """One sequence of the workload through the fp64 oracle: fill, then timed steps."""
    spec, seed, b, n_timed = args
    import numpy as np  # noqa: F401
    from oracle.tova_oracle import TovaOracle
    from workloads import Stream
    try:
        from threadpoolctl import threadpool_limits
        limiter = threadpool_limits(limits=1)       # one thread per worker: cores = workers
    except Exception:                                # pragma: no cover
        limiter = None
    st = Stream(spec, seed, device="cpu", layers=[0], seqs=[b])
    orc = TovaOracle(spec.k, spec.H, spec.H_kv, spec.d)
    c = st.chunk(0, spec.k + n_timed)
    q, kk, vv = (c[n][:, 0, 0].double().numpy() for n in "qkv")
    for t in range(spec.k):
        orc.step(q[t], kk[t], vv[t])
    t0 = time.perf_counter()
    for t in range(spec.k, spec.k + n_timed):
        orc.step(q[t], kk[t], vv[t])
    dt = time.perf_counter() - t0
    del limiter
    return dt


def cpu_leg(spec, seed, n_timed=512):
    """The fp64 oracle as it stands on the host's cores: one sequence per core on min(16, cores) cores
    at once (a one-GPU machine's share is 16, whatever os.cpu_count() shows), then one sequence alone on one core."""
    import multiprocessing as mp
    cores = max(1, min(16, os.cpu_count() or 1, spec.B))
    jobs = [(spec, seed, b, n_timed) for b in range(cores)]
    t0 = time.perf_counter()
    with mp.get_context("spawn").Pool(cores) as pool:
        times = pool.map(_oracle_worker, jobs)
        one = pool.map(_oracle_worker, [(spec, seed, 0, n_timed // 2)])[0]     # alone: the other workers idle
    wall_total = time.perf_counter() - t0
    timed_wall = max(times)                          # workers run concurrently
    unit_steps_per_s = cores * n_timed / timed_wall
    one_core = (n_timed // 2) / one
    return dict(value=unit_steps_per_s / (spec.L * spec.B), unit="decode steps/s", cores=cores, kind="oracle",
                sample=(f"{cores} of {spec.B} sequences, one per core, {n_timed} full-occupancy steps each after "
                        f"an untimed {spec.k}-step fill; unit-steps/s scaled by 1/{spec.L * spec.B} units per step"),
                unit_steps_per_s=unit_steps_per_s, wall_s_including_fill=wall_total,
                one_core={"value": one_core / (spec.L * spec.B), "unit": "decode steps/s", "cores": 1,
                          "unit_steps_per_s": one_core,
                          "sample": f"sequence 0 alone on one core, {n_timed // 2} full-occupancy steps after the fill"},
                os_cpu_count=os.cpu_count())


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2048)
    ap.add_argument("--warmup", type=int, default=64)
    ap.add_argument("--seed", type=int, default=3)
    ap.add_argument("--layers", type=int, default=1, help="stack this many independent layers (1 = the named config)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-hbm-variant", action="store_true",  # (also skips the config-4-shape, repositioned and policy variants)
                    help="skip the extra 32-layer run whose 8 GiB cache cannot sit in the last-level cache")
    ap.add_argument("--legs", default="all",
                    help="which of the further configurations to run after the headline: comma list of "
                         "x32,c2,c5,c4,repos,policy, or all / none (for profiling one kernel at a time)")
    ap.add_argument("--prefill", action="store_true",
                    help="lay the first k tokens down directly instead of running k fill steps, so that every "
                         "step-kernel dispatch in the process is a full-occupancy one (for rocprofv3 --stats)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch a plain elementwise copy kernel of known size (1 GiB in, 1 GiB out) five "
                         "times, so that hardware byte counters collected over this run can be scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus must be 1 (the path shards by batch/layer "
              "without communication; nothing here uses a second GPU)", file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    from workloads import spec_for

    REPEATS = 5
    spec = spec_for("c3_mistral_gqa", L=args.layers, T=1024 + args.warmup + args.steps * (1 + REPEATS))
    g = gpu_leg(spec, args.seed, args.steps, args.warmup, "cuda:0", prefill=args.prefill, repeats=REPEATS)
    ms_per_step = g["event_ms"] / args.steps
    abytes = algorithmic_bytes_per_step(spec)
    achieved = abytes / (ms_per_step * 1e-3) / 1e9
    steps_per_launch = args.steps if g["plan"]["multi_step_blocks"] else 1
    per_step_traffic = (PROFILED_TRAFFIC_BYTES_PER_STEP if spec.L == 1 else
                        PROFILED_TRAFFIC_BYTES_PER_STEP_X32 if spec.L == 32 else None)
    reps = sorted(g["repeat_ms_per_step"])
    result = {
        "metric": "TOVA decode steps/sec and achieved HBM GB/s (% of peak), 1 MI355X",
        "value": 1e3 / ms_per_step,
        "unit": "decode steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 storage, f32 arithmetic", "data": "synthetic",
        "config": {"workload": "c3_mistral_gqa: Mistral-7B-shaped GQA layer, 32 q heads / 8 KV heads, d=128, bf16, "
                               f"batch 64, k=1024, L={spec.L}; 1024 untimed fill steps then timed decode steps "
                               "at full occupancy", "seed": args.seed, "plan": g["plan"],
                   "sequence_steps_per_s": 1e3 / ms_per_step * spec.L * spec.B},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     # bytes that left L2 per launch: the per-step figure of the committed rocprofv3 counter
                     # runs (not collected live) x the steps of this launch
                     "traffic": per_step_traffic * steps_per_launch if per_step_traffic else None,
                     "traffic_per_step_profiled": per_step_traffic,
                     "traffic_source": "profiles/tova_step_kernel_c3_mistral_gqa.txt (FETCH_SIZE + WRITE_SIZE per step, "
                                       "scaled by a 1 GiB copy); multiplied by steps_per_launch here",
                     "kernel": "tova_step_kernel<bf16, d=128, G=4, " +
                               ("workgroup per unit, " if g["plan"]["unit_workgroups"] else "") +
                               ("multi-step, service wave>" if steps_per_launch > 1 and g["plan"]["service_wave"]
                                else "multi-step>" if steps_per_launch > 1 else "per-step>"),
                     "steps_per_launch": steps_per_launch, "algorithmic_bytes_per_step": abytes,
                     "algorithmic_bytes_per_launch": abytes * steps_per_launch,
                     "avg_launch_us": ms_per_step * 1e3 * steps_per_launch,
                     "note": "this workload's 256 MiB of K/V is the size of the memory-side cache, and every step "
                             "re-reads the same rows: hits there are possible and the counters cannot tell them "
                             "from HBM.  frac_dram_bound is the same kernel on 32 such layers (8 GiB per step)."},
        "repeat_ms_per_step": {"n": len(reps), "median": reps[len(reps) // 2], "min": reps[0], "max": reps[-1],
                               "what": f"the timed call and {REPEATS} more calls of {args.steps} steps each on further tokens"},
        "sane": g["sane"], "new_token_dropped_frac": g["new_token_dropped_frac"],
        "wall_s_timed_region": g["wall_s"],
    }
    legs = not args.no_hbm_variant and args.layers == 1
    want = (set() if args.legs == "none" else {"x32", "c2", "c5", "c4", "repos", "policy"} if args.legs == "all"
            else set(args.legs.split(",")))
    if legs and "x32" in want:
        # same kernel, 32 independent layers: 8 GiB of cache per step cannot be served from the
        # 256 MB last-level cache, so this is the DRAM-bound figure
        s32 = spec_for("c3_mistral_gqa", L=32, T=1024 + 8 + 192)
        g32 = gpu_leg(s32, args.seed, 192, 8, "cuda:0", chunk=32)
        r32 = leg_record("config 3's layer shape x 32 layers (8 GiB cache; 2048 units, a workgroup per unit)", s32, g32, 192,
                         "tova_step_kernel<bf16, d=128, G=4, workgroup per unit, multi-step>")
        r32["roofline"]["traffic_per_step_profiled"] = PROFILED_TRAFFIC_BYTES_PER_STEP_X32
        result["hbm_resident_variant"] = r32
        result["roofline"]["frac_dram_bound"] = r32["roofline"]["frac"]
    else:
        result["roofline"]["frac_dram_bound"] = None
    if legs and "c2" in want:
        # config 2: one sequence, one layer, k = 512 -- 32 workgroups, latency-bound (ideal: 1 us per step)
        s2 = spec_for("c2_llama7b_layer", T=512 + 64 + 2048)
        g2 = gpu_leg(s2, 2, 2048, 64, "cuda:0")
        result["c2_llama7b_layer"] = leg_record("config 2: LLaMA-2-7B layer, 32 heads MHA, d=128, bf16, batch 1, k=512; 512 fill "
                                                "steps, then timed steps at full occupancy", s2, g2, 2048,
                                                "tova_step_kernel<bf16, d=128, G=1, multi-step>")
    if legs and "c5" in want:
        # config 5 at its full shape: 32 layers x 1 sequence, 8 query heads per KV head, k = 4096 (split cache,
        # hand-off form).  The first 4096 tokens are laid down directly (what the fill steps produce).
        s5 = spec_for("c5_yi_long", T=4096 + 32 + 512)
        g5 = gpu_leg(s5, 5, 512, 32, "cuda:0", chunk=128, prefill=True)
        result["c5_yi_long"] = leg_record("config 5: Yi-7B-shaped GQA 32/4, d=128, bf16, batch 1, 32 layers, k=4096 (split cache), "
                                          "timed steps at full occupancy of the 70,000-token stream's steady state", s5, g5, 512,
                                          "tova_step_kernel<bf16, d=128, G=8, split cache, multi-step>")
    if legs and "c4" in want:
        # config 4 at its full shape: 32 layers x 64 sequences of LLaMA-2-7B's layer shape, k = 4096 -- 128 GiB of
        # cache, 2048 units, a workgroup per unit.  The first 4096 tokens are laid down directly.
        free, _ = torch.cuda.mem_get_info()
        L4 = 32 if free > 150 * 2 ** 30 else max(1, int((free - 8 * 2 ** 30) // (4.2 * 2 ** 30)))
        s4 = spec_for("c4_llama7b_stack", L=L4, T=4096 + 4 + 32)
        g4 = gpu_leg(s4, 4, 32, 4, "cuda:0", chunk=16, prefill=True, also_prompt=True)
        r4 = leg_record(f"config 4: LLaMA-2-7B stack, 32 heads MHA, d=128, bf16, batch 64, k=4096, L={L4} "
                        f"({L4 * 4} GiB cache; {L4 * 64} units, a workgroup per unit), timed steps at full occupancy", s4, g4, 32,
                        "tova_step_kernel<bf16, d=128, G=1, workgroup per unit, multi-step>")
        r4["prompt_ms_per_token"] = g4["prompt_event_ms"] / 32
        r4["prompt_speedup_over_decode_steps"] = r4["ms_per_step"] / (g4["prompt_event_ms"] / 32)
        result["c4_llama7b_stack"] = r4
    if legs and "repos" in want:
        # decode steps beyond the training length (Sec. 7.2): LLaMA-2-7B layer shape with the multi-state of
        # 512 the paper uses there, keys cached without positions; 32 layers x 16 sequences = 512 units
        sr = spec_for("c2_llama7b_layer", L=32, B=16, T=512 + 8 + 32)
        gr = gpu_leg(sr, args.seed + 2, 32, 8, "cuda:0", chunk=16, prefill=True, repositioned=True)
        msr = gr["event_ms"] / 32
        abr = algorithmic_bytes_per_step(sr)
        result["repositioned_variant"] = {"workload": "tova_decode_steps_repositioned: config 2 layer shape (32 heads MHA, d=128, bf16, "
                                                      "k=512) x 32 layers x 16 sequences (4 GiB cache; 512 units, a workgroup per unit)",
                                          "steps": 32, "ms_per_step": msr, "achieved_GBps": abr / (msr * 1e-3) / 1e9,
                                          "frac": abr / (msr * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                          "sequence_steps_per_s": 1e3 / msr * 32 * 16, "sane": gr["sane"]}
    if legs and "policy" in want:
        # the policy on its own (App. B): fp32 attention weights [L][B][H][k+1] handed in, one launch per step;
        # config 3's layer shape x 32 layers, cache full
        from paper_2401_06104_amd import TovaCache
        sp = spec_for("c3_mistral_gqa", L=32)
        pc = TovaCache(sp.L, sp.B, sp.k, sp.H, sp.H_kv, sp.d, dtype=sp.dtype, device="cuda:0")
        pc.occupancy.fill_(sp.k)
        pc.slot_token.copy_(torch.arange(sp.k, dtype=torch.int32, device="cuda:0").expand_as(pc.slot_token))
        pc.set_tokens_seen(sp.k)
        gen = torch.Generator(device="cuda:0").manual_seed(args.seed + 3)
        W = torch.rand(sp.L, sp.B, sp.H, sp.k + 1, device="cuda:0", generator=gen)
        W /= W.sum(dim=-1, keepdim=True)
        kn = torch.randn(sp.L, sp.B, sp.H_kv, sp.d, device="cuda:0", generator=gen).to(torch.bfloat16)
        vn = torch.randn(sp.L, sp.B, sp.H_kv, sp.d, device="cuda:0", generator=gen).to(torch.bfloat16)
        evp = torch.empty(sp.L, sp.B, dtype=torch.int32, device="cuda:0")
        for _ in range(4):
            pc.policy_step(W, kn, vn, evp)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(32):
            pc.policy_step(W, kn, vn, evp)
        e1.record()
        torch.cuda.synchronize()
        msp = e0.elapsed_time(e1) / 32
        bp = W.numel() * 4 + 4 * kn.numel() * 2 + 8 * sp.L * sp.B       # weights in; new rows in, slot rows out; log + map
        result["policy_variant"] = {"workload": "tova_policy_step: config 3 layer shape x 32 layers (2048 units), fp32 attention "
                                                "weights [32][64][32][1025] given, one launch per step", "steps": 32,
                                    "ms_per_step": msp, "algorithmic_bytes_per_step": bp,
                                    "achieved_GBps": bp / (msp * 1e-3) / 1e9, "frac": bp / (msp * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                    "sane": bool(((evp >= 0) & (evp <= sp.k)).all())}
        pc.destroy()
        del W, pc
    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")       # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(5):
            torch.mul(src, 1.0, out=dst)                                      # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        result["calibration_copy"] = {"kernel": "torch elementwise mul(src, 1.0, out=dst)", "bytes_read": 1 << 30,
                                      "bytes_written": 1 << 30, "launches": 5}
        del src, dst
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_leg(spec_for("c3_mistral_gqa"), args.seed)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
