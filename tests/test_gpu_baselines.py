"""GPU parity of the baseline policies (Sec. 4.1: Window, Window+i, H2O) through the same fused step
kernel, against their fp64 oracles (oracle/tova_baselines.py) on the same seeded streams.  Bars as
for TOVA (tests/parity.py): outputs per vector within 2e-2 (bf16) / 1e-5 (fp32) of the oracle;
Window / Window+i victims bit-exact (they depend on integers only); H2O victims equal except where
the oracle's two lowest aggregated scores outside the window are closer than 1e-6 and the GPU's
choice is within that distance of the lowest -- counted, and the oracle then follows the GPU; final
slot -> token map and cached rows bit-exact; H2O's aggregated scores within 1e-4 relative."""
import numpy as np
import pytest
import torch

from workloads import Stream, StreamSpec, spec_for

import parity

pytestmark = pytest.mark.gpu


def _check_unit(spec, seed, unit, ui, res, policy, pinned, heavy):
    from oracle.tova_baselines import H2OOracle, WindowOracle
    l, b = unit
    st = Stream(spec, seed, device="cpu", layers=[l], seqs=[b])
    c = st.chunk(0, spec.T)
    q, kk, vv = (c[n][:, 0, 0].double().numpy() for n in "qkv")
    orc = (WindowOracle(spec.k, spec.H, spec.H_kv, spec.d, pinned=pinned) if policy == "window"
           else H2OOracle(spec.k, spec.H, spec.H_kv, spec.d, heavy=heavy if heavy else None))
    tol = parity.OUT_TOL[spec.dtype]
    ev = res["evicted"][:, l, b]
    out = res["out"][:, ui].astype(np.float64)
    near = worst = 0
    for t in range(spec.T):
        ge = int(ev[t])
        full = orc.n == spec.k
        el = orc.eligible() if (policy == "h2o" and full) else None
        r = orc.step(q[t], kk[t], vv[t], force_victim=ge if full else None)
        err = (np.abs(out[t] - r.out).max(axis=1) / np.maximum(np.abs(r.out).max(axis=1), 1e-30)).max()
        assert err <= tol, f"{policy} unit {unit} step {t}: output rel err {err:.3e}"
        worst = max(worst, err)
        if not full:
            assert ge == -1
            continue
        assert 0 <= ge < spec.k, f"{policy} unit {unit} step {t}: victim {ge} (the incoming token always stays)"
        if ge != r.evicted:
            assert policy == "h2o", f"window unit {unit} step {t}: GPU victim {ge} != {r.evicted}"
            assert el[ge] and r.gap < parity.GAP_EXEMPT and r.s[ge] - r.s[r.evicted] < parity.GAP_EXEMPT, \
                f"h2o unit {unit} step {t}: GPU victim {ge} != oracle {r.evicted}, gap {r.gap:.3e}"
            near += 1
    assert np.array_equal(orc.slot_token, res["slot_token"][l, b].astype(np.int64))
    assert np.array_equal(orc.K, res["K"][ui].astype(np.float64)) and np.array_equal(orc.V, res["V"][ui].astype(np.float64))
    if policy == "h2o":
        np.testing.assert_allclose(res["h2o_acc"][l, b] / spec.H, orc.acc, rtol=1e-4, atol=1e-7)
    return dict(unit=unit, steps=spec.T, evict_steps=spec.T - spec.k, near_tie_choices=near, max_rel_err=float(worst))


CASES = [
    # policy, dtype, d, H, H_kv, k, T, L, B, pinned (Window+i), heavy (H2O; 0 = half)
    ("window", "f32", 32, 4, 4, 16, 120, 1, 2, 0, 0),          # plain Window
    ("window", "bf16", 128, 32, 8, 300, 700, 1, 3, 4, 0),      # Window+4 at config 3's head layout
    ("window", "bf16", 64, 8, 8, 1, 40, 2, 2, 0, 0),           # capacity 1: only the last token
    ("window", "f32", 64, 8, 2, 37, 200, 2, 2, 1, 0),          # Window+1
    ("h2o", "f32", 32, 4, 4, 16, 160, 1, 2, 0, 0),
    ("h2o", "bf16", 128, 32, 8, 300, 800, 1, 3, 0, 0),
    ("h2o", "bf16", 128, 32, 4, 513, 900, 2, 1, 0, 100),       # 8 heads per KV head, uneven window
    ("h2o", "f32", 64, 8, 2, 37, 260, 2, 2, 0, 36),            # a window of one token
    ("h2o", "bf16", 64, 8, 8, 48, 200, 8, 40, 0, 0),           # 320 units: workgroups walk several units per step
]


@pytest.mark.parametrize("policy,dtype,d,H,H_kv,k,T,L,B,pinned,heavy", CASES)
def test_baseline_policy_shape_sweep(policy, dtype, d, H, H_kv, k, T, L, B, pinned, heavy):
    spec = StreamSpec(f"{policy}_{dtype}_d{d}_h{H}_{H_kv}_k{k}", L=L, B=B, H=H, H_kv=H_kv, d=d, dtype=dtype, k=k, T=T,
                      sink="first", n_sinks=2)
    units = sorted({(0, 0), (L - 1, B - 1), (L // 2, B // 3)})
    print(f"[parity] {spec.name} L={L} B={B} T={T} pinned={pinned} heavy={heavy} units={units}", flush=True)
    res = parity.run_gpu(spec, 1200 + k, units, n_pinned=pinned, policy=policy, h2o_heavy=heavy, chunk_steps=97)
    assert res["unit_workgroups"] == 1
    parity.check_global_invariants(spec, res)
    assert (res["evicted"][k:] < k).all()
    for ui, u in enumerate(units):
        s = _check_unit(spec, 1200 + k, u, ui, res, policy, pinned, heavy)
        print(f"[parity]   {s}", flush=True)
        if dtype == "f32":
            assert s["near_tie_choices"] == 0


def test_window_victims_follow_the_closed_form_at_config3_shape():
    """Window+4 on config 3's full shape (64 sequences, k = 1024): after the fill the victims walk the
    slots behind the first four as a ring, for every sequence (Sec. 4.1: first in, first out)."""
    spec = spec_for("c3_mistral_gqa", T=1024 + 300)
    res = parity.run_gpu(spec, 3, [(0, 0)], n_pinned=4, policy="window")
    ev = res["evicted"][spec.k:]
    want = 4 + (np.arange(300) % (spec.k - 4))
    assert (ev == want[:, None, None]).all()


def test_h2o_head_wise_variant():
    """The head-wise H2O the paper reports (Sec. 4.1): every KV head keeps its own rows; it is the
    layer-wise computation with each KV head as a sequence of its own, which is how it is checked."""
    H, H_kv, k = 8, 4, 40
    spec = StreamSpec("h2o_perhead", L=2, B=3, H=H, H_kv=H_kv, d=64, dtype="bf16", k=k, T=k + 200)
    view = spec.replace(B=spec.B * H_kv, H=H // H_kv, H_kv=1)
    units = [(0, 0), (0, H_kv - 1), (1, view.B - 1)]
    res = parity.run_gpu(spec, 47, units, per_head=True, policy="h2o")
    parity.check_global_invariants(view, res)
    ev = res["evicted"][k:].reshape(-1, spec.L, spec.B, H_kv)
    assert (ev != ev[..., :1]).any(), "all heads always agreed: the variant was not exercised"
    for ui, u in enumerate(units):
        print(f"[parity]   {_check_unit(view, 47, u, ui, res, 'h2o', 0, 0)}", flush=True)


def test_baseline_policies_refuse_the_other_entry_points():
    from paper_2401_06104_amd import TovaCache, TovaError, TOVA_ENOSUP, TOVA_EINVAL
    cache = TovaCache(1, 2, 16, 4, 2, 32, dtype="bf16", policy="h2o")
    q = torch.zeros(2, 1, 2, 4, 32, dtype=torch.bfloat16, device="cuda:0")
    kv = torch.zeros(2, 1, 2, 2, 32, dtype=torch.bfloat16, device="cuda:0")
    out = torch.empty_like(q)
    with pytest.raises(TovaError) as e:
        cache.decode_steps_repositioned(q, kv, kv, out)
    assert e.value.status == TOVA_ENOSUP
    w = torch.zeros(1, 2, 4, 17, device="cuda:0")
    with pytest.raises(TovaError) as e:
        cache.policy_step(w, kv[0], kv[0])
    assert e.value.status == TOVA_ENOSUP
    cache.prefill(q, kv, kv, out)                       # a prompt goes token by token
    torch.cuda.synchronize()
    assert cache.tokens_seen == 2
    cache.destroy()
    with pytest.raises(TovaError) as e:
        TovaCache(1, 2, 16, 4, 2, 32, dtype="bf16", policy="h2o", n_pinned=2)
    assert e.value.status == TOVA_EINVAL
