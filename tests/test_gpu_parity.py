"""GPU parity tests: the HIP library, called through the C ABI, against the fp64 oracle on
the same seeded streams.  Bars and the near-tie rule are defined in tests/parity.py."""
import pytest
import torch

from workloads import StreamSpec, spec_for

import parity

pytestmark = pytest.mark.gpu


def _run(spec, seed, units, n_splits=0, workers=1, single_step_calls=False, chunk_steps=256):
    print(f"[parity] {spec.name} L={spec.L} B={spec.B} H={spec.H}/{spec.H_kv} d={spec.d} {spec.dtype} "
          f"k={spec.k} T={spec.T} seed={seed} splits={n_splits} units={units}", flush=True)
    res = parity.run_gpu(spec, seed, units, n_splits=n_splits, single_step_calls=single_step_calls,
                         chunk_steps=chunk_steps)
    parity.check_global_invariants(spec, res)
    stats = parity.check_units(spec, seed, units, res, workers=workers)
    for s in stats:
        print(f"[parity]   {s}  plan(S,R,block,grid)={res['layout']}", flush=True)
    return stats, res


# ---- config 1: the tiny fp32 case, complete, bit-exact victims -------------------------------
def test_c1_tiny_fp32_exact():
    spec = spec_for("c1_tiny")
    stats, _ = _run(spec, seed=1, units=[(0, 0)])
    assert stats[0]["mismatches"] == 0 and stats[0]["evict_steps"] == spec.T - spec.k


def test_c1_single_step_entry_point_matches():
    spec = spec_for("c1_tiny")
    stats, _ = _run(spec, seed=2, units=[(0, 0)], single_step_calls=True)
    assert stats[0]["mismatches"] == 0


# ---- shape sweep: every element type / head_dim / group size, ragged capacities, several
#      units, forced split counts (several tiles and a ragged tail in each) ----------------------
SWEEP = [
    # dtype, d, H, H_kv, k, T, L, B, splits
    ("f32", 32, 4, 4, 37, 150, 2, 3, 0),
    ("f32", 64, 8, 4, 100, 260, 1, 2, 3),
    ("f32", 128, 8, 1, 257, 420, 1, 2, 0),
    ("f32", 128, 4, 2, 1, 40, 1, 1, 0),          # capacity 1
    ("f32", 32, 2, 2, 2, 40, 1, 2, 2),           # one slot per chunk
    ("bf16", 128, 32, 8, 300, 520, 1, 3, 0),
    ("bf16", 128, 32, 8, 300, 520, 1, 3, 7),
    ("bf16", 128, 32, 4, 513, 700, 2, 1, 5),
    ("bf16", 128, 8, 8, 1025, 1300, 1, 2, 0),
    ("bf16", 64, 16, 8, 130, 300, 2, 2, 4),
    ("bf16", 32, 8, 2, 77, 200, 1, 5, 0),
    ("bf16", 128, 2, 1, 640, 900, 1, 9, 2),     # more units than one XCD round
]


@pytest.mark.parametrize("dtype,d,H,H_kv,k,T,L,B,splits", SWEEP)
def test_shape_sweep(dtype, d, H, H_kv, k, T, L, B, splits):
    spec = StreamSpec(f"sweep_{dtype}_d{d}_h{H}_{H_kv}_k{k}", L=L, B=B, H=H, H_kv=H_kv, d=d, dtype=dtype,
                      k=k, T=T, sink="first", n_sinks=2)
    units = [(l, b) for l in range(L) for b in range(B)][:4]
    stats, _ = _run(spec, seed=100 + k, units=units, n_splits=splits, workers=4)
    if dtype == "f32":
        assert all(s["mismatches"] == 0 for s in stats)


def test_cache_never_fills_is_full_attention():
    """k >= T: plain causal attention, no eviction (App. B early return)."""
    spec = StreamSpec("nofill", L=1, B=2, H=8, H_kv=2, d=64, dtype="f32", k=300, T=200)
    stats, res = _run(spec, seed=5, units=[(0, 0), (0, 1)])
    assert (res["evicted"] == -1).all() and stats[0]["evict_steps"] == 0


def test_identical_keys_evict_slot_zero():
    """Exact ties on the GPU too: with all keys equal every candidate has the same score and
    the lowest slot index must leave at every step."""
    from paper_2401_06104_amd import TovaCache
    dev = torch.device("cuda:0")
    L, B, H, H_kv, d, k, T = 1, 2, 8, 4, 128, 70, 120
    g = torch.Generator().manual_seed(0)
    key = torch.randn(1, L, B, H_kv, d, generator=g).expand(T, L, B, H_kv, d).contiguous()
    q = torch.randn(T, L, B, H, d, generator=g)
    v = torch.randn(T, L, B, H_kv, d, generator=g)
    for dtype, splits in ((torch.float32, 0), (torch.bfloat16, 3)):
        cache = TovaCache(L, B, k, H, H_kv, d, dtype=dtype, n_splits=splits, device=dev)
        qd, kd, vd = (x.to(dtype).to(dev) for x in (q, key, v))
        out = torch.empty_like(qd)
        ev = torch.empty(T, L, B, dtype=torch.int32, device=dev)
        cache.decode_steps(qd, kd, vd, out, ev)
        torch.cuda.synchronize()
        ev = ev.cpu()
        assert (ev[:k] == -1).all() and (ev[k:] == 0).all(), ev[k:].unique()
        # uniform weights: the output is the mean of the candidate V rows
        # candidates at the last step: slot 0 holds token T-2, slots 1..k-1 hold tokens 1..k-1, new = T-1
        cand = torch.cat([vd[[T - 2] + list(range(1, k)) + [T - 1]].float()]).mean(dim=0)   # [L,B,H_kv,d]
        ref = cand.repeat_interleave(H // H_kv, dim=2)
        torch.testing.assert_close(out[T - 1].float(), ref, rtol=2e-2, atol=2e-2)
        cache.destroy()


# ---- the paper-shaped configs ----------------------------------------------------------------
def test_c2_llama7b_layer_prefix():
    """Config 2 shape (split over 16 chunks per head), first 1100 tokens."""
    spec = spec_for("c2_llama7b_layer", T=1100)
    stats, res = _run(spec, seed=2, units=[(0, 0)])
    assert res["layout"][0] == 16


def test_c3_mistral_gqa_reduced_batch():
    """Config 3 shape per unit (G=4, k=1024), 8 sequences, 1024 fill + 300 decode steps."""
    spec = spec_for("c3_mistral_gqa", B=8, T=1024 + 300)
    _run(spec, seed=3, units=[(0, 0), (0, 5), (0, 7)], workers=3)


def test_c5_yi_long_reduced():
    """Config 5 shape per unit (G=8, split cache), 4 layers, k=1024, drifting mean."""
    spec = spec_for("c5_yi_long", L=4, k=1024, T=1500)
    _run(spec, seed=5, units=[(0, 0), (3, 0)], workers=2)


def test_c4_stack_reduced():
    """Config 4 shape per unit (MHA, one unsplit chunk, boosted keys), 2 layers x 3 sequences,
    capacity halved to keep the oracle's fill phase short."""
    spec = spec_for("c4_llama7b_stack", L=2, B=3, k=2048, T=2048 + 100)
    _run(spec, seed=4, units=[(1, 2)], chunk_steps=128)
