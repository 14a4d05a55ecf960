"""GPU test of tova_decode_steps_static, the entry point that allocates nothing: the hand-off
scratch of the step kernel (arrival counters, per-unit state words, partial score rows, chunk
statistics, PV partials) lives in the library's static device array instead of the cache's
scratch_mem.  Its results must be those of tova_decode_steps bit for bit -- outputs, victims, the
slot -> token map and the cached rows -- on two calls in a row that share the array, the second on
a smaller configuration with another layout (so it meets the first one's leftovers), and on a
cache that has no scratch buffer of its own at all."""
import pytest
import torch

from workloads import Stream, StreamSpec

pytestmark = pytest.mark.gpu

CASES = [
    # split cache (3 chunks per KV head): counters, chunk statistics, PV partials, score rows all in use;
    # 500 steps on a full cache run as one multi-step launch (state words)
    (StreamSpec("static_a", L=2, B=3, H=8, H_kv=2, d=128, dtype="bf16", k=300, T=800, sink="first", n_sinks=2), 3),
    # the second call: smaller, another layout (2 chunks, fp32, other strides) over the same array
    (StreamSpec("static_b", L=1, B=2, H=4, H_kv=4, d=64, dtype="f32", k=50, T=170, sink="first", n_sinks=1), 2),
]


def _run(spec, splits, how, cut):
    from paper_2401_06104_amd import TovaCache
    cache = TovaCache(spec.L, spec.B, spec.k, spec.H, spec.H_kv, spec.d, dtype=spec.dtype, n_splits=splits,
                      own_scratch=(how != "static_no_scratch"))
    assert cache.layout.unit_workgroups == 0 and cache.layout.n_splits == splits
    c = Stream(spec, 17, device="cuda:0").chunk(0, spec.T)
    out = torch.empty_like(c["q"])
    ev = torch.empty(spec.T, spec.L, spec.B, dtype=torch.int32, device="cuda:0")
    step = cache.decode_steps if how == "caller_scratch" else cache.decode_steps_static
    for a, b in ((0, cut), (cut, spec.T)):          # the fill phase and part of the rest, then the rest
        step(c["q"][a:b], c["k"][a:b], c["v"][a:b], out[a:b], ev[a:b])
    torch.cuda.synchronize()
    assert int(cache.error_flag.item()) == 0 and cache.tokens_seen == spec.T
    res = (out.cpu(), ev.cpu(), cache.slot_token.cpu().clone(), cache.occupancy.cpu().clone(),
           cache.K.cpu().clone(), cache.V.cpu().clone())
    cache.destroy()
    return res


def test_static_scratch_entry_point_matches_decode_steps():
    for spec, splits in CASES:                       # two calls in a row on the shared array, the second smaller
        cut = spec.k + 37
        ref = _run(spec, splits, "caller_scratch", cut)
        for how in ("static", "static_no_scratch"):
            got = _run(spec, splits, how, cut)
            for name, a, b in zip(("out", "evicted", "slot_token", "occupancy", "K", "V"), ref, got):
                assert torch.equal(a, b), f"{spec.name} ({how}): {name} differs from tova_decode_steps"
        assert (ref[1][spec.k:] >= 0).all() and (ref[1][:spec.k] == -1).all()


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    """A configuration whose hand-off scratch exceeds the static area is refused before anything is
    enqueued; a cache without scratch of its own refuses the calls that need one."""
    from paper_2401_06104_amd import TovaCache, TovaError, TOVA_ETOOBIG, TOVA_EINVAL, tova_cache_bytes
    # 8 query heads per KV head, 8 chunks: exp-value fallback area alone is pairs * (k+1) * 8 floats
    cache = TovaCache(4, 16, 4096, 32, 4, 128, dtype="bf16", n_splits=8, own_scratch=False)
    assert tova_cache_bytes(cache.cfg)[2] > 32 << 20
    q = torch.zeros(1, 4, 16, 32, 128, dtype=torch.bfloat16, device="cuda:0")
    kv = torch.zeros(1, 4, 16, 4, 128, dtype=torch.bfloat16, device="cuda:0")
    out = torch.empty_like(q)
    with pytest.raises(TovaError) as e:
        cache.decode_steps_static(q, kv, kv, out)
    assert e.value.status == TOVA_ETOOBIG and cache.tokens_seen == 0
    with pytest.raises(TovaError) as e:
        cache.decode_steps(q, kv, kv, out)
    assert e.value.status == TOVA_EINVAL and cache.tokens_seen == 0
    cache.destroy()
