"""Counter-based, seeded generator of synthetic decode streams.

A stream is, for every decode step t, layer l and sequence b, the post-projection
query q_t [H, d] and the incoming token's key/value k_t, v_t [H_kv, d] -- the
inputs of one bounded-cache decode step (Sec. 3.2: the layer receives q_t, k_t,
v_t and its multi-state).  They stand in for the activations of the ~7B models
the paper runs (Sec. 4.3); no dataset or model weight is involved.

Design constraints (why this is not just torch.randn):

* Any (layer, sequence) unit can be regenerated alone, on any device, with the
  same bits: the CPU checker re-creates only the units it samples while the GPU
  run generates all of them in HBM.  Every value is therefore a pure function
  of (seed, tensor, step, layer, sequence, head, element).
* Bit-identical on CPU and GPU.  Only integer ops, a table gather and single,
  individually rounded fp32 multiplies/adds are used (never a fused
  multiply-add, a transcendental or a floating-point reduction), so the two
  devices cannot round differently.  Gaussians come from a 65536-entry
  quantile table built once on the host in fp64.

The integer mixing function is the public-domain "lowbias32" finaliser
(two xor-shift-multiply rounds); per-step keys come from splitmix64.
"""
from __future__ import annotations

import dataclasses
import math
from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

_M32 = 0xFFFFFFFF
_M64 = 0xFFFFFFFFFFFFFFFF

# tensor salts (distinct streams of the same seed)
_T_Q, _T_K, _T_V = 1, 2, 3
_T_WALK_Q, _T_WALK_K, _T_WALK_V = 11, 12, 13
_T_BOOST = 21
_T_SINK_U = 31
_T_SINK_POS = 32

_WALK_FIX = 1024  # fixed-point denominator of the integer random-walk increments


# --------------------------------------------------------------------------
# host-side scalar hashing (python ints)
# --------------------------------------------------------------------------
def _splitmix64(x: int) -> int:
    x = (x + 0x9E3779B97F4A7C15) & _M64
    z = x
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
    return z ^ (z >> 31)


def _key64(seed: int, tensor: int, t: int) -> int:
    return _splitmix64(_splitmix64(_splitmix64(seed & _M64) ^ tensor) ^ (t & _M64))


# --------------------------------------------------------------------------
# device-agnostic 32-bit mixing on int64 tensors holding values in [0, 2^32)
# --------------------------------------------------------------------------
def _mul32(x: torch.Tensor, c: int) -> torch.Tensor:
    # (x * c) mod 2^32 without ever exceeding 2^63 (signed overflow is avoided
    # so CPU and GPU agree by construction, not by wrap-around behaviour).
    lo = x & 0xFFFF
    hi = x >> 16
    return (lo * c + (((hi * c) & 0xFFFF) << 16)) & _M32


def _mix32(x: torch.Tensor) -> torch.Tensor:
    x = x ^ (x >> 16)
    x = _mul32(x, 0x7FEB352D)
    x = x ^ (x >> 15)
    x = _mul32(x, 0x846CA68B)
    x = x ^ (x >> 16)
    return x


def _mix32_int(x: int) -> int:
    x &= _M32
    x ^= x >> 16
    x = (x * 0x7FEB352D) & _M32
    x ^= x >> 15
    x = (x * 0x846CA68B) & _M32
    x ^= x >> 16
    return x


_TABLE_CACHE: Dict[str, torch.Tensor] = {}


def _gauss_table_host() -> np.ndarray:
    """Standard-normal quantiles at (i + 0.5) / 65536, fp64 -> fp32."""
    from scipy.special import ndtri

    p = (np.arange(65536, dtype=np.float64) + 0.5) / 65536.0
    return ndtri(p).astype(np.float32)


def _tables(device) -> tuple:
    key = str(device)
    if key not in _TABLE_CACHE:
        host = _gauss_table_host()
        ftab = torch.from_numpy(host.copy())
        itab = torch.from_numpy(np.rint(host.astype(np.float64) * _WALK_FIX).astype(np.int64))
        _TABLE_CACHE[key] = (ftab.to(device), itab.to(device))
    return _TABLE_CACHE[key]


# --------------------------------------------------------------------------
# specs
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class StreamSpec:
    """Shape and recipe of one synthetic stream (names follow the paper: k is
    the multi-state size, T the number of tokens streamed through it)."""

    name: str
    L: int
    B: int
    H: int
    H_kv: int
    d: int
    dtype: str            # "f32" | "bf16"
    k: int
    T: int
    elem_scale: float = 1.0   # every Gaussian entry is multiplied by this
    sink: str = "none"        # "none" | "first" | "per_seq"
    n_sinks: int = 0
    sink_bias: float = 3.0    # keys of sink tokens get + sink_bias * u
    q_align: float = 0.0      # optional: every query gets + q_align * u
    boost_prob: float = 0.0   # fraction of tokens whose keys are scaled up
    boost: float = 2.0        # expected key-norm increase of a boosted token
    drift_sigma: float = 0.0  # per-step std of the random-walk mean

    def replace(self, **kw) -> "StreamSpec":
        return dataclasses.replace(self, **kw)

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16


CONFIGS: Dict[str, StreamSpec] = {
    # batch 1, 1 layer, 4 heads MHA, d=32, fp32, k=16, 256 tokens, token 0 is a sink
    "c1_tiny": StreamSpec("c1_tiny", L=1, B=1, H=4, H_kv=4, d=32, dtype="f32", k=16, T=256,
                          sink="first", n_sinks=1),
    # LLaMA-2-7B-shaped single layer, k=512, 4096 tokens, entries N(0,1)/sqrt(128)
    "c2_llama7b_layer": StreamSpec("c2_llama7b_layer", L=1, B=1, H=32, H_kv=32, d=128, dtype="bf16",
                                   k=512, T=4096, elem_scale=1.0 / math.sqrt(128.0),
                                   sink="first", n_sinks=4),
    # Mistral-7B-shaped GQA layer, batch 64, k=1024: 1024 fill steps + 2048 decode steps
    "c3_mistral_gqa": StreamSpec("c3_mistral_gqa", L=1, B=64, H=32, H_kv=8, d=128, dtype="bf16",
                                 k=1024, T=1024 + 2048, sink="per_seq", n_sinks=4),
    # 32-layer LLaMA-2-7B-shaped stack, batch 64, k=4096: 4096 fill + 512 decode steps
    "c4_llama7b_stack": StreamSpec("c4_llama7b_stack", L=32, B=64, H=32, H_kv=32, d=128, dtype="bf16",
                                   k=4096, T=4096 + 512, boost_prob=0.05, boost=2.0),
    # Yi-7B-shaped GQA, 32 layers, batch 1, k=4096, 70,000-token stream with drifting mean
    "c5_yi_long": StreamSpec("c5_yi_long", L=32, B=1, H=32, H_kv=4, d=128, dtype="bf16",
                             k=4096, T=70000, drift_sigma=0.01),
}


def spec_for(name: str, **overrides) -> StreamSpec:
    """A named config, optionally scaled down (e.g. B=4, T=300) for a test."""
    return CONFIGS[name].replace(**overrides) if overrides else CONFIGS[name]


# --------------------------------------------------------------------------
# the stream
# --------------------------------------------------------------------------
class Stream:
    """Generates chunks of steps of one spec for a subset of (layer, sequence)
    units.  Values do not depend on the subset, the chunking or the device.

    chunk(t0, t1) returns q [T, Ls, Bs, H, d], k [T, Ls, Bs, H_kv, d] and v (same
    shape as k) in the spec's dtype, T = t1 - t0, Ls/Bs = selected layers/seqs.
    With drift_sigma > 0 chunks must be requested in increasing, contiguous
    order starting at 0 (the walk state is carried); reset() starts over.
    """

    def __init__(self, spec: StreamSpec, seed: int, device="cpu",
                 layers: Optional[Sequence[int]] = None, seqs: Optional[Sequence[int]] = None):
        self.spec = spec
        self.seed = int(seed)
        self.device = torch.device(device)
        self.layers = list(range(spec.L)) if layers is None else [int(x) for x in layers]
        self.seqs = list(range(spec.B)) if seqs is None else [int(x) for x in seqs]
        assert all(0 <= l < spec.L for l in self.layers) and all(0 <= b < spec.B for b in self.seqs)
        s = spec
        self._ftab, self._itab = _tables(self.device)
        # flat element index inside one step, from GLOBAL layer / sequence ids
        self._idx = {
            "q": self._flat_index(s.H),
            "kv": self._flat_index(s.H_kv),
        }
        assert s.L * s.B * s.H * s.d < 2 ** 32
        # sink direction u: unit vector in R^d shared by all heads (host fp64 -> fp32)
        self._u = None
        if s.sink != "none" or s.q_align != 0.0:
            z = np.array([_gauss_table_host()[_mix32_int(_key64(self.seed, _T_SINK_U, i)) >> 16]
                          for i in range(s.d)], dtype=np.float64)
            u = z / np.linalg.norm(z)
            self._u = u  # fp64, host
            self._k_bias = torch.from_numpy((s.sink_bias * u).astype(np.float32)).to(self.device)
            self._q_bias = torch.from_numpy((s.q_align * u).astype(np.float32)).to(self.device)
        self._sink_pos = self._make_sink_positions()
        self._walk_t = 0
        self._walk: Dict[str, torch.Tensor] = {}

    # ---- helpers ---------------------------------------------------------
    def _flat_index(self, heads: int) -> torch.Tensor:
        s = self.spec
        l = torch.tensor(self.layers, dtype=torch.int64).view(-1, 1, 1, 1)
        b = torch.tensor(self.seqs, dtype=torch.int64).view(1, -1, 1, 1)
        h = torch.arange(heads, dtype=torch.int64).view(1, 1, -1, 1)
        i = torch.arange(s.d, dtype=torch.int64).view(1, 1, 1, -1)
        return (((l * s.B + b) * heads + h) * s.d + i).to(self.device)

    def _make_sink_positions(self) -> Optional[List[List[int]]]:
        """For every selected sequence the token positions that are sinks."""
        s = self.spec
        if s.sink == "none":
            return None
        if s.sink == "first":
            return [list(range(s.n_sinks)) for _ in self.seqs]
        assert s.sink == "per_seq"
        out = []
        hi = min(s.k, s.T)
        assert s.n_sinks <= hi
        for b in self.seqs:
            chosen: List[int] = []
            ctr = 0
            while len(chosen) < s.n_sinks:  # distinct uniform draws by rejection
                p = _key64(self.seed, _T_SINK_POS, b * 4096 + ctr) % hi
                ctr += 1
                if p not in chosen:
                    chosen.append(p)
            out.append(sorted(chosen))
        return out

    def sink_positions(self) -> Optional[List[List[int]]]:
        return self._sink_pos

    def _keys(self, tensor: int, t0: int, t1: int):
        ks = [_key64(self.seed, tensor, t) for t in range(t0, t1)]
        a = torch.tensor([x & _M32 for x in ks], dtype=torch.int64, device=self.device)
        b = torch.tensor([x >> 32 for x in ks], dtype=torch.int64, device=self.device)
        return a.view(-1, 1, 1, 1, 1), b.view(-1, 1, 1, 1, 1)

    def _u16(self, tensor: int, idx: torch.Tensor, t0: int, t1: int) -> torch.Tensor:
        a, b = self._keys(tensor, t0, t1)
        x = _mix32((idx.unsqueeze(0) + a) & _M32)
        x = _mix32(x ^ b)
        return x >> 16

    def _gauss(self, tensor: int, idx: torch.Tensor, t0: int, t1: int) -> torch.Tensor:
        return self._ftab[self._u16(tensor, idx, t0, t1)]

    def reset(self):
        self._walk_t = 0
        self._walk = {}

    # ---- main entry --------------------------------------------------------
    def chunk(self, t0: int, t1: int, need_q: bool = True) -> Dict[str, torch.Tensor]:
        """Steps t0..t1-1.  With need_q=False the queries are not generated (the returned
        "q" is None): used to lay down cached rows without stepping through them."""
        s = self.spec
        assert 0 <= t0 < t1 <= s.T, (t0, t1, s.T)
        T = t1 - t0
        q = self._gauss(_T_Q, self._idx["q"], t0, t1) if need_q else None
        k = self._gauss(_T_K, self._idx["kv"], t0, t1)
        v = self._gauss(_T_V, self._idx["kv"], t0, t1)
        if s.elem_scale != 1.0:
            c = float(np.float32(s.elem_scale))
            q, k, v = (q * c if need_q else None), k * c, v * c

        if s.drift_sigma > 0.0:
            if t0 != self._walk_t:
                raise ValueError("drifting stream: chunks must be contiguous from 0 "
                                 f"(expected t0={self._walk_t}, got {t0}); call reset()")
            c = float(np.float32(s.drift_sigma / _WALK_FIX))
            for name, tid, idx in (("q", _T_WALK_Q, self._idx["q"]),
                                   ("k", _T_WALK_K, self._idx["kv"]),
                                   ("v", _T_WALK_V, self._idx["kv"])):
                inc = self._itab[self._u16(tid, idx, t0, t1)]
                if t0 == 0:
                    inc[0].zero_()          # mu_0 = 0
                w = torch.cumsum(inc, dim=0)    # exact integer walk
                if name in self._walk:
                    w = w + self._walk[name]
                self._walk[name] = w[-1].clone()
                mu = w.to(torch.float32) * c    # |w| < 2^24: exact conversion, one rounding
                if name == "q":
                    q = q + mu if need_q else None
                elif name == "k":
                    k = k + mu
                else:
                    v = v + mu
            self._walk_t = t1

        if s.boost_prob > 0.0:
            # one Bernoulli per (step, layer, sequence); factor raises the
            # expected key norm sqrt(d) by `boost`
            lb = (self._idx["kv"][:, :, :1, :1] // (s.H_kv * s.d))
            thr = int(round(s.boost_prob * 65536))
            hit = self._u16(_T_BOOST, lb, t0, t1) < thr
            f = float(np.float32(1.0 + s.boost / math.sqrt(s.d)))
            k = torch.where(hit, k * f, k)

        if self._sink_pos is not None:
            m = torch.zeros(T, len(self.seqs), dtype=torch.bool)
            for bi, plist in enumerate(self._sink_pos):
                for p in plist:
                    if t0 <= p < t1:
                        m[p - t0, bi] = True
            if bool(m.any()):
                m = m.to(self.device).view(T, 1, len(self.seqs), 1, 1)
                k = torch.where(m, k + self._k_bias, k)
        if s.q_align != 0.0 and need_q:
            q = q + self._q_bias

        dt = s.torch_dtype
        return {"q": q.to(dt).contiguous() if need_q else None,
                "k": k.to(dt).contiguous(), "v": v.to(dt).contiguous()}

    def boosted(self, t0: int, t1: int) -> torch.Tensor:
        """[T, Ls, Bs] bool: which tokens got the key-norm boost (for inspection)."""
        s = self.spec
        lb = (self._idx["kv"][:, :, :1, :1] // (s.H_kv * s.d))
        thr = int(round(s.boost_prob * 65536))
        return (self._u16(_T_BOOST, lb, t0, t1) < thr)[..., 0, 0]
