"""ctypes binding of include/tova.h: argument marshalling only.

Function names follow the C ABI (tova_cache_bytes, tova_cache_layout, and the
TovaCache methods init / decode_step / decode_steps / destroy map one-to-one to
tova_cache_init / tova_decode_step / tova_decode_steps / tova_cache_destroy).
There is no fallback: if libtova.so is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, byref, c_char_p, c_float, c_int, c_int32, c_int64, c_size_t, c_void_p
from typing import Optional

TOVA_OK, TOVA_EINVAL, TOVA_ENOSUP, TOVA_EHIP, TOVA_ENOMEM, TOVA_ETOOBIG = 0, -1, -2, -3, -4, -5
TOVA_F32, TOVA_BF16 = 0, 1
TOVA_POLICY_TOVA, TOVA_POLICY_WINDOW, TOVA_POLICY_H2O = 0, 1, 2

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
_LIB: Optional[ctypes.CDLL] = None


class TovaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {tova_strerror(status)} (status {status})")


class TovaConfig(ctypes.Structure):
    _fields_ = [("n_layers", c_int32), ("batch", c_int32), ("capacity_k", c_int32),
                ("n_q_heads", c_int32), ("n_kv_heads", c_int32), ("head_dim", c_int32),
                ("dtype", c_int32), ("softmax_scale", c_float), ("n_splits", c_int32),
                ("n_pinned", c_int32), ("per_head", c_int32), ("policy", c_int32), ("h2o_heavy", c_int32)]


class TovaLayout(ctypes.Structure):
    _fields_ = [("k_offset", c_size_t), ("v_offset", c_size_t), ("occupancy_offset", c_size_t),
                ("slot_token_offset", c_size_t), ("error_flag_offset", c_size_t), ("n_splits", c_int32), ("rows_per_split", c_int32),
                ("block_threads", c_int32), ("grid_blocks", c_int32), ("lds_bytes", c_int32),
                ("unit_workgroups", c_int32), ("prefill_group", c_int32), ("tokens_seen_offset", c_size_t), ("h2o_acc_offset", c_size_t),
                ("service_wave", c_int32)]


def library_path() -> str:
    return os.path.join(_PKG_DIR, "libtova.so")


def load_library() -> ctypes.CDLL:
    """Loads the in-tree libtova.so.  Raises if it has not been built."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    if not os.path.exists(path):
        raise RuntimeError(f"{path} not found: build it with `python -m paper_2401_06104_amd.build` "
                           "(there is no CPU fallback)")
    # torch first: libtova.so needs the HIP runtime, and a process must have only one -- the one
    # torch brings.  (Loaded before torch, the library pulls in the system's copy, and its first
    # launch then reports that there is no device.)
    import torch  # noqa: F401
    lib = ctypes.CDLL(path)
    cfgp = POINTER(TovaConfig)
    lib.tova_cache_bytes.argtypes = [cfgp, POINTER(c_size_t), POINTER(c_size_t), POINTER(c_size_t)]
    lib.tova_cache_layout.argtypes = [cfgp, POINTER(TovaLayout)]
    lib.tova_cache_init.argtypes = [POINTER(c_void_p), cfgp, c_void_p, c_void_p, c_void_p, c_void_p]
    lib.tova_decode_step.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
    lib.tova_decode_steps.argtypes = [c_void_p, c_int32, c_void_p, c_void_p, c_void_p, c_void_p,
                                      c_void_p, c_void_p]
    lib.tova_decode_steps_static.argtypes = [c_void_p, c_int32, c_void_p, c_void_p, c_void_p, c_void_p,
                                             c_void_p, c_void_p]
    lib.tova_prefill.argtypes = [c_void_p, c_int32, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
    lib.tova_decode_steps_repositioned.argtypes = [c_void_p, c_int32, c_void_p, c_void_p, c_void_p, c_void_p,
                                                   c_void_p, c_float, c_void_p]
    lib.tova_policy_step.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
    lib.tova_cache_tokens_seen.argtypes = [c_void_p, POINTER(c_int64)]
    lib.tova_cache_multi_step_blocks.argtypes = [c_void_p, POINTER(c_int32)]
    lib.tova_cache_set_tokens_seen.argtypes = [c_void_p, c_int64]
    lib.tova_decode_step_graph.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
    lib.tova_cache_publish_tokens_seen.argtypes = [c_void_p, c_void_p]
    lib.tova_cache_fetch_tokens_seen.argtypes = [c_void_p, c_void_p, POINTER(c_int64)]
    lib.tova_cache_status.argtypes = [c_void_p, c_void_p, POINTER(c_int32)]
    lib.tova_cache_recover.argtypes = [c_void_p, c_int64, c_void_p]
    lib.tova_cache_destroy.argtypes = [c_void_p]
    lib.tova_strerror.argtypes = [c_int]
    lib.tova_strerror.restype = c_char_p
    for name in ("tova_cache_bytes", "tova_cache_layout", "tova_cache_init", "tova_decode_step",
                 "tova_decode_steps", "tova_decode_steps_static", "tova_prefill", "tova_cache_tokens_seen", "tova_cache_set_tokens_seen",
                 "tova_cache_multi_step_blocks", "tova_cache_status", "tova_cache_recover", "tova_decode_step_graph",
                 "tova_cache_publish_tokens_seen", "tova_cache_fetch_tokens_seen",
                 "tova_decode_steps_repositioned", "tova_policy_step", "tova_cache_destroy"):
        getattr(lib, name).restype = c_int
    _LIB = lib
    return lib


def tova_strerror(status: int) -> str:
    return load_library().tova_strerror(int(status)).decode()


def tova_cache_bytes(cfg: TovaConfig):
    """(kv_bytes, state_bytes, scratch_bytes) of the caller-owned device buffers."""
    kv, st, sc = c_size_t(), c_size_t(), c_size_t()
    rc = load_library().tova_cache_bytes(byref(cfg), byref(kv), byref(st), byref(sc))
    if rc != TOVA_OK:
        raise TovaError(rc, "tova_cache_bytes")
    return kv.value, st.value, sc.value


def tova_cache_layout(cfg: TovaConfig) -> TovaLayout:
    lay = TovaLayout()
    rc = load_library().tova_cache_layout(byref(cfg), byref(lay))
    if rc != TOVA_OK:
        raise TovaError(rc, "tova_cache_layout")
    return lay


def _stream_handle(stream) -> int:
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return int(s.cuda_stream)


class TovaCache:
    """Owns the three device buffers (torch tensors) and the library's descriptor."""

    def __init__(self, n_layers: int, batch: int, capacity_k: int, n_q_heads: int, n_kv_heads: int,
                 head_dim: int, dtype="bf16", softmax_scale: float = 0.0, n_splits: int = 0,
                 device="cuda:0", stream=None, n_pinned: int = 0, per_head: bool = False,
                 own_scratch: bool = True, policy="tova", h2o_heavy: int = 0):
        import torch
        self._torch = torch
        self.lib = load_library()
        code = {"f32": TOVA_F32, "fp32": TOVA_F32, "float32": TOVA_F32, torch.float32: TOVA_F32,
                "bf16": TOVA_BF16, "bfloat16": TOVA_BF16, torch.bfloat16: TOVA_BF16}[dtype]
        pol = {"tova": TOVA_POLICY_TOVA, "window": TOVA_POLICY_WINDOW, "h2o": TOVA_POLICY_H2O}.get(policy, policy)
        self.cfg = TovaConfig(n_layers, batch, capacity_k, n_q_heads, n_kv_heads, head_dim, code,
                              float(softmax_scale), int(n_splits), int(n_pinned), int(bool(per_head)),
                              int(pol), int(h2o_heavy))
        # shape of evicted / occupancy (slot_token: + [k]); TOVA-head keeps them per KV head
        self.state_shape = (n_layers, batch, n_kv_heads) if per_head else (n_layers, batch)
        self.torch_dtype = torch.float32 if code == TOVA_F32 else torch.bfloat16
        self.device = torch.device(device)
        self.layout = tova_cache_layout(self.cfg)
        kvb, stb, scb = tova_cache_bytes(self.cfg)
        self.kv_mem = torch.empty(kvb, dtype=torch.uint8, device=self.device)
        self.state_mem = torch.empty(stb, dtype=torch.uint8, device=self.device)
        # own_scratch=False: no scratch buffer (a cache that is only stepped through decode_steps_static)
        self.scratch_mem = torch.empty(scb, dtype=torch.uint8, device=self.device) if own_scratch else None
        self._h = c_void_p()
        with torch.cuda.device(self.device):
            rc = self.lib.tova_cache_init(byref(self._h), byref(self.cfg), self.kv_mem.data_ptr(),
                                          self.state_mem.data_ptr(),
                                          self.scratch_mem.data_ptr() if own_scratch else None,
                                          _stream_handle(stream))
        if rc != TOVA_OK:
            raise TovaError(rc, "tova_cache_init")

    # ---- views into the caller-owned buffers (no copies) -----------------
    def _shape_kv(self):
        c = self.cfg
        return (c.n_layers, c.batch, c.n_kv_heads, c.capacity_k, c.head_dim)

    @property
    def K(self):
        n = self.kv_mem.numel() // 2
        return self.kv_mem[self.layout.k_offset:self.layout.k_offset + n].view(self.torch_dtype).view(self._shape_kv())

    @property
    def V(self):
        n = self.kv_mem.numel() // 2
        return self.kv_mem[self.layout.v_offset:self.layout.v_offset + n].view(self.torch_dtype).view(self._shape_kv())

    @property
    def occupancy(self):
        o = self.layout.occupancy_offset
        n = 1
        for x in self.state_shape:
            n *= x
        return self.state_mem[o:o + 4 * n].view(self._torch.int32).view(self.state_shape)

    @property
    def slot_token(self):
        c = self.cfg
        o = self.layout.slot_token_offset
        n = c.capacity_k
        for x in self.state_shape:
            n *= x
        return self.state_mem[o:o + 4 * n].view(self._torch.int32).view(*self.state_shape, c.capacity_k)

    @property
    def h2o_acc(self):
        """H2O: per slot, the attention weights summed over query heads and over the steps since its token came in."""
        c = self.cfg
        o = self.layout.h2o_acc_offset
        n = c.capacity_k
        for x in self.state_shape:
            n *= x
        return self.state_mem[o:o + 4 * n].view(self._torch.float32).view(*self.state_shape, c.capacity_k)

    @property
    def error_flag(self):
        o = self.layout.error_flag_offset
        return self.state_mem[o:o + 4].view(self._torch.int32)

    @property
    def multi_step_blocks(self) -> int:
        b = c_int32()
        rc = self.lib.tova_cache_multi_step_blocks(self._h, byref(b))
        if rc != TOVA_OK:
            raise TovaError(rc, "tova_cache_multi_step_blocks")
        return b.value

    @property
    def tokens_seen(self) -> int:
        t = c_int64()
        rc = self.lib.tova_cache_tokens_seen(self._h, byref(t))
        if rc != TOVA_OK:
            raise TovaError(rc, "tova_cache_tokens_seen")
        return t.value

    def status(self, stream=None) -> int:
        """Waits for the stream; 1 if a multi-step launch gave up waiting since the flag was last cleared."""
        f = c_int32()
        rc = self.lib.tova_cache_status(self._h, _stream_handle(stream), byref(f))
        if rc != TOVA_OK:
            raise TovaError(rc, "tova_cache_status")
        return f.value

    def recover(self, tokens_seen: int, stream=None):
        """After status() == 1 and after the caller restored kv_mem / state_mem from its snapshot."""
        rc = self.lib.tova_cache_recover(self._h, int(tokens_seen), _stream_handle(stream))
        if rc != TOVA_OK:
            raise TovaError(rc, "tova_cache_recover")

    def set_tokens_seen(self, t: int):
        rc = self.lib.tova_cache_set_tokens_seen(self._h, int(t))
        if rc != TOVA_OK:
            raise TovaError(rc, "tova_cache_set_tokens_seen")

    # ---- the calls ----------------------------------------------------------
    def _check(self, name, x, shape):
        if x.dtype != self.torch_dtype or x.device != self.kv_mem.device or not x.is_contiguous() \
                or tuple(x.shape) != tuple(shape):
            raise ValueError(f"{name}: expected contiguous {self.torch_dtype} {tuple(shape)} on "
                             f"{self.kv_mem.device}, got {x.dtype} {tuple(x.shape)} on {x.device}")

    def decode_step(self, q, k_new, v_new, out, evicted=None, stream=None):
        c = self.cfg
        self._check("q", q, (c.n_layers, c.batch, c.n_q_heads, c.head_dim))
        self._check("k_new", k_new, (c.n_layers, c.batch, c.n_kv_heads, c.head_dim))
        self._check("v_new", v_new, (c.n_layers, c.batch, c.n_kv_heads, c.head_dim))
        self._check("out", out, (c.n_layers, c.batch, c.n_q_heads, c.head_dim))
        ev = self._evicted_ptr(evicted, self.state_shape)
        rc = self.lib.tova_decode_step(self._h, q.data_ptr(), k_new.data_ptr(), v_new.data_ptr(),
                                       out.data_ptr(), ev, _stream_handle(stream))
        if rc != TOVA_OK:
            raise TovaError(rc, "tova_decode_step")

    def decode_step_graph(self, q, k_new, v_new, out, evicted=None, stream=None):
        """decode_step whose token index lives in state_mem: can be recorded into a graph and replayed."""
        c = self.cfg
        self._check("q", q, (c.n_layers, c.batch, c.n_q_heads, c.head_dim))
        self._check("k_new", k_new, (c.n_layers, c.batch, c.n_kv_heads, c.head_dim))
        self._check("v_new", v_new, (c.n_layers, c.batch, c.n_kv_heads, c.head_dim))
        self._check("out", out, (c.n_layers, c.batch, c.n_q_heads, c.head_dim))
        ev = self._evicted_ptr(evicted, self.state_shape)
        rc = self.lib.tova_decode_step_graph(self._h, q.data_ptr(), k_new.data_ptr(), v_new.data_ptr(),
                                             out.data_ptr(), ev, _stream_handle(stream))
        if rc != TOVA_OK:
            raise TovaError(rc, "tova_decode_step_graph")

    def publish_tokens_seen(self, stream=None):
        rc = self.lib.tova_cache_publish_tokens_seen(self._h, _stream_handle(stream))
        if rc != TOVA_OK:
            raise TovaError(rc, "tova_cache_publish_tokens_seen")

    def fetch_tokens_seen(self, stream=None) -> int:
        t = c_int64()
        rc = self.lib.tova_cache_fetch_tokens_seen(self._h, _stream_handle(stream), byref(t))
        if rc != TOVA_OK:
            raise TovaError(rc, "tova_cache_fetch_tokens_seen")
        return t.value

    def decode_steps(self, q, k_new, v_new, out, evicted=None, stream=None):
        c = self.cfg
        T = q.shape[0]
        self._check("q", q, (T, c.n_layers, c.batch, c.n_q_heads, c.head_dim))
        self._check("k_new", k_new, (T, c.n_layers, c.batch, c.n_kv_heads, c.head_dim))
        self._check("v_new", v_new, (T, c.n_layers, c.batch, c.n_kv_heads, c.head_dim))
        self._check("out", out, (T, c.n_layers, c.batch, c.n_q_heads, c.head_dim))
        ev = self._evicted_ptr(evicted, (T, *self.state_shape))
        rc = self.lib.tova_decode_steps(self._h, T, q.data_ptr(), k_new.data_ptr(), v_new.data_ptr(),
                                        out.data_ptr(), ev, _stream_handle(stream))
        if rc != TOVA_OK:
            raise TovaError(rc, "tova_decode_steps")

    def decode_steps_static(self, q, k_new, v_new, out, evicted=None, stream=None):
        """decode_steps with the hand-off scratch in the library's static device array (allocates nothing)."""
        c = self.cfg
        T = q.shape[0]
        self._check("q", q, (T, c.n_layers, c.batch, c.n_q_heads, c.head_dim))
        self._check("k_new", k_new, (T, c.n_layers, c.batch, c.n_kv_heads, c.head_dim))
        self._check("v_new", v_new, (T, c.n_layers, c.batch, c.n_kv_heads, c.head_dim))
        self._check("out", out, (T, c.n_layers, c.batch, c.n_q_heads, c.head_dim))
        ev = self._evicted_ptr(evicted, (T, *self.state_shape))
        rc = self.lib.tova_decode_steps_static(self._h, T, q.data_ptr(), k_new.data_ptr(), v_new.data_ptr(),
                                               out.data_ptr(), ev, _stream_handle(stream))
        if rc != TOVA_OK:
            raise TovaError(rc, "tova_decode_steps_static")

    def prefill(self, q, k_new, v_new, out, evicted=None, stream=None):
        """A prompt of T tokens known in advance: same arguments and results as decode_steps."""
        c = self.cfg
        T = q.shape[0]
        self._check("q", q, (T, c.n_layers, c.batch, c.n_q_heads, c.head_dim))
        self._check("k_new", k_new, (T, c.n_layers, c.batch, c.n_kv_heads, c.head_dim))
        self._check("v_new", v_new, (T, c.n_layers, c.batch, c.n_kv_heads, c.head_dim))
        self._check("out", out, (T, c.n_layers, c.batch, c.n_q_heads, c.head_dim))
        ev = self._evicted_ptr(evicted, (T, *self.state_shape))
        rc = self.lib.tova_prefill(self._h, T, q.data_ptr(), k_new.data_ptr(), v_new.data_ptr(),
                                   out.data_ptr(), ev, _stream_handle(stream))
        if rc != TOVA_OK:
            raise TovaError(rc, "tova_prefill")

    def decode_steps_repositioned(self, q, k_new, v_new, out, evicted=None, rope_base=0.0, stream=None):
        """T steps on a cache of un-rotated keys, positions re-assigned before each attention."""
        c = self.cfg
        T = q.shape[0]
        self._check("q", q, (T, c.n_layers, c.batch, c.n_q_heads, c.head_dim))
        self._check("k_new", k_new, (T, c.n_layers, c.batch, c.n_kv_heads, c.head_dim))
        self._check("v_new", v_new, (T, c.n_layers, c.batch, c.n_kv_heads, c.head_dim))
        self._check("out", out, (T, c.n_layers, c.batch, c.n_q_heads, c.head_dim))
        ev = self._evicted_ptr(evicted, (T, *self.state_shape))
        rc = self.lib.tova_decode_steps_repositioned(self._h, T, q.data_ptr(), k_new.data_ptr(), v_new.data_ptr(),
                                                     out.data_ptr(), ev, float(rope_base), _stream_handle(stream))
        if rc != TOVA_OK:
            raise TovaError(rc, "tova_decode_steps_repositioned")

    def policy_step(self, attn_weights, k_new, v_new, evicted=None, stream=None):
        """The policy alone: attn_weights fp32 [L][B][H][k+1] computed by the caller over the slots + the new token."""
        c = self.cfg
        torch = self._torch
        if attn_weights.dtype != torch.float32 or not attn_weights.is_contiguous() \
                or tuple(attn_weights.shape) != (c.n_layers, c.batch, c.n_q_heads, c.capacity_k + 1) \
                or attn_weights.device != self.kv_mem.device:
            raise ValueError("attn_weights: expected contiguous float32 [L][B][H][k+1] on the cache's device")
        self._check("k_new", k_new, (c.n_layers, c.batch, c.n_kv_heads, c.head_dim))
        self._check("v_new", v_new, (c.n_layers, c.batch, c.n_kv_heads, c.head_dim))
        ev = self._evicted_ptr(evicted, self.state_shape)
        rc = self.lib.tova_policy_step(self._h, attn_weights.data_ptr(), k_new.data_ptr(), v_new.data_ptr(), ev,
                                       _stream_handle(stream))
        if rc != TOVA_OK:
            raise TovaError(rc, "tova_policy_step")

    def _evicted_ptr(self, evicted, shape):
        if evicted is None:
            return None
        if evicted.dtype != self._torch.int32 or not evicted.is_contiguous() \
                or tuple(evicted.shape) != tuple(shape) or evicted.device != self.kv_mem.device:
            raise ValueError(f"evicted: expected contiguous int32 {tuple(shape)} on {self.kv_mem.device}")
        return evicted.data_ptr()

    def destroy(self):
        if self._h:
            self.lib.tova_cache_destroy(self._h)
            self._h = c_void_p()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass
