"""ctypes binding of the layer glue (include/fllayer.h): argument marshalling only.

Tensors are anything with `data_ptr()` (torch tensors serve as device memory) or raw addresses.
"""
import ctypes as C

import numpy as np

from . import flpool
from .flpool import _check, _ptr, _stream

EXPORTS = ("fll_rmsnorm", "fll_add_rmsnorm", "fll_rope", "fll_silu_mul", "fll_layer_scratch_bytes",
           "fll_layer_forward")
PROJ_ORDER = ("q", "k", "v", "o", "gate", "up", "down")


class LayerConfig(C.Structure):
    _fields_ = [("hidden", C.c_int32), ("n_q_heads", C.c_int32), ("mlp_dim", C.c_int32), ("rms_eps", C.c_float),
                ("rope_theta", C.c_float), ("reserved", C.c_int32)]


class LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("in_norm", "post_norm", "wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")]


class LoraPlace(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("a_tab_off", "a_row_base", "b_tab_off", "b_row_base")]


class LayerBatch(C.Structure):
    _fields_ = [("n_tokens", C.c_int32), ("n_seqs", C.c_int32), ("n_adapters", C.c_int32), ("max_rank", C.c_int32),
                ("max_blocks_per_seq", C.c_int32), ("reserved", C.c_int32), ("cu_new", C.c_void_p),
                ("prefix_len", C.c_void_p), ("positions", C.c_void_p), ("kv_tables", C.c_void_p),
                ("token_adapter", C.c_void_p), ("rank", C.c_void_p), ("scale", C.c_void_p), ("lora_tables", C.c_void_p),
                ("lora", LoraPlace * 7)]


_ready = False


def _lib():
    global _ready
    L = flpool.load()
    if not _ready:
        vp, i32, i64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
        for name in EXPORTS:
            getattr(L, name)
        L.fll_rmsnorm.argtypes = [i32, vp, vp, vp, i32, i32, f32, vp]
        L.fll_add_rmsnorm.argtypes = [i32, vp, vp, vp, vp, i32, i32, f32, vp]
        L.fll_rope.argtypes = [i32, vp, vp, vp, i32, i32, i32, i32, f32, vp]
        L.fll_silu_mul.argtypes = [i32, vp, i64, vp, i64, vp, i64, i32, i32, vp]
        L.fll_layer_scratch_bytes.argtypes = [vp, C.POINTER(LayerConfig), i32]
        L.fll_layer_scratch_bytes.restype = i64
        L.fll_layer_forward.argtypes = [vp, C.POINTER(LayerConfig), C.POINTER(LayerWeights), C.POINTER(LayerBatch), vp,
                                        vp, i64, vp]
        _ready = True
    return L


def _dt(dtype):
    return flpool.DTYPE_CODE[dtype] if isinstance(dtype, str) else int(dtype)


def rmsnorm(dtype, x, w, y, n_tokens, hidden, eps=1e-5, stream=None):
    _check(_lib().fll_rmsnorm(_dt(dtype), _ptr(x), _ptr(w), _ptr(y), n_tokens, hidden, eps, _stream(stream)))


def add_rmsnorm(dtype, resid, delta, w, y, n_tokens, hidden, eps=1e-5, stream=None):
    _check(_lib().fll_add_rmsnorm(_dt(dtype), _ptr(resid), _ptr(delta), _ptr(w), _ptr(y), n_tokens, hidden, eps,
                                  _stream(stream)))


def rope(dtype, q, k, positions, n_tokens, n_q_heads, n_kv_heads, head_dim, theta=10000.0, stream=None):
    _check(_lib().fll_rope(_dt(dtype), _ptr(q), _ptr(k), _ptr(positions), n_tokens, n_q_heads, n_kv_heads, head_dim,
                           theta, _stream(stream)))


def silu_mul(dtype, gate, up, out, n_tokens, width, ld_gate=None, ld_up=None, ld_out=None, stream=None):
    _check(_lib().fll_silu_mul(_dt(dtype), _ptr(gate), ld_gate or width, _ptr(up), ld_up or width, _ptr(out),
                               ld_out or width, n_tokens, width, _stream(stream)))


class Layer:
    """One decoder layer's configuration and weights, bound to the pool that holds its KV blocks and LoRA pages."""

    def __init__(self, pool, hidden, n_q_heads, mlp_dim, weights, rms_eps=1e-5, rope_theta=10000.0):
        """weights: dict in_norm, post_norm [hidden]; q, k, v, o, gate, up, down as [d_out, d_in] device tensors."""
        self.pool = pool
        self.cfg = LayerConfig(hidden, n_q_heads, mlp_dim, rms_eps, rope_theta, 0)
        self._keep = dict(weights)
        self.w = LayerWeights(_ptr(weights["in_norm"]), _ptr(weights["post_norm"]), _ptr(weights["q"]),
                              _ptr(weights["k"]), _ptr(weights["v"]), _ptr(weights["o"]), _ptr(weights["gate"]),
                              _ptr(weights["up"]), _ptr(weights["down"]))

    def scratch_bytes(self, n_tokens):
        n = _lib().fll_layer_scratch_bytes(self.pool._h, C.byref(self.cfg), n_tokens)
        if n < 0:
            raise flpool.FlpError(flpool.FLP_EINVAL, "fll_layer_scratch_bytes: bad layer shape")
        return int(n)

    def forward(self, batch, h, scratch, scratch_bytes, stream=None):
        _check(_lib().fll_layer_forward(self.pool._h, C.byref(self.cfg), C.byref(self.w), C.byref(batch.c), _ptr(h),
                                        _ptr(scratch), scratch_bytes, _stream(stream)))


class Batch:
    """The per-step arguments of Layer.forward (kept alive here)."""

    def __init__(self, cu_new, prefix_len, positions, kv_tables, token_adapter, rank, scale, lora_tables, places,
                 n_adapters, max_rank, max_blocks_per_seq):
        """cu_new, prefix_len: host int32 arrays; the rest device tensors; places: dict projection name ->
        dict(a_tab_off, a_row_base, b_tab_off, b_row_base) of device tensors."""
        self._cu = np.ascontiguousarray(cu_new, dtype=np.int32)
        self._pl = np.ascontiguousarray(prefix_len, dtype=np.int32)
        self._keep = (positions, kv_tables, token_adapter, rank, scale, lora_tables, places)
        c = LayerBatch()
        c.n_tokens, c.n_seqs = int(self._cu[-1]), len(self._pl)
        c.n_adapters, c.max_rank, c.max_blocks_per_seq = n_adapters, max_rank, max_blocks_per_seq
        c.cu_new, c.prefix_len = self._cu.ctypes.data, self._pl.ctypes.data
        c.positions, c.kv_tables = _ptr(positions), _ptr(kv_tables)
        c.token_adapter, c.rank, c.scale, c.lora_tables = _ptr(token_adapter), _ptr(rank), _ptr(scale), _ptr(lora_tables)
        for i, name in enumerate(PROJ_ORDER):
            pl = places.get(name)
            if pl is not None:
                c.lora[i] = LoraPlace(_ptr(pl["a_tab_off"]), _ptr(pl["a_row_base"]), _ptr(pl["b_tab_off"]),
                                      _ptr(pl["b_row_base"]))
        self.c = c
