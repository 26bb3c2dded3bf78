"""ctypes binding of libflpool.so (see include/flpool.h).

Argument marshalling only: every step of the path runs in the HIP kernels.
Tensors are passed as anything with a `.data_ptr()` (torch tensors) or as raw
integer addresses; streams as torch streams or raw hipStream_t values.  There
is no CPU fallback: if the library is missing or a call fails, FlpError is
raised.
"""
from __future__ import annotations

import ctypes as C
import os
import weakref
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libflpool.so")

FLP_OK, FLP_EINVAL, FLP_ENOSPC, FLP_ERANGE, FLP_EDUP, FLP_EHIP, FLP_ENOTSUP = 0, -1, -2, -3, -4, -5, -6
DTYPE_CODE = {"f32": 0, "f16": 1, "bf16": 2}
TIER_DEVICE, TIER_HOST = 0, 1
MAX_PROJ = 4

EXPORTS = ("flp_pool_create", "flp_pool_destroy", "flp_pool_block_bytes", "flp_pool_num_free", "flp_pool_base",
           "flp_pool_alloc", "flp_pool_free", "flp_pool_swap_in", "flp_pool_swap_out", "flp_kv_append",
           "flp_paged_prefix_attention", "flp_lora_apply_paged", "flp_lora_segment", "flp_last_error",
           "flp_version", "flp_lora_apply_paged_static", "flp_static_scratch_bytes")


class FlpError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("flpool error %d: %s" % (code, msg))
        self.code = code


class PoolConfig(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("block_tokens", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("n_dev_blocks", C.c_int64), ("n_host_blocks", C.c_int64),
                ("dev_base", C.c_void_p), ("host_base", C.c_void_p)]


class AttnBatch(C.Structure):
    _fields_ = [("n_seqs", C.c_int32), ("n_q_heads", C.c_int32), ("max_blocks_per_seq", C.c_int32),
                ("sm_scale", C.c_float), ("q", C.c_void_p), ("k_new", C.c_void_p), ("v_new", C.c_void_p),
                ("out", C.c_void_p), ("cu_new", C.c_void_p), ("prefix_len", C.c_void_p),
                ("block_tables", C.c_void_p)]


class LoraProj(C.Structure):
    _fields_ = [("d_out", C.c_int32), ("w_base_layout", C.c_int32), ("ld_y", C.c_int64), ("y", C.c_void_p),
                ("w_base", C.c_void_p), ("a_tab_off", C.c_void_p), ("a_row_base", C.c_void_p),
                ("b_tab_off", C.c_void_p), ("b_row_base", C.c_void_p)]


class LoraBatch(C.Structure):
    _fields_ = [("n_tokens", C.c_int32), ("d_in", C.c_int32), ("ld_x", C.c_int64), ("n_adapters", C.c_int32),
                ("max_rank", C.c_int32), ("n_proj", C.c_int32), ("reserved", C.c_int32), ("x", C.c_void_p),
                ("token_adapter", C.c_void_p), ("rank", C.c_void_p), ("scale", C.c_void_p),
                ("block_tables", C.c_void_p), ("proj", LoraProj * MAX_PROJ)]


_lib = None


def load():
    """Load the shared library (raises if it has not been built)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FlpError(FLP_EINVAL, "libflpool.so is not built; run `python -m paper_2505_03756_amd.build` "
                                   "(or __graft_entry__.build()) first")
    # Device memory and streams come from torch, which ships a HIP runtime of its own: it has to be in the process
    # before this library is, so that both resolve to the one runtime (loaded the other way round, this library's
    # HIP calls report that there is no device).
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    lib.flp_pool_create.argtypes = [C.POINTER(PoolConfig), C.POINTER(vp)]
    lib.flp_pool_destroy.argtypes = [vp]
    lib.flp_pool_block_bytes.argtypes = [vp]
    lib.flp_pool_block_bytes.restype = i64
    lib.flp_pool_num_free.argtypes = [vp, i32]
    lib.flp_pool_num_free.restype = i64
    lib.flp_pool_base.argtypes = [vp, i32]
    lib.flp_pool_base.restype = vp
    lib.flp_pool_alloc.argtypes = [vp, i32, i32, vp]
    lib.flp_pool_free.argtypes = [vp, i32, i32, vp]
    lib.flp_pool_swap_in.argtypes = [vp, i32, vp, vp, vp]
    lib.flp_pool_swap_out.argtypes = [vp, i32, vp, vp, vp]
    lib.flp_kv_append.argtypes = [vp, C.POINTER(AttnBatch), vp]
    lib.flp_paged_prefix_attention.argtypes = [vp, C.POINTER(AttnBatch), vp]
    lib.flp_lora_apply_paged.argtypes = [vp, C.POINTER(LoraBatch), vp]
    lib.flp_lora_segment.argtypes = [vp, i32, vp, i32, vp, vp, vp, vp, vp]
    lib.flp_lora_apply_paged_static.argtypes = [vp, C.POINTER(LoraBatch), vp]
    lib.flp_static_scratch_bytes.restype = i64
    lib.flp_last_error.restype = C.c_char_p
    lib.flp_version.restype = C.c_char_p
    for name in EXPORTS:
        getattr(lib, name)
    _lib = lib
    return lib


def _check(rc):
    if rc != FLP_OK:
        raise FlpError(rc, load().flp_last_error().decode("utf-8", "replace"))


def _ptr(t):
    if t is None:
        return None
    if hasattr(t, "data_ptr"):
        return t.data_ptr()
    return int(t)


def _stream(s):
    if s is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if hasattr(s, "cuda_stream"):
        return s.cuda_stream
    return int(s)


def _host_i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(C.c_void_p)


class Pool:
    """flp_pool handle.  `dev` / `host` may be caller-owned tensors (kept alive here)."""

    def __init__(self, dtype: str, n_kv_heads: int, head_dim: int, n_dev_blocks: int, n_host_blocks: int,
                 block_tokens: int = 16, dev=None, host=None):
        self._lib = load()
        self.dtype = dtype
        self._keep = (dev, host)
        cfg = PoolConfig(DTYPE_CODE[dtype], block_tokens, n_kv_heads, head_dim, n_dev_blocks, n_host_blocks,
                         _ptr(dev), _ptr(host))
        h = C.c_void_p()
        _check(self._lib.flp_pool_create(C.byref(cfg), C.byref(h)))
        self._h = h
        self._dependents = weakref.WeakSet()   # objects created on this pool that must be closed before it
        self.block_bytes = int(self._lib.flp_pool_block_bytes(h))
        self.block_elems = 2 * block_tokens * n_kv_heads * head_dim

    def close(self):
        if getattr(self, "_h", None):
            for d in list(getattr(self, "_dependents", ())):   # a cache hands its blocks back to the pool it is closed on
                d.close()
            self._lib.flp_pool_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- a1
    def num_free(self, tier=TIER_DEVICE):
        return int(self._lib.flp_pool_num_free(self._h, tier))

    def base(self, tier=TIER_DEVICE):
        return self._lib.flp_pool_base(self._h, tier)

    def alloc(self, n, tier=TIER_DEVICE):
        out = np.empty(max(int(n), 0), dtype=np.int32)
        _check(self._lib.flp_pool_alloc(self._h, tier, int(n), out.ctypes.data_as(C.c_void_p)))
        return out

    def free(self, ids, tier=TIER_DEVICE):
        a, p = _host_i32(ids)
        _check(self._lib.flp_pool_free(self._h, tier, len(a), p))

    # ---- a2
    def swap_in(self, host_ids, dev_ids, stream=None):
        h, hp = _host_i32(host_ids)
        d, dp = _host_i32(dev_ids)
        if len(h) != len(d):
            raise FlpError(FLP_EINVAL, "swap lists differ in length")
        _check(self._lib.flp_pool_swap_in(self._h, len(h), hp, dp, _stream(stream)))

    def swap_out(self, dev_ids, host_ids, stream=None):
        d, dp = _host_i32(dev_ids)
        h, hp = _host_i32(host_ids)
        if len(h) != len(d):
            raise FlpError(FLP_EINVAL, "swap lists differ in length")
        _check(self._lib.flp_pool_swap_out(self._h, len(d), dp, hp, _stream(stream)))

    # ---- a6 / a7
    def _attn_batch(self, cu_new, prefix_len, block_tables, max_blocks, n_q_heads, q, out, k_new, v_new, sm_scale):
        cu, cup = _host_i32(cu_new)
        pl, plp = _host_i32(prefix_len)
        if len(cu) != len(pl) + 1:
            raise FlpError(FLP_EINVAL, "cu_new must have n_seqs + 1 entries")
        b = AttnBatch(len(pl), n_q_heads, max_blocks, float(sm_scale), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out),
                      cup, plp, _ptr(block_tables))
        return b, (cu, pl)

    def kv_append(self, k_new, v_new, cu_new, prefix_len, block_tables, max_blocks=None, stream=None):
        mb = block_tables.shape[1] if max_blocks is None else max_blocks
        b, keep = self._attn_batch(cu_new, prefix_len, block_tables, mb, 0, None, None, k_new, v_new, 0.0)
        _check(self._lib.flp_kv_append(self._h, C.byref(b), _stream(stream)))

    def paged_prefix_attention(self, q, out, cu_new, prefix_len, block_tables, n_q_heads, k_new=None, v_new=None,
                               sm_scale=0.0, max_blocks=None, stream=None):
        mb = block_tables.shape[1] if max_blocks is None else max_blocks
        b, keep = self._attn_batch(cu_new, prefix_len, block_tables, mb, n_q_heads, q, out, k_new, v_new, sm_scale)
        _check(self._lib.flp_paged_prefix_attention(self._h, C.byref(b), _stream(stream)))

    # ---- a3 / a4 / a5
    def lora_segment(self, token_adapter, n_tokens, n_adapters, n_seg, seg_adapter, seg_start, perm, stream=None):
        _check(self._lib.flp_lora_segment(self._h, int(n_tokens), _ptr(token_adapter), int(n_adapters), _ptr(n_seg),
                                          _ptr(seg_adapter), _ptr(seg_start), _ptr(perm), _stream(stream)))

    def lora_apply_paged(self, x, token_adapter, rank, scale, block_tables, projs: Sequence[dict], n_tokens, d_in,
                         n_adapters, max_rank, ld_x=None, stream=None, static=False):
        """projs: dicts with y, d_out, a_tab_off, a_row_base, b_tab_off, b_row_base and optional ld_y, w_base, w_base_layout
        (0: w_base is [d_in, d_out]; 1: [d_out, d_in]).  static=True calls flp_lora_apply_paged_static (same
        arguments, intermediates in the library's fixed scratch array, nothing allocated)."""
        if not 1 <= len(projs) <= MAX_PROJ:
            raise FlpError(FLP_EINVAL, "1..%d projections per call" % MAX_PROJ)
        b = LoraBatch()
        b.n_tokens, b.d_in, b.ld_x = int(n_tokens), int(d_in), int(d_in if ld_x is None else ld_x)
        b.n_adapters, b.max_rank, b.n_proj = int(n_adapters), int(max_rank), len(projs)
        b.x, b.token_adapter, b.rank, b.scale = _ptr(x), _ptr(token_adapter), _ptr(rank), _ptr(scale)
        b.block_tables = _ptr(block_tables)
        for i, p in enumerate(projs):
            pr = b.proj[i]
            pr.d_out = int(p["d_out"])
            pr.ld_y = int(p.get("ld_y", p["d_out"]))
            pr.y, pr.w_base = _ptr(p["y"]), _ptr(p.get("w_base"))
            pr.w_base_layout = int(p.get("w_base_layout", 0))
            pr.a_tab_off, pr.a_row_base = _ptr(p["a_tab_off"]), _ptr(p["a_row_base"])
            pr.b_tab_off, pr.b_row_base = _ptr(p["b_tab_off"]), _ptr(p["b_row_base"])
        fn = self._lib.flp_lora_apply_paged_static if static else self._lib.flp_lora_apply_paged
        _check(fn(self._h, C.byref(b), _stream(stream)))


def static_scratch_bytes():
    return int(load().flp_static_scratch_bytes())


def version():
    return load().flp_version().decode()
