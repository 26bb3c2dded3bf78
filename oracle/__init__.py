"""ctypes front end of the CPU oracle (TEST INFRASTRUCTURE ONLY).

Argument marshalling for `flp_oracle.c`; every definition lives in the C file.
Only the tests, the smoke check and the benchmark's cpu_baseline leg may import
this package; the product path never does.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liborc.so")
_lib = None
_default_threads = None

DTYPE_CODE = {"f32": 0, "f16": 1, "bf16": 2}


def set_variant(name):
    """Which build of flp_oracle.c the calls below go to: "parity" (double running sums; the default and the only
    one any comparison may use) or "f32acc" (fp32 running sums, -O3: the benchmark's second CPU timing)."""
    global _lib, _LIB_PATH
    _LIB_PATH = os.path.join(_HERE, {"parity": "liborc.so", "f32acc": "liborc_f32acc.so"}[name])
    _lib = None


def set_threads(n):
    """Number of OpenMP threads of the following oracle calls (0: all cores again)."""
    global _default_threads
    omp = C.CDLL("libgomp.so.1")
    if _default_threads is None:
        _default_threads = int(omp.omp_get_max_threads())      # what the environment gave the process
    omp.omp_set_num_threads(int(n) if n > 0 else _default_threads)


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            from . import build as _b
            _b.build()
        _lib = C.CDLL(_LIB_PATH)
        _lib.orc_alloc_create.restype = C.c_void_p
        _lib.orc_alloc_create.argtypes = [C.c_int64]
        _lib.orc_alloc_destroy.argtypes = [C.c_void_p]
        _lib.orc_alloc_num_free.restype = C.c_int64
        _lib.orc_alloc_num_free.argtypes = [C.c_void_p]
        _lib.orc_alloc_alloc.argtypes = [C.c_void_p, C.c_int32, C.c_void_p]
        _lib.orc_alloc_free.argtypes = [C.c_void_p, C.c_int32, C.c_void_p]
        _lib.orc_round_to_dtype.restype = C.c_double
        _lib.orc_round_to_dtype.argtypes = [C.c_double, C.c_int]
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


class OracleError(RuntimeError):
    def __init__(self, code):
        super().__init__("oracle returned %d" % code)
        self.code = code


def _chk(rc):
    if rc != 0:
        raise OracleError(rc)


class Allocator:
    """O1: LIFO free list of block ids (first allocations return 0,1,2,...)."""

    def __init__(self, n):
        self._h = lib().orc_alloc_create(int(n))

    def __del__(self):
        if getattr(self, "_h", None):
            lib().orc_alloc_destroy(self._h)
            self._h = None

    def alloc(self, n):
        out = np.empty(max(int(n), 0), dtype=np.int32)
        _chk(lib().orc_alloc_alloc(self._h, int(n), _p(out)))
        return out

    def free(self, ids):
        ids = _i32(ids)
        _chk(lib().orc_alloc_free(self._h, len(ids), _p(ids)))

    @property
    def num_free(self):
        return int(lib().orc_alloc_num_free(self._h))


def swap(dst_pool, src_pool, src_ids, dst_ids):
    """O2: dst_pool[dst_ids[k]] <- src_pool[src_ids[k]]; pools are [n_blocks, block_elems] arrays."""
    assert dst_pool.flags.c_contiguous and src_pool.flags.c_contiguous
    bb = dst_pool.shape[1] * dst_pool.itemsize
    assert bb == src_pool.shape[1] * src_pool.itemsize
    src_ids, dst_ids = _i32(src_ids), _i32(dst_ids)
    assert len(src_ids) == len(dst_ids)
    _chk(lib().orc_swap(_p(dst_pool), C.c_int64(dst_pool.shape[0]), _p(src_pool), C.c_int64(src_pool.shape[0]),
                        C.c_int64(bb), C.c_int32(len(src_ids)), _p(src_ids), _p(dst_ids)))


def segment(token_adapter, n_adapters):
    ta = _i32(token_adapter)
    T = len(ta)
    n_seg = C.c_int32(0)
    seg_adapter = np.zeros(max(n_adapters, 1), np.int32)
    seg_start = np.zeros(n_adapters + 1, np.int32)
    perm = np.zeros(max(T, 1), np.int32)
    _chk(lib().orc_segment(C.c_int32(T), _p(ta), C.c_int32(n_adapters), C.byref(n_seg), _p(seg_adapter),
                           _p(seg_start), _p(perm)))
    n = n_seg.value
    return seg_adapter[:n].copy(), seg_start[:n + 1].copy(), perm[:int(seg_start[n])].copy()


def lora_apply(pool, dtype, x, token_adapter, rank, scale, a_tab_off, a_row_base, b_tab_off, b_row_base,
               block_tables, d_out, y_in=None, w_base=None, sel=None):
    """O3.  pool: [n_blocks, block_elems] storage array; x: [T, d_in]; returns float64 [n_sel, d_out]."""
    assert pool.flags.c_contiguous and x.flags.c_contiguous
    T, d_in = x.shape
    ta = _i32(token_adapter)
    rank, a_tab_off, a_row_base = _i32(rank), _i32(a_tab_off), _i32(a_row_base)
    b_tab_off, b_row_base, block_tables = _i32(b_tab_off), _i32(b_row_base), _i32(block_tables)
    scale = np.ascontiguousarray(scale, dtype=np.float32)
    if y_in is not None:
        assert y_in.flags.c_contiguous and y_in.shape == (T, d_out)
    if w_base is not None:
        assert w_base.flags.c_contiguous and w_base.shape == (d_in, d_out)
    sel_a = None if sel is None else _i32(sel)
    n_sel = T if sel is None else len(sel_a)
    out = np.zeros((n_sel, d_out), dtype=np.float64)
    _chk(lib().orc_lora_apply(_p(pool), C.c_int(DTYPE_CODE[dtype]), C.c_int64(pool.shape[1]),
                              C.c_int32(T), C.c_int32(d_in), C.c_int32(d_out),
                              _p(x), C.c_int64(d_in), _p(y_in), C.c_int64(d_out), _p(w_base),
                              _p(ta), C.c_int32(len(rank)), _p(rank), _p(scale),
                              _p(a_tab_off), _p(a_row_base), _p(b_tab_off), _p(b_row_base), _p(block_tables),
                              C.c_int32(n_sel), _p(sel_a), _p(out)))
    return out


def lora_dense_delta(pool, dtype, d_in, d_out, r, table_a, a_row_base, table_b, b_row_base):
    table_a, table_b = _i32(table_a), _i32(table_b)
    dW = np.zeros((d_in, d_out), dtype=np.float64)
    _chk(lib().orc_lora_dense_delta(_p(pool), C.c_int(DTYPE_CODE[dtype]), C.c_int64(pool.shape[1]),
                                    C.c_int32(d_in), C.c_int32(d_out), C.c_int32(r), _p(table_a),
                                    C.c_int32(a_row_base), _p(table_b), C.c_int32(b_row_base), _p(dW)))
    return dW


def lora_write_row(pool, dtype, table, row, values):
    table = _i32(table)
    values = np.ascontiguousarray(values, dtype=pool.dtype)
    _chk(lib().orc_lora_write_row(_p(pool), C.c_int(DTYPE_CODE[dtype]), C.c_int64(pool.shape[1]), _p(table),
                                  C.c_int32(len(values)), C.c_int64(row), _p(values)))


def lora_read_row(pool, dtype, table, row_len, row):
    table = _i32(table)
    out = np.zeros(row_len, dtype=np.float64)
    _chk(lib().orc_lora_read_row(_p(pool), C.c_int(DTYPE_CODE[dtype]), C.c_int64(pool.shape[1]), _p(table),
                                 C.c_int32(row_len), C.c_int64(row), _p(out)))
    return out


def kv_append(pool, dtype, bt, n_kv, d, cu_new, prefix_len, tables, k_new, v_new):
    """O4 (in place on `pool`)."""
    cu_new, prefix_len = _i32(cu_new), _i32(prefix_len)
    tables = _i32(tables)
    assert pool.flags.c_contiguous and pool.shape[1] == 2 * bt * n_kv * d
    assert k_new.flags.c_contiguous and v_new.flags.c_contiguous
    S = len(prefix_len)
    _chk(lib().orc_kv_append(_p(pool), C.c_int(DTYPE_CODE[dtype]), C.c_int32(bt), C.c_int32(n_kv), C.c_int32(d),
                             C.c_int32(S), _p(cu_new), _p(prefix_len), _p(tables), C.c_int32(tables.shape[1]),
                             _p(k_new), _p(v_new)))


def kv_gather(pool, dtype, bt, n_kv, d, table, L):
    table = _i32(table)
    K = np.zeros((L, n_kv, d), dtype=np.float64)
    V = np.zeros((L, n_kv, d), dtype=np.float64)
    _chk(lib().orc_kv_gather(_p(pool), C.c_int(DTYPE_CODE[dtype]), C.c_int32(bt), C.c_int32(n_kv), C.c_int32(d),
                             _p(table), C.c_int32(L), _p(K), _p(V)))
    return K, V


def paged_attention(pool, dtype, bt, n_kv, d, n_h, cu_new, prefix_len, tables, q, sm_scale=0.0, sel=None,
                    want_wsum=False):
    """O5.  q: [T, n_h*d] or [T, n_h, d] storage array; returns float64 [n_sel, n_h, d] (and weight sums)."""
    cu_new, prefix_len, tables = _i32(cu_new), _i32(prefix_len), _i32(tables)
    S = len(prefix_len)
    T = int(cu_new[-1])
    assert q.flags.c_contiguous and q.size == T * n_h * d
    sel_a = None if sel is None else _i32(sel)
    n_sel = T if sel is None else len(sel_a)
    out = np.zeros((n_sel, n_h, d), dtype=np.float64)
    wsum = np.zeros((n_sel, n_h), dtype=np.float64) if want_wsum else None
    _chk(lib().orc_paged_attention(_p(pool), C.c_int(DTYPE_CODE[dtype]), C.c_int32(bt), C.c_int32(n_kv),
                                   C.c_int32(d), C.c_int32(S), C.c_int32(n_h), _p(cu_new), _p(prefix_len),
                                   _p(tables), C.c_int32(tables.shape[1]), _p(q), C.c_double(sm_scale),
                                   C.c_int32(n_sel), _p(sel_a), _p(out), _p(wsum)))
    return (out, wsum) if want_wsum else out


def contig_attention(K, V, q, P, sm_scale=0.0):
    K = np.ascontiguousarray(K, dtype=np.float64)
    V = np.ascontiguousarray(V, dtype=np.float64)
    q = np.ascontiguousarray(q, dtype=np.float64)
    L, n_kv, d = K.shape
    N, n_h, _ = q.shape
    assert L == P + N
    out = np.zeros((N, n_h, d), dtype=np.float64)
    _chk(lib().orc_contig_attention(_p(K), _p(V), _p(q), C.c_int32(P), C.c_int32(N), C.c_int32(n_h),
                                    C.c_int32(n_kv), C.c_int32(d), C.c_double(sm_scale), _p(out)))
    return out


def round_to_dtype(a, dtype):
    """Nearest-even rounding of float64 values to the storage format (values returned as float64)."""
    f = np.vectorize(lambda v: lib().orc_round_to_dtype(float(v), DTYPE_CODE[dtype]), otypes=[np.float64])
    return f(np.asarray(a, dtype=np.float64))


def num_threads():
    return int(lib().orc_num_threads())
