"""ctypes binding of include/flcache.h (cache manager and cache swapper): argument marshalling only.
Every decision is taken inside libflpool.so; there is no Python fallback."""
import ctypes as C

import numpy as np

from . import flpool

EXPORTS = ("flc_create", "flc_destroy", "flc_add_lora", "flc_match", "flc_insert", "flc_release", "flc_tick",
           "flc_low_lora", "flc_eval", "flc_get_stats", "flc_snapshot")


class Config(C.Structure):
    _fields_ = [("block_tokens", C.c_int32), ("use_lru", C.c_int32), ("ignore_dependencies", C.c_int32),
                ("no_lora_reward", C.c_int32), ("upper", C.c_double), ("lower", C.c_double),
                ("pcie_bytes_per_s", C.c_double), ("time_scale_s", C.c_double)]


class Stats(C.Structure):
    _fields_ = [("n_nodes", C.c_int64), ("n_lora_nodes", C.c_int64), ("n_kv_nodes", C.c_int64),
                ("n_lora_hbm", C.c_int64), ("n_queries", C.c_int64), ("n_running", C.c_int64),
                ("hbm_blocks_held", C.c_int64), ("host_blocks_held", C.c_int64), ("invalid_kv_blocks", C.c_int64),
                ("usage", C.c_double)]


class NodeInfo(C.Structure):
    _fields_ = [("id", C.c_int32), ("kind", C.c_int32), ("parent", C.c_int32), ("tier", C.c_int32),
                ("first_block", C.c_int32), ("n_blocks", C.c_int32), ("pins", C.c_int32), ("pad", C.c_int32),
                ("visits", C.c_int64), ("last_use", C.c_double)]


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


class Cache:
    """flc_cache handle on a flpool.Pool (which must outlive it)."""

    def __init__(self, pool, block_tokens=16, upper=0.95, lower=0.70, pcie_bytes_per_s=64e9, time_scale_s=60.0,
                 use_lru=False, ignore_dependencies=False, no_lora_reward=False):
        self._lib = flpool.load()
        for name in EXPORTS:
            getattr(self._lib, name)
        vp, i32, i64, dbl = C.c_void_p, C.c_int32, C.c_int64, C.c_double
        L = self._lib
        L.flc_create.argtypes = [vp, C.POINTER(Config), C.POINTER(vp)]
        L.flc_destroy.argtypes = [vp]
        L.flc_add_lora.argtypes = [vp, i32, i32, i32, dbl, vp]
        L.flc_match.argtypes = [vp, i32, vp, i32, dbl, C.POINTER(i64), vp, i32, C.POINTER(i32), vp, i32,
                                C.POINTER(i32), vp, vp, i32, C.POINTER(i32)]
        L.flc_insert.argtypes = [vp, i64, vp, i32, vp, i32, dbl, vp, C.POINTER(i32)]
        L.flc_release.argtypes = [vp, i64]
        L.flc_tick.argtypes = [vp, dbl, i32, vp, vp, i32, C.POINTER(i32), vp, vp, i32, C.POINTER(i32), vp, i32,
                               C.POINTER(i32)]
        L.flc_low_lora.argtypes = [vp, i32, C.POINTER(dbl)]
        L.flc_eval.argtypes = [vp, i32, dbl, i32, C.POINTER(dbl)]
        L.flc_get_stats.argtypes = [vp, C.POINTER(Stats)]
        L.flc_snapshot.argtypes = [vp, vp, i64, C.POINTER(i64)]
        self.pool = pool
        self.bt = block_tokens
        cfg = Config(block_tokens, int(use_lru), int(ignore_dependencies), int(no_lora_reward), upper, lower,
                     pcie_bytes_per_s, time_scale_s)
        h = C.c_void_p()
        flpool._check(L.flc_create(pool._h, C.byref(cfg), C.byref(h)))
        self._h = h
        pool._dependents.add(self)             # closing the pool closes this cache first
        self._cap = 0
        self._grow(4096)

    def _grow(self, n):
        if n > self._cap:
            self._cap = int(n)
            self._bufs = [np.empty(self._cap, np.int32) for _ in range(5)]

    def close(self):
        if getattr(self, "_h", None):
            self._lib.flc_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def add_lora(self, lora_id, n_blocks, tier, now):
        out = np.empty(n_blocks, np.int32)
        flpool._check(self._lib.flc_add_lora(self._h, lora_id, n_blocks, tier, now, _p(out)))
        return out

    def match(self, lora_id, tokens, now, lora_cap=256):
        tok = _i32(tokens)
        nb = len(tok) // self.bt
        self._grow(lora_cap + nb)
        lb, kv, sh, sd = self._bufs[:4]
        q, nl, nk, ns = C.c_int64(), C.c_int32(), C.c_int32(), C.c_int32()
        flpool._check(self._lib.flc_match(self._h, lora_id, _p(tok), len(tok), now, C.byref(q), _p(lb), lora_cap,
                                          C.byref(nl), _p(kv), nb, C.byref(nk), _p(sh), _p(sd), lora_cap + nb,
                                          C.byref(ns)))
        lora_blocks = None if nl.value < 0 else lb[:nl.value].copy()
        return q.value, lora_blocks, kv[:nk.value].copy(), sh[:ns.value].copy(), sd[:ns.value].copy()

    def insert(self, query, tokens, new_blocks, now):
        tok, new = _i32(tokens), _i32(new_blocks)
        back = np.empty(max(len(new), 1), np.int32)
        nb = C.c_int32()
        flpool._check(self._lib.flc_insert(self._h, query, _p(tok), len(tok), _p(new), len(new), now, _p(back),
                                           C.byref(nb)))
        return back[:nb.value].copy()

    def release(self, query):
        flpool._check(self._lib.flc_release(self._h, query))

    def tick(self, now, batch_size, cap=None):
        if cap:
            self._grow(cap)
        cap = self._cap
        od, oh, ih, idv, dr = self._bufs
        no, ni, nd = C.c_int32(), C.c_int32(), C.c_int32()
        flpool._check(self._lib.flc_tick(self._h, now, batch_size, _p(od), _p(oh), cap, C.byref(no), _p(ih), _p(idv),
                                         cap, C.byref(ni), _p(dr), cap, C.byref(nd)))
        return ((od[:no.value].copy(), oh[:no.value].copy()), (ih[:ni.value].copy(), idv[:ni.value].copy()),
                dr[:min(nd.value, cap)].copy())

    def low_lora(self, batch_size):
        out = C.c_double()
        flpool._check(self._lib.flc_low_lora(self._h, batch_size, C.byref(out)))
        return out.value

    def eval(self, node_id, now, batch_size):
        out = C.c_double()
        flpool._check(self._lib.flc_eval(self._h, node_id, now, batch_size, C.byref(out)))
        return out.value

    def stats(self):
        s = Stats()
        flpool._check(self._lib.flc_get_stats(self._h, C.byref(s)))
        return {k: getattr(s, k) for k, _ in Stats._fields_}

    def snapshot(self):
        n = C.c_int64()
        flpool._check(self._lib.flc_snapshot(self._h, None, 0, C.byref(n)))
        rows = (NodeInfo * max(n.value, 1))()
        flpool._check(self._lib.flc_snapshot(self._h, rows, n.value, C.byref(n)))
        return [(r.id, r.kind, r.parent, r.tier, r.first_block, r.n_blocks, r.visits, r.last_use, r.pins)
                for r in rows[:n.value]]
