"""ctypes binding of include/flsched.h (argument marshalling only)."""
import ctypes as C

import numpy as np

from . import flpool

EXPORTS = ("fls_create", "fls_destroy", "fls_submit", "fls_poll", "fls_wait_next", "fls_stream_wait",
           "fls_compute_enqueued", "fls_complete", "fls_get_stats")


class Stats(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("submitted", "ready_returned", "waiting", "blocks_in", "blocks_out", "polls",
                                         "polls_empty")]


def _ids(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, (a.ctypes.data_as(C.c_void_p) if len(a) else None)


class Planner:
    """fls_sched handle on a flpool.Pool (manual=True: no pool needed, completion by complete())."""

    def __init__(self, pool=None, manual=False):
        L = flpool.load()
        vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
        L.fls_create.argtypes = [vp, i32, C.POINTER(vp)]
        L.fls_destroy.argtypes = [vp]
        L.fls_submit.argtypes = [vp, i64, i32, vp, vp, i32, vp, vp, i32]
        L.fls_poll.argtypes = [vp, i32, vp, C.POINTER(i32)]
        L.fls_wait_next.argtypes = [vp]
        L.fls_stream_wait.argtypes = [vp, i64, vp]
        L.fls_compute_enqueued.argtypes = [vp, vp]
        L.fls_complete.argtypes = [vp, i64]
        L.fls_get_stats.argtypes = [vp, C.POINTER(Stats)]
        for name in EXPORTS:
            getattr(L, name)
        self._lib, self._pool = L, pool
        h = vp()
        flpool._check(L.fls_create(pool._h if pool is not None else None, 1 if manual else 0, C.byref(h)))
        self._h = h
        if pool is not None:
            pool._dependents.add(self)

    def close(self):
        if getattr(self, "_h", None):
            self._lib.fls_destroy(self._h)
            self._h = None

    __del__ = close

    def submit(self, req_id, host_ids=(), dev_ids=(), out_dev_ids=(), out_host_ids=(), fetch_into_released=False,
               unhurried=False):
        h, hp = _ids(host_ids)
        d, dp = _ids(dev_ids)
        od, odp = _ids(out_dev_ids)
        oh, ohp = _ids(out_host_ids)
        if len(h) != len(d) or len(od) != len(oh):
            raise flpool.FlpError(flpool.FLP_EINVAL, "id lists of one direction must have equal lengths")
        flpool._check(self._lib.fls_submit(self._h, int(req_id), len(h), hp, dp, len(od), odp, ohp,
                                           (1 if fetch_into_released else 0) | (2 if unhurried else 0)))

    def poll(self, max_ready=1 << 20):
        out = np.zeros(max(1, min(max_ready, 1 << 20)), dtype=np.int64)
        n = C.c_int32(0)
        flpool._check(self._lib.fls_poll(self._h, min(max_ready, len(out)), out.ctypes.data_as(C.c_void_p), C.byref(n)))
        return out[:n.value].copy()

    def wait_next(self):
        flpool._check(self._lib.fls_wait_next(self._h))

    def stream_wait(self, req_id, stream):
        flpool._check(self._lib.fls_stream_wait(self._h, int(req_id), flpool._stream(stream)))

    def compute_enqueued(self, stream):
        flpool._check(self._lib.fls_compute_enqueued(self._h, flpool._stream(stream)))

    def complete(self, req_id):
        flpool._check(self._lib.fls_complete(self._h, int(req_id)))

    def stats(self):
        s = Stats()
        flpool._check(self._lib.fls_get_stats(self._h, C.byref(s)))
        return {n: int(getattr(s, n)) for n, _ in Stats._fields_}
