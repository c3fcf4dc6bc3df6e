"""ctypes access to the C oracle (`het_oracle.c`).  Test infrastructure only.

Argument marshalling and nothing else: every rule of the method lives in the C file.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
HIT, STALE, MISS = 0, 1, 2
ERR_RANGE, ERR_STATE, ERR_ARG = 1, 2, 4
S_INF = (1 << 63) - 1
STAT_FIELDS = ("n", "U", "hit", "stale", "miss", "evicted", "evicted_dirty", "stale_dirty",
               "flushed")

_libs = {}


def _load(real: str):
    if real in _libs:
        return _libs[real]
    name = "libhet_oracle.so" if real == "f64" else "libhet_oracle_f32.so"
    path = os.path.join(_HERE, name)
    if not os.path.exists(path):
        from . import build as _b
        _b.build()
    lib = C.CDLL(path)
    p, i64, i32 = C.c_void_p, C.c_int64, C.c_int32
    rl = C.c_double if real == "f64" else C.c_float
    lib.het_oracle_create.restype = p
    lib.het_oracle_create.argtypes = [i64, i32, i64, i32, i64, i32, C.c_double]
    lib.het_oracle_attach.argtypes = [p, p, p, p, i64]
    lib.het_oracle_destroy.argtypes = [p]
    lib.het_oracle_destroy.restype = None
    lib.het_oracle_lookup.argtypes = [p, p, i64, p]
    lib.het_oracle_lookup_pooled.argtypes = [p, p, i64, p, i64, p]
    lib.het_oracle_update.argtypes = [p, p, p, i64, rl]
    lib.het_oracle_update_pooled.argtypes = [p, p, i64, p, p, i64, rl]
    lib.het_oracle_flush.argtypes = [p]
    lib.het_oracle_set_many_writers.argtypes = [p]
    lib.het_oracle_set_lfu_cap.argtypes = [p, C.c_uint32]
    lib.het_oracle_foreign_update.argtypes = [p, p, p, i64]
    for f in ("export_state", "export_rows", "last_lookup", "last_evicted", "size", "iteration"):
        getattr(lib, "het_oracle_" + f).restype = i64
    lib.het_oracle_export_state.argtypes = [p] * 7
    lib.het_oracle_export_rows.argtypes = [p, p, p]
    lib.het_oracle_last_lookup.argtypes = [p, p, p, p]
    lib.het_oracle_last_evicted.argtypes = [p, p]
    lib.het_oracle_stats.argtypes = [p, p]
    lib.het_oracle_stats.restype = None
    lib.het_oracle_size.argtypes = [p]
    lib.het_oracle_iteration.argtypes = [p]
    lib.het_oracle_error.argtypes = [p]
    lib.het_oracle_clear_error.argtypes = [p]
    lib.het_oracle_clear_error.restype = None
    _libs[real] = lib
    return lib


def _ptr(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


class Oracle:
    """One cache over one global table, on host arrays.  `table` (fp32 or fp64 [V, D]) is copied;
    the oracle's own global table is `self.W` (and `self.A`, `self.Cg`)."""

    def __init__(self, capacity, dim, s, policy, max_batch_ids, optimizer, eps, table,
                 real: str = "f64", many_writers: bool = False, share_with: "Oracle" = None, lfu_cap: int = None):
        """`many_writers`: this cache is one of several workers' (Evict pushes deltas).
        `share_with`: another Oracle whose global table (W, A, Cg) this one works on too;
        `table` is then ignored."""
        self.lib = _load(real)
        self.dtype = np.float64 if real == "f64" else np.float32
        self.dim, self.P = dim, capacity + max_batch_ids
        self.h = self.lib.het_oracle_create(capacity, dim, s, policy, max_batch_ids, optimizer,
                                            float(eps))
        if not self.h:
            raise ValueError("het_oracle_create rejected the arguments")
        if lfu_cap is not None and self.lib.het_oracle_set_lfu_cap(self.h, lfu_cap):
            raise ValueError("het_oracle_set_lfu_cap rejected the cap")
        if many_writers and self.lib.het_oracle_set_many_writers(self.h):
            raise ValueError("het_oracle_set_many_writers failed")
        if share_with is not None:
            self.W, self.A, self.Cg = share_with.W, share_with.A, share_with.Cg
        else:
            self.W = np.ascontiguousarray(table, dtype=self.dtype).copy()
            self.A = np.zeros_like(self.W) if optimizer == 1 else (np.zeros((self.W.shape[0], 1), self.dtype) if optimizer == 2 else None)
            self.Cg = np.zeros(self.W.shape[0], dtype=np.uint32)
        V = self.W.shape[0]
        rc = self.lib.het_oracle_attach(self.h, _ptr(self.W), _ptr(self.A), _ptr(self.Cg), V)
        if rc:
            raise ValueError("het_oracle_attach rejected the arguments")

    def close(self):
        if self.h:
            self.lib.het_oracle_destroy(self.h)
            self.h = None

    def __del__(self):
        self.close()

    def lookup(self, ids):
        ids = np.ascontiguousarray(ids, dtype=np.int64)
        out = np.empty((ids.size, self.dim), dtype=self.dtype)
        rc = self.lib.het_oracle_lookup(self.h, _ptr(ids), ids.size, _ptr(out))
        return out, rc

    def lookup_pooled(self, ids, offsets):
        ids = np.ascontiguousarray(ids, dtype=np.int64)
        offsets = np.ascontiguousarray(offsets, dtype=np.int64)
        nb = offsets.size - 1
        out = np.empty((nb, self.dim), dtype=self.dtype)
        rc = self.lib.het_oracle_lookup_pooled(self.h, _ptr(ids), ids.size, _ptr(offsets), nb,
                                               _ptr(out))
        return out, rc

    def update(self, ids, grads, lr):
        ids = np.ascontiguousarray(ids, dtype=np.int64)
        g = np.ascontiguousarray(grads, dtype=self.dtype)
        return self.lib.het_oracle_update(self.h, _ptr(ids), _ptr(g), ids.size, float(lr))

    def update_pooled(self, ids, offsets, bag_grads, lr):
        ids = np.ascontiguousarray(ids, dtype=np.int64)
        offsets = np.ascontiguousarray(offsets, dtype=np.int64)
        g = np.ascontiguousarray(bag_grads, dtype=self.dtype)
        return self.lib.het_oracle_update_pooled(self.h, _ptr(ids), ids.size, _ptr(offsets),
                                                 _ptr(g), offsets.size - 1, float(lr))

    def flush(self):
        return self.lib.het_oracle_flush(self.h)

    def foreign_update(self, ids, deltas):
        ids = np.ascontiguousarray(ids, dtype=np.int64)
        d = np.ascontiguousarray(deltas, dtype=self.dtype)
        return self.lib.het_oracle_foreign_update(self.h, _ptr(ids), _ptr(d), ids.size)

    def export_state(self):
        P = self.P
        keys, slots = np.empty(P, np.int64), np.empty(P, np.int64)
        cs, cc, lu, fr = (np.empty(P, np.uint32) for _ in range(4))
        r = self.lib.het_oracle_export_state(self.h, *map(_ptr, (keys, slots, cs, cc, lu, fr)))
        return {"key": keys[:r], "slot": slots[:r], "cs": cs[:r], "cc": cc[:r],
                "last_use": lu[:r], "freq": fr[:r]}

    def export_rows(self):
        rows = np.empty((self.P, self.dim), self.dtype)
        acc = np.empty((self.P, self.A.shape[1]), self.dtype) if self.A is not None else None
        r = self.lib.het_oracle_export_rows(self.h, _ptr(rows), _ptr(acc))
        return rows[:r], (acc[:r] if acc is not None else None)

    def last_lookup(self):
        n = self.P
        keys, cls, slots = np.empty(n, np.int64), np.empty(n, np.int32), np.empty(n, np.int64)
        u = self.lib.het_oracle_last_lookup(self.h, _ptr(keys), _ptr(cls), _ptr(slots))
        return keys[:u], cls[:u], slots[:u]

    def last_evicted(self):
        ids = np.empty(self.P, np.int64)
        r = self.lib.het_oracle_last_evicted(self.h, _ptr(ids))
        return ids[:r]

    def stats(self):
        buf = np.zeros(18, np.int64)
        self.lib.het_oracle_stats(self.h, _ptr(buf))
        return (dict(zip(STAT_FIELDS, buf[:9].tolist())), dict(zip(STAT_FIELDS, buf[9:].tolist())))

    @property
    def size(self):
        return self.lib.het_oracle_size(self.h)

    @property
    def iteration(self):
        return self.lib.het_oracle_iteration(self.h)

    @property
    def error(self):
        return self.lib.het_oracle_error(self.h)

    def clear_error(self):
        self.lib.het_oracle_clear_error(self.h)
