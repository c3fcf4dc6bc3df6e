"""ctypes binding of the C-ABI library (`include/het_cache.h`), same names, marshalling only.

PyTorch supplies device memory and the stream; every step of the cache path runs in the HIP
kernels of `libhet_cache.so`.  There is no fallback: if the library is missing or no GPU is
visible, `load()` raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhet_cache.so")

HET_OK, HET_EINVAL, HET_ENOMEM, HET_EHIP, HET_ERANGE, HET_ESTATE = 0, -1, -2, -3, -4, -5
POLICY_LRU, POLICY_LFU, POLICY_NONE, POLICY_LFU_LIGHT = 0, 1, 2, 3
OPT_SGD, OPT_ADAGRAD, OPT_ADAGRAD_ROWWISE = 0, 1, 2
BACKING_HBM, BACKING_PINNED_HOST = 0, 1
CLASS_HIT, CLASS_STALE, CLASS_MISS = 0, 1, 2
S_INFINITE = (1 << 63) - 1

EXPORTS = (
    "het_cache_create", "het_cache_configure", "het_attach_backing", "het_prefetch",
    "het_prefetch_cancel", "het_lookup",
    "het_lookup_pooled", "het_update", "het_update_pooled", "het_flush", "het_stats",
    "het_clear_error", "het_export_state", "het_export_rows", "het_last_lookup",
    "het_last_evicted", "het_cache_destroy", "het_strerror", "het_profile_begin",
    "het_profile_end", "het_profile_kernel_count", "het_profile_kernel_name", "het_profile_rows", "het_profile_trace",
    "het_lookup_nocache_static", "het_build_id", "het_cache_set_many_writers",
    "het_backing_foreign_update", "het_cache_set_lfu_cap",
)

COUNTER_FIELDS = ("n", "unique", "hit", "stale", "miss", "evicted", "evicted_dirty",
                  "stale_dirty", "flushed")


class Counters(C.Structure):
    _fields_ = [(f, C.c_int64) for f in COUNTER_FIELDS]

    def as_dict(self):
        return {f: getattr(self, f) for f in COUNTER_FIELDS}


class Stats(C.Structure):
    _fields_ = [("last", Counters), ("total", Counters), ("resident", C.c_int64),
                ("iteration", C.c_int64), ("error_bits", C.c_int32)]


class HetError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__(f"{what}: {strerror(status)} ({status})")


_lib = None


def load() -> C.CDLL:
    """Loads `libhet_cache.so` (built by `python -m paper_2112_07221_amd.build`)."""
    global _lib
    if _lib is not None:
        return _lib
    # PyTorch ships its own HIP runtime; importing it first makes that copy the process's only
    # one, so that torch's streams and device pointers are valid inside the library.
    import torch  # noqa: F401
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is not built; run `python -m paper_2112_07221_amd.build` (needs hipcc)")
    lib = C.CDLL(LIB_PATH)
    p, i64, i32 = C.c_void_p, C.c_int64, C.c_int32
    lib.het_cache_create.argtypes = [C.POINTER(p), i64, i32, i64, i32]
    lib.het_cache_configure.argtypes = [p, i64, i32, C.c_float, p]
    lib.het_attach_backing.argtypes = [p, p, p, p, i64, i32]
    lib.het_lookup.argtypes = [p, p, i64, p]
    lib.het_prefetch.argtypes = [p, p, i64]
    lib.het_prefetch_cancel.argtypes = [p]
    lib.het_cache_set_many_writers.argtypes = [p]
    lib.het_cache_set_lfu_cap.argtypes = [p, C.c_uint32]
    lib.het_backing_foreign_update.argtypes = [p, p, p, i64]
    lib.het_lookup_pooled.argtypes = [p, p, i64, p, i64, p]
    lib.het_update.argtypes = [p, p, p, i64, C.c_float]
    lib.het_update_pooled.argtypes = [p, p, i64, p, p, i64, C.c_float]
    lib.het_flush.argtypes = [p]
    lib.het_stats.argtypes = [p, C.POINTER(Stats)]
    lib.het_clear_error.argtypes = [p]
    lib.het_export_state.argtypes = [p] * 7 + [C.POINTER(i64)]
    lib.het_export_rows.argtypes = [p, p, p]
    lib.het_last_lookup.argtypes = [p, p, p, p, C.POINTER(i64)]
    lib.het_last_evicted.argtypes = [p, p, C.POINTER(i64)]
    lib.het_cache_destroy.argtypes = [p]
    lib.het_strerror.argtypes = [C.c_int]
    lib.het_strerror.restype = C.c_char_p
    lib.het_build_id.argtypes = []
    lib.het_build_id.restype = C.c_char_p
    lib.het_lookup_nocache_static.argtypes = [p, i64, i32, p, i64, p, p, p]
    lib.het_profile_begin.argtypes = [p]
    lib.het_profile_end.argtypes = [p, p, p, i32]
    lib.het_profile_kernel_count.argtypes = []
    lib.het_profile_trace.argtypes = [p, i32, p, i64]
    lib.het_profile_rows.argtypes = [i32, p, p, p, p, i64, i32, p, i32, i32, p, p]
    lib.het_profile_kernel_name.argtypes = [C.c_int]
    lib.het_profile_kernel_name.restype = C.c_char_p
    for name in EXPORTS:
        if name not in ("het_strerror", "het_profile_kernel_name", "het_build_id"):
            getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def build_id() -> str:
    return load().het_build_id().decode()


def strerror(status: int) -> str:
    return load().het_strerror(status).decode()


def _np_ptr(a):
    return a.ctypes.data_as(C.c_void_p)


def _check_dev(t, dtype, what):
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise TypeError(f"{what} must be a contiguous {dtype} tensor on the GPU")
    return t


NOALLOC_MAX_IDS = 65536


def lookup_nocache_static(table, ids, out, err_bits=None, stream=None):
    """out[i] = table[ids[i]] through het_lookup_nocache_static (no cache object, no allocation).
    Returns the status code."""
    import torch
    lib = load()
    _check_dev(ids, torch.int64, "ids"); _check_dev(out, torch.float32, "out")
    if table.dtype != torch.float32 or not table.is_contiguous() or table.dim() != 2:
        raise TypeError("table must be a contiguous fp32 matrix")
    if out.numel() < ids.numel() * table.shape[1]:
        raise ValueError("out is too small")
    st = stream if stream is not None else torch.cuda.current_stream()
    return lib.het_lookup_nocache_static(table.data_ptr(), table.shape[0], table.shape[1], ids.data_ptr(),
                                         ids.numel(), out.data_ptr(),
                                         err_bits.data_ptr() if err_bits is not None else None,
                                         C.c_void_p(st.cuda_stream))


PATTERN_COPY, PATTERN_GATHER, PATTERN_UPDATE = 0, 1, 2
TRACE_WORDS = 8


def profile_rows(pattern, x, a=None, src=None, idx=None, n=None, gidx=None, per=0, reps=20, stream=None):
    """Average milliseconds per launch of het_profile_rows' reference kernel (see the header).
    x, a, src: fp32 matrices of equal row width on the GPU; idx: int32 row numbers on the GPU."""
    import torch
    lib = load()
    _check_dev(x, torch.float32, "x")
    dim = x.shape[1]
    for t, what in ((a, "a"), (src, "src")):
        if t is not None:
            _check_dev(t, torch.float32, what)
            if t.dim() != 2 or t.shape[1] != dim:
                raise ValueError(f"{what} must have rows of {dim} floats")
    for t, what in ((idx, "idx"), (gidx, "gidx")):
        if t is not None:
            _check_dev(t, torch.int32, what)
    n = int(n if n is not None else (idx.numel() if idx is not None else x.shape[0]))
    if (idx is not None and idx.numel() < n) or (pattern != PATTERN_UPDATE and x.shape[0] < n) or \
            (per and (gidx is None or gidx.numel() < n * per)):
        raise ValueError("a buffer is too small for n rows")
    st = stream if stream is not None else torch.cuda.current_stream()
    ms = C.c_double()
    rc = lib.het_profile_rows(pattern, x.data_ptr(), a.data_ptr() if a is not None else None,
                              src.data_ptr() if src is not None else None, idx.data_ptr() if idx is not None else None,
                              n, dim, gidx.data_ptr() if gidx is not None else None, per, reps, C.byref(ms),
                              C.c_void_p(st.cuda_stream))
    if rc != 0:
        raise RuntimeError(f"het_profile_rows: {strerror(rc)}")
    return ms.value


class HetCache:
    """One cache object over one backing table.  Methods mirror the C entry points; tensor
    arguments must be contiguous GPU tensors (pinned host tensors for a host backing store).
    Calls are enqueued on the current torch stream captured at construction."""

    def __init__(self, capacity, dim, s, policy, max_batch_ids, optimizer=OPT_SGD, eps=0.0,
                 stream=None, many_writers=False, lfu_cap=None):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("the embedding-cache library needs a GPU; none is visible")
        self.lib = load()
        self.capacity, self.dim, self.max_batch_ids = capacity, dim, max_batch_ids
        self.n_slots = capacity + max_batch_ids
        self.optimizer = optimizer
        self._stream = stream if stream is not None else torch.cuda.current_stream()
        h = C.c_void_p()
        self._rc(self.lib.het_cache_create(C.byref(h), capacity, dim, s, policy), "het_cache_create")
        self.h = h
        if many_writers:
            self._rc(self.lib.het_cache_set_many_writers(h), "het_cache_set_many_writers")
        if lfu_cap is not None:
            self._rc(self.lib.het_cache_set_lfu_cap(h, lfu_cap), "het_cache_set_lfu_cap")
        self._rc(self.lib.het_cache_configure(h, max_batch_ids, optimizer, eps,
                                              C.c_void_p(self._stream.cuda_stream)),
                 "het_cache_configure")
        self._keep = None

    @staticmethod
    def _rc(status, what):
        if status != HET_OK:
            raise HetError(status, what)

    def attach_backing(self, table, state, cg, location=BACKING_HBM):
        """table [V, dim] fp32, state [V, dim] fp32 or None, cg [V] int32 (read as uint32, zeroed)."""
        import torch
        V = table.shape[0]
        for t, dt in ((table, torch.float32), (state, torch.float32), (cg, torch.int32)):
            if t is None:
                continue
            if t.dtype != dt or not t.is_contiguous():
                raise TypeError("backing arrays must be contiguous fp32 / int32 tensors")
            if location == BACKING_HBM and not t.is_cuda:
                raise TypeError("HBM backing arrays must live on the GPU")
            if location == BACKING_PINNED_HOST and not t.is_pinned():
                raise TypeError("host backing arrays must be pinned")
        self._keep = (table, state, cg)
        self._rc(self.lib.het_attach_backing(self.h, table.data_ptr(),
                                             state.data_ptr() if state is not None else None,
                                             cg.data_ptr(), V, location), "het_attach_backing")

    def prefetch(self, ids):
        import torch
        _check_dev(ids, torch.int64, "ids")
        self._rc(self.lib.het_prefetch(self.h, ids.data_ptr(), ids.numel()), "het_prefetch")

    def foreign_update(self, ids, deltas):
        import torch
        _check_dev(ids, torch.int64, "ids"); _check_dev(deltas, torch.float32, "deltas")
        if deltas.numel() < ids.numel() * self.dim:
            raise ValueError("deltas is too small")
        self._rc(self.lib.het_backing_foreign_update(self.h, ids.data_ptr(), deltas.data_ptr(), ids.numel()),
                 "het_backing_foreign_update")

    def prefetch_cancel(self):
        self._rc(self.lib.het_prefetch_cancel(self.h), "het_prefetch_cancel")

    def lookup(self, ids, out):
        import torch
        _check_dev(ids, torch.int64, "ids"); _check_dev(out, torch.float32, "out")
        if out.numel() < ids.numel() * self.dim:
            raise ValueError("out is too small")
        self._rc(self.lib.het_lookup(self.h, ids.data_ptr(), ids.numel(), out.data_ptr()), "het_lookup")

    def lookup_pooled(self, ids, offsets, out):
        import torch
        _check_dev(ids, torch.int64, "ids"); _check_dev(offsets, torch.int64, "offsets")
        _check_dev(out, torch.float32, "out")
        nb = offsets.numel() - 1
        if out.numel() < nb * self.dim:
            raise ValueError("out is too small")
        self._rc(self.lib.het_lookup_pooled(self.h, ids.data_ptr(), ids.numel(), offsets.data_ptr(),
                                            nb, out.data_ptr()), "het_lookup_pooled")

    def update(self, ids, grads, lr):
        import torch
        _check_dev(ids, torch.int64, "ids"); _check_dev(grads, torch.float32, "grads")
        if grads.numel() < ids.numel() * self.dim:
            raise ValueError("grads is too small")
        self._rc(self.lib.het_update(self.h, ids.data_ptr(), grads.data_ptr(), ids.numel(), lr),
                 "het_update")

    def update_pooled(self, ids, offsets, bag_grads, lr):
        import torch
        _check_dev(ids, torch.int64, "ids"); _check_dev(offsets, torch.int64, "offsets")
        _check_dev(bag_grads, torch.float32, "bag_grads")
        nb = offsets.numel() - 1
        if bag_grads.numel() < nb * self.dim:
            raise ValueError("bag_grads is too small")
        self._rc(self.lib.het_update_pooled(self.h, ids.data_ptr(), ids.numel(), offsets.data_ptr(),
                                            bag_grads.data_ptr(), nb, lr), "het_update_pooled")

    def flush(self):
        return self.lib.het_flush(self.h)

    def stats(self):
        st = Stats()
        self._rc(self.lib.het_stats(self.h, C.byref(st)), "het_stats")
        return {"last": st.last.as_dict(), "total": st.total.as_dict(), "resident": st.resident,
                "iteration": st.iteration, "error_bits": st.error_bits}

    def clear_error(self):
        self._rc(self.lib.het_clear_error(self.h), "het_clear_error")

    def export_state(self):
        P = self.n_slots
        keys = np.empty(P, np.int64); slots = np.empty(P, np.int32)
        cs, cc, lu, fr = (np.empty(P, np.uint32) for _ in range(4))
        n = C.c_int64()
        self._rc(self.lib.het_export_state(self.h, *map(_np_ptr, (keys, slots, cs, cc, lu, fr)),
                                           C.byref(n)), "het_export_state")
        r = n.value
        return {"key": keys[:r], "slot": slots[:r].astype(np.int64), "cs": cs[:r], "cc": cc[:r],
                "last_use": lu[:r], "freq": fr[:r]}

    def export_rows(self):
        r = int(self.stats()["resident"])
        rows = np.empty((r, self.dim), np.float32)
        acc = None
        if self.optimizer == OPT_ADAGRAD:
            acc = np.empty((r, self.dim), np.float32)
        elif self.optimizer == OPT_ADAGRAD_ROWWISE:
            acc = np.empty((r, 1), np.float32)
        self._rc(self.lib.het_export_rows(self.h, _np_ptr(rows), _np_ptr(acc) if acc is not None else None),
                 "het_export_rows")
        return rows, acc

    def last_lookup(self):
        N = self.max_batch_ids
        keys = np.empty(N, np.int64); cls = np.empty(N, np.int32); slots = np.empty(N, np.int32)
        n = C.c_int64()
        self._rc(self.lib.het_last_lookup(self.h, _np_ptr(keys), _np_ptr(cls), _np_ptr(slots),
                                          C.byref(n)), "het_last_lookup")
        u = n.value
        return keys[:u], cls[:u], slots[:u].astype(np.int64)

    def last_evicted(self):
        ids = np.empty(self.n_slots, np.int64)
        n = C.c_int64()
        self._rc(self.lib.het_last_evicted(self.h, _np_ptr(ids), C.byref(n)), "het_last_evicted")
        return ids[: n.value]

    def profile_begin(self):
        self._rc(self.lib.het_profile_begin(self.h), "het_profile_begin")

    def profile_end(self):
        """{kernel name: (total milliseconds, launches)} since profile_begin."""
        k = self.lib.het_profile_kernel_count()
        ms = np.zeros(k, np.float64); cnt = np.zeros(k, np.int64)
        self._rc(self.lib.het_profile_end(self.h, _np_ptr(ms), _np_ptr(cnt), k), "het_profile_end")
        return {self.lib.het_profile_kernel_name(i).decode(): (float(ms[i]), int(cnt[i]))
                for i in range(k) if cnt[i]}

    def profile_trace(self, records=None, kernel="apply_kernel"):
        """Switches the per-workgroup time stamps of `kernel` ("apply_kernel" or "fill_gather_kernel")
        on (records: zeroed int64 GPU tensor of shape [workgroups, TRACE_WORDS]) or off (None)."""
        import torch
        names = [self.lib.het_profile_kernel_name(i).decode() for i in range(self.lib.het_profile_kernel_count())]
        k = names.index(kernel)
        if records is None:
            self._rc(self.lib.het_profile_trace(self.h, k, None, 0), "het_profile_trace")
        else:
            _check_dev(records, torch.int64, "records")
            self._rc(self.lib.het_profile_trace(self.h, k, records.data_ptr(), records.shape[0]), "het_profile_trace")
        self._trace_records = getattr(self, "_trace_records", {})
        self._trace_records[kernel] = records

    def close(self):
        if getattr(self, "h", None):
            self.lib.het_cache_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
