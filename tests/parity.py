"""Shared driver of the GPU parity tests: runs the HIP path (through the C ABI) and the CPU
oracle side by side on the same seeded inputs and compares them after every call.

Bar: everything integer (unique keys, HIT/STALE/MISS classes, id -> slot map, clocks, policy
counters, evicted id sets, counters, global clocks) is compared exactly; fp32 values against
the fp64 oracle within 1e-5 relative + 1e-6 absolute (the order of the fp32 gradient sum and
fused multiply-adds differ)."""
from __future__ import annotations

import numpy as np
import torch

from oracle.het_oracle import Oracle
from paper_2112_07221_amd import hetcache as hc
from paper_2112_07221_amd import workloads as wl

RTOL, ATOL = 1e-5, 1e-6


def close(got, want, what):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    err = np.abs(got - want)
    bad = err > ATOL + RTOL * np.abs(want)
    assert not bad.any(), f"{what}: {int(bad.sum())} of {bad.size} values off, worst {err.max():.3e}"


class Pair:
    """A HIP cache and an oracle over equal tables."""

    def __init__(self, w: wl.Workload, table: np.ndarray, max_ids=None, host_backing=None, many_writers=False,
                 share_with: "Pair" = None, lfu_cap=None):
        """`many_writers`: the cache and the oracle are one of several workers over one global table
        (Evict pushes deltas); `share_with`: another Pair whose global table this one works on too."""
        self.w = w
        N = max_ids or w.n
        dev = torch.device("cuda:0")
        host = (w.backing == "host") if host_backing is None else host_backing
        self.oracle = Oracle(w.capacity, w.dim, w.s, w.policy, N, w.optimizer, w.eps, table, many_writers=many_writers,
                             share_with=share_with.oracle if share_with is not None else None, lfu_cap=lfu_cap)
        self.cache = hc.HetCache(w.capacity, w.dim, w.s, w.policy, N, w.optimizer, w.eps, many_writers=many_writers,
                                 lfu_cap=lfu_cap)
        if share_with is not None:
            self.W, self.A, self.Cg = share_with.W, share_with.A, share_with.Cg
        else:
            V = table.shape[0]
            if host:
                self.W = torch.from_numpy(table.astype(np.float32)).pin_memory()
                self.A = torch.zeros(V, w.dim if w.optimizer == 1 else 1).pin_memory() if w.optimizer else None
                self.Cg = torch.zeros(V, dtype=torch.int32).pin_memory()
            else:
                self.W = torch.from_numpy(table.astype(np.float32)).to(dev)
                self.A = torch.zeros(V, w.dim if w.optimizer == 1 else 1, device=dev) if w.optimizer else None    # (row-wise Adagrad: one per row)
                self.Cg = torch.zeros(V, dtype=torch.int32, device=dev)
        self.cache.attach_backing(self.W, self.A, self.Cg,
                                  hc.BACKING_PINNED_HOST if host else hc.BACKING_HBM)
        self.dev = dev
        self.offsets = None
        if w.pooled:
            self.offsets_np = wl.bag_offsets(w)
            self.offsets = torch.from_numpy(self.offsets_np).to(dev)

    # -- one Read on both sides, compared
    def lookup(self, ids_np, check_values=True, expect_rc=0, ids_dev=None):
        ids = torch.from_numpy(ids_np).to(self.dev) if ids_dev is None else ids_dev
        if self.w.pooled:
            out = torch.full((self.w.batch, self.w.dim), float("nan"), device=self.dev)
            self.cache.lookup_pooled(ids, self.offsets, out)
            want, rc = self.oracle.lookup_pooled(ids_np, self.offsets_np)
        else:
            out = torch.full((len(ids_np), self.w.dim), float("nan"), device=self.dev)
            self.cache.lookup(ids, out)
            want, rc = self.oracle.lookup(ids_np)
        assert rc == expect_rc
        keys, cls, slots = self.cache.last_lookup()
        okeys, ocls, oslots = self.oracle.last_lookup()
        assert np.array_equal(keys, okeys), "unique key sets differ"
        assert np.array_equal(cls, ocls), "HIT/STALE/MISS classes differ"
        assert np.array_equal(slots, oslots), "id -> slot maps differ"
        if check_values:
            close(out.cpu().numpy(), want, "lookup output")
        return out

    def update(self, ids_np, grads_np, lr=None, ids_dev=None):
        lr = self.w.lr if lr is None else lr
        ids = torch.from_numpy(ids_np).to(self.dev) if ids_dev is None else ids_dev
        g = torch.from_numpy(grads_np).to(self.dev)
        if self.w.pooled:
            self.cache.update_pooled(ids, self.offsets, g, lr)
            self.oracle.update_pooled(ids_np, self.offsets_np, grads_np, lr)
        else:
            self.cache.update(ids, g, lr)
            self.oracle.update(ids_np, grads_np, lr)
        assert np.array_equal(np.sort(self.cache.last_evicted()), np.sort(self.oracle.last_evicted())), \
            "evicted id sets differ"

    def compare_state(self, values=False):
        st, ost = self.cache.export_state(), self.oracle.export_state()
        for col in ("key", "slot", "cs", "cc", "last_use", "freq"):
            assert np.array_equal(st[col], ost[col]), f"cache column {col} differs"
        if values:
            rows, acc = self.cache.export_rows()
            orows, oacc = self.oracle.export_rows()
            close(rows, orows, "cached rows")
            if acc is not None:
                close(acc, oacc, "cached accumulators")

    def compare_counters(self):
        got = self.cache.stats()
        last, total = self.oracle.stats()
        olast = dict(last); ototal = dict(total)
        for d in (olast, ototal):
            d["unique"] = d.pop("U")
        assert got["last"] == olast, (got["last"], olast)
        assert got["total"] == ototal, (got["total"], ototal)
        assert got["resident"] == self.oracle.size
        assert got["iteration"] == self.oracle.iteration

    def compare_table(self):
        close(self.W.cpu().numpy(), self.oracle.W, "global table")
        if self.A is not None:
            close(self.A.cpu().numpy(), self.oracle.A, "global accumulators")
        assert np.array_equal(self.Cg.cpu().numpy().view(np.uint32), self.oracle.Cg), "global clocks differ"

    def flush_and_compare(self):
        rc = self.cache.flush()
        self.oracle.flush()
        assert rc == 0, hc.strerror(rc)
        close(self.W.cpu().numpy(), self.oracle.W, "global table after flush")
        if self.A is not None:
            close(self.A.cpu().numpy(), self.oracle.A, "global accumulators after flush")
        assert np.array_equal(self.Cg.cpu().numpy().view(np.uint32), self.oracle.Cg), "global clocks differ"
        self.compare_state(values=True)
        self.compare_counters()

    def close(self):
        self.cache.close()
        self.oracle.close()


def run_workload(w: wl.Workload, iters: int, state_every: int = 1, table=None, ids=None, grads=None,
                 values_every: int = 0, prefetch=False, lfu_cap=None):
    """Runs `iters` lookup+update iterations of workload `w` on both sides.  With `prefetch` the
    ids of iteration t+2 are announced before lookup t (prefetch="before", as the benchmark
    does), between lookup t and update t (prefetch=True or "between") or after update t
    (prefetch="after")."""
    table = wl.table_init(w) if table is None else table
    ids = wl.IdStream(w).batches(iters) if ids is None else ids
    grads = wl.grad_pool(w) if grads is None else grads
    p = Pair(w, table, lfu_cap=lfu_cap)
    try:
        ids_dev = torch.from_numpy(ids).to(p.dev) if prefetch else None
        for t in range(iters):
            if prefetch == "before":        # two batches ahead, as the benchmark does
                if t == 0 and iters > 1:
                    p.cache.prefetch(ids_dev[1])
                if t + 2 < iters:
                    p.cache.prefetch(ids_dev[t + 2])
            p.lookup(ids[t], ids_dev=ids_dev[t] if prefetch else None)
            if prefetch and prefetch not in ("after", "before") and t + 1 < iters:
                p.cache.prefetch(ids_dev[t + 1])
            p.update(ids[t], grads[t % len(grads)], ids_dev=ids_dev[t] if prefetch else None)
            if prefetch == "after" and t + 1 < iters:
                p.cache.prefetch(ids_dev[t + 1])
            if state_every and (t % state_every == 0 or t == iters - 1):
                p.compare_state(values=bool(values_every) and t % values_every == 0)
                p.compare_counters()
        p.flush_and_compare()
        return p.cache.stats()
    finally:
        p.close()
