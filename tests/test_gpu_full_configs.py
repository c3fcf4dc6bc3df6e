"""The stated configurations at their stated sizes and lengths, HIP path against the CPU oracle
through the C ABI (what the smaller cases of test_gpu_parity.py leave open)."""
import numpy as np
import pytest
import torch

from paper_2112_07221_amd import hetcache as hc
from paper_2112_07221_amd import workloads as wl
from parity import Pair, run_workload

pytestmark = pytest.mark.gpu


def free_run(p, ids, ids_dev, gdev, grads, t0, t1, out, announce=True):
    """Iterations [t0, t1) on both sides with no waiting call in between on the GPU side: the
    calls are only enqueued, as a training loop does (so a host-backed table's write-back is
    still staged when the next lookup's fetches come)."""
    w, T = p.w, len(ids)
    for t in range(t0, t1):
        if announce:
            if t == 0 and T > 1:
                p.cache.prefetch(ids_dev[1])
            if t + 2 < T:
                p.cache.prefetch(ids_dev[t + 2])
        if w.pooled:
            p.cache.lookup_pooled(ids_dev[t], p.offsets, out)
            p.cache.update_pooled(ids_dev[t], p.offsets, gdev[t % len(gdev)], w.lr)
            p.oracle.lookup_pooled(ids[t], p.offsets_np)
            p.oracle.update_pooled(ids[t], p.offsets_np, grads[t % len(grads)], w.lr)
        else:
            p.cache.lookup(ids_dev[t], out)
            p.cache.update(ids_dev[t], gdev[t % len(gdev)], w.lr)
            p.oracle.lookup(ids[t])
            p.oracle.update(ids[t], grads[t % len(grads)], w.lr)


@pytest.mark.timeout(600)
def test_config2_at_its_stated_length():
    """Config 2 exactly as stated: 1M ids, dim 64, 4096 x 26 lookups, LFU cache of 100k rows,
    s = 100, Adagrad, 1000 iterations, batches announced two ahead (what the benchmark times).
    Rows go stale from iteration 101 on.  Every integer of a Read (key set, classes, slots) and of
    the state (clocks, policy fields, evicted ids, counters) is compared every 100 iterations and
    over the last 50; values of the Reads there too; cached rows, accumulators and the whole
    global table at the end."""
    w = wl.WORKLOADS[2]
    T = w.iters
    ids = wl.IdStream(w).batches(T)
    grads = wl.grad_pool(w)
    p = Pair(w, wl.table_init(w))
    try:
        ids_dev = torch.from_numpy(ids).to(p.dev)
        gdev = [torch.from_numpy(g).to(p.dev) for g in grads]
        out = torch.empty(w.n, w.dim, device=p.dev)
        t = 0
        while t < T:
            checked = t % 100 == 0 or t >= T - 50
            if not checked:
                nxt = min((t // 100 + 1) * 100, T - 50)
                free_run(p, ids, ids_dev, gdev, grads, t, nxt, out)
                t = nxt
                continue
            if t == 0:
                p.cache.prefetch(ids_dev[1])
            if t + 2 < T:
                p.cache.prefetch(ids_dev[t + 2])
            p.lookup(ids[t], ids_dev=ids_dev[t])
            p.update(ids[t], grads[t % len(grads)], ids_dev=ids_dev[t])
            p.compare_state(values=False)
            p.compare_counters()
            t += 1
        st = p.cache.stats()
        assert st["total"]["stale"] > 0 and st["total"]["stale_dirty"] > 0 and st["total"]["evicted_dirty"] > 0
        p.flush_and_compare()
    finally:
        p.close()


@pytest.mark.timeout(600)
def test_config3_host_backed_cache_of_a_million_rows_overflowing_at_full_batch():
    """Config 3's launch shapes with the table in pinned host memory: 8192 x 26 ids, dim 128, LRU,
    SGD.  Cut: the vocabulary to 4M ids (so that the oracle's fp64 table fits in host memory)
    and the cache to 1M rows (so that it overflows within this run: 26 iterations fill it, every
    later one evicts about 24 000 rows); s = 3 so that rows also go stale.  The first 34 iterations
    run without a waiting call, as the benchmark does: the rows a trim evicts are still staged when
    the next lookup fetches, some of them the very keys it misses.  Then six iterations compared
    call by call."""
    w = wl.WORKLOADS[3].scaled(vocab=4_000_000, capacity=1_000_000, s=3)
    T, free = 40, 34
    ids = wl.IdStream(w).batches(T)
    grads = wl.grad_pool(w)
    p = Pair(w, wl.table_init(w))
    try:
        ids_dev = torch.from_numpy(ids).to(p.dev)
        gdev = [torch.from_numpy(g).to(p.dev) for g in grads]
        out = torch.empty(w.n, w.dim, device=p.dev)
        free_run(p, ids, ids_dev, gdev, grads, 0, free, out)
        p.compare_counters()
        st = p.cache.stats()
        assert st["total"]["evicted_dirty"] > 100_000 and st["total"]["stale_dirty"] > 0, st["total"]
        p.compare_state(values=True)
        for t in range(free, T):
            if t + 2 < T:
                p.cache.prefetch(ids_dev[t + 2])
            p.lookup(ids[t], ids_dev=ids_dev[t])
            p.update(ids[t], grads[t % len(grads)], ids_dev=ids_dev[t])
            p.compare_counters()
        p.compare_state(values=True)
        p.flush_and_compare()
    finally:
        p.close()


@pytest.mark.parametrize("policy,opt", [(wl.LRU, wl.SGD), (wl.LFU, wl.ADAGRAD)])
def test_host_backed_free_running_evictions_and_immediate_misses(policy, opt):
    """A small vocabulary behind a small cache in pinned host memory, driven without any waiting call
    for 40 iterations: every update's write-back leaves inside the next lookup's fetch kernel, and
    the keys it evicted are missed again at once (their rows come from the staging buffer).  State,
    counters and the flushed table are compared at the end only."""
    w = wl.WORKLOADS[1].scaled(vocab=3000, capacity=150, s=2, policy=policy, optimizer=opt, eps=1e-8, backing="host")
    T = 40
    ids = wl.IdStream(w).batches(T)
    grads = wl.grad_pool(w)
    p = Pair(w, wl.table_init(w))
    try:
        ids_dev = torch.from_numpy(ids).to(p.dev)
        gdev = [torch.from_numpy(g).to(p.dev) for g in grads]
        out = torch.empty(w.n, w.dim, device=p.dev)
        free_run(p, ids, ids_dev, gdev, grads, 0, T, out)
        p.compare_counters()
        assert p.cache.stats()["total"]["evicted_dirty"] > 1000
        p.compare_state(values=True)
        p.flush_and_compare()
    finally:
        p.close()


@pytest.mark.timeout(600)
@pytest.mark.parametrize("s", [0, 10, 100, 1000])
def test_config5_full_size_at_every_staleness_bound(s):
    """Config 5 at full size (1M tokens, dim 256, 2048 bags of 200, cache of 50k rows, Adagrad, pooled
    Read and Write, more unique ids per batch than cache rows) at each staleness bound of its sweep.
    With s = 0 every cached key that was updated is refreshed at its next Read."""
    w = wl.WORKLOADS[5].scaled(s=s)
    st = run_workload(w, 5, state_every=2, values_every=2, prefetch="before")
    assert st["total"]["evicted_dirty"] > 0
    if s == 0:
        assert st["total"]["stale_dirty"] > 0


@pytest.mark.parametrize("s", [0, 10, 100, 1000])
def test_config5_reduced_staleness_sweep_long_enough_to_go_stale(s):
    """Config 5's structure at a tenth of its size for 130 iterations: rows of popular tokens stay
    cached and go stale after s + 1 updates (s = 0, 10 and 100 refresh; s = 1000 never does)."""
    w = wl.WORKLOADS[5].scaled(vocab=100_000, dim=32, batch=128, capacity=12_000, s=s)
    st = run_workload(w, 130, state_every=13, values_every=65)
    if s <= 100:
        assert st["total"]["stale_dirty"] > 0
    else:
        assert st["total"]["stale"] == 0


def test_withdrawn_announcements_are_not_used():
    """het_prefetch_cancel: an announced batch that is withdrawn is sorted by its lookup itself, and a
    new buffer with other ids at the same address is not taken for the old announcement."""
    w = wl.WORKLOADS[1].scaled(capacity=400, s=3)
    ids_np = wl.IdStream(w).batches(5)
    g = wl.grad_pool(w)
    p = Pair(w, wl.table_init(w))
    try:
        d = torch.from_numpy(ids_np).cuda()
        buf = d[3].clone()
        p.cache.prefetch(d[1]); p.cache.prefetch(buf)
        p.lookup(ids_np[0], ids_dev=d[0]); p.update(ids_np[0], g[0], ids_dev=d[0])     # carry stages of both sorts
        p.cache.prefetch_cancel()
        buf.copy_(d[4])                                   # the same address now holds other ids
        p.lookup(ids_np[4], ids_dev=buf); p.update(ids_np[4], g[1], ids_dev=buf)
        p.lookup(ids_np[1], ids_dev=d[1]); p.update(ids_np[1], g[2], ids_dev=d[1])
        assert p.cache.stats()["error_bits"] == 0
        p.compare_state(values=True); p.compare_counters()
        p.flush_and_compare()
    finally:
        p.close()


@pytest.mark.parametrize("policy,opt", [(wl.LRU, wl.SGD), (wl.LFU, wl.ADAGRAD)])
def test_rows_fetched_ahead_are_used_only_by_the_lookup_they_were_fetched_for(policy, opt):
    """Host-backed table: while an update runs, the rows the announced batch will miss are brought into
    HBM on a stream beside the main one.  Here the announced batch does not come next, comes later, is
    withdrawn, or comes after a flush; rows evicted or updated in between must come from where they
    are then (cache, staging buffer, table), never from a copy fetched ahead that has gone stale."""
    w = wl.WORKLOADS[1].scaled(vocab=3000, capacity=150, s=2, policy=policy, optimizer=opt, eps=1e-8, backing="host")
    T = 12
    ids = wl.IdStream(w).batches(T)
    g = wl.grad_pool(w)
    p = Pair(w, wl.table_init(w))
    try:
        d = torch.from_numpy(ids).to(p.dev)
        step = lambda t, gi: (p.lookup(ids[t], ids_dev=d[t]), p.update(ids[t], g[gi % len(g)], ids_dev=d[t]))
        p.cache.prefetch(d[1])
        step(0, 0)                      # lists batch 1 and fetches its rows ahead
        step(2, 1)                      # another batch comes first (and lists batch 1 again, after its own changes)
        step(1, 2)                      # now the announced one
        p.compare_state(values=True); p.compare_counters()
        p.cache.prefetch(d[3])
        step(4, 3)                      # lists batch 3
        p.cache.prefetch_cancel()       # withdrawn: batch 3 sorts and fetches for itself
        step(3, 4)
        p.cache.prefetch(d[5])
        step(6, 5)
        assert p.cache.flush() == 0     # a flush in between: announcements are void
        p.oracle.flush()
        step(5, 6)
        p.cache.prefetch(d[7]); p.cache.prefetch(d[8])
        for t in (9, 7, 8):             # free running: nothing waits between these calls
            p.cache.lookup(d[t], torch.empty(w.n, w.dim, device=p.dev))
            p.cache.update(d[t], torch.from_numpy(g[t % len(g)]).to(p.dev), w.lr)
            p.oracle.lookup(ids[t]); p.oracle.update(ids[t], g[t % len(g)], w.lr)
        p.compare_state(values=True); p.compare_counters()
        p.flush_and_compare()
    finally:
        p.close()
