"""HIP path against the CPU oracle, through the C ABI, on an MI355X."""
import numpy as np
import pytest
import torch

from paper_2112_07221_amd import hetcache as hc
from paper_2112_07221_amd import workloads as wl
from parity import Pair, close, run_workload

pytestmark = pytest.mark.gpu


def test_prefetch_changes_nothing_and_an_unused_prefetch_is_harmless():
    """Announcing the next ids only moves their sort into the kernels of the calls in between; a
    lookup with other ids than the announced ones sorts for itself."""
    w = wl.WORKLOADS[1].scaled(policy=wl.LFU, s=2)
    run_workload(w, 25, state_every=1, values_every=5, prefetch="before")
    run_workload(w, 25, state_every=1, values_every=5, prefetch="between")
    run_workload(w, 25, state_every=1, values_every=5, prefetch="after")
    ids_np = wl.IdStream(w).batches(4)
    g = wl.grad_pool(w)
    p = Pair(w, wl.table_init(w))
    try:
        d = torch.from_numpy(ids_np).cuda()
        p.lookup(ids_np[0], ids_dev=d[0])
        p.cache.prefetch(d[3])                     # announced, never looked up next
        p.update(ids_np[0], g[0], ids_dev=d[0])
        p.lookup(ids_np[1], ids_dev=d[1])
        p.update(ids_np[1], g[1], ids_dev=d[1])
        p.cache.prefetch(d[2])
        p.cache.prefetch(d[2])                     # twice is allowed
        p.lookup(ids_np[2], ids_dev=d[2])
        p.update(ids_np[2], g[2])                  # other buffer: sorted afresh
        p.compare_state(values=True); p.compare_counters()
        p.flush_and_compare()
    finally:
        p.close()


def test_tiny_config_full_length():
    """Config 1 as stated: 10k ids, dim 16, 128 x 26 lookups, LRU cache of 1000, s = 10, SGD,
    100 iterations, every integer of the state compared after every iteration."""
    st = run_workload(wl.WORKLOADS[1], 100, state_every=1, values_every=10)
    assert st["total"]["stale"] > 0 and st["total"]["evicted"] > 0


@pytest.mark.parametrize("policy", [wl.LRU, wl.LFU])
@pytest.mark.parametrize("opt", [wl.SGD, wl.ADAGRAD])
@pytest.mark.parametrize("s", [0, 3, hc.S_INFINITE])
def test_policies_optimizers_staleness(policy, opt, s):
    w = wl.WORKLOADS[1].scaled(policy=policy, optimizer=opt, s=s, eps=1e-8, lr=0.05)
    run_workload(w, 30, state_every=1, values_every=7)


@pytest.mark.parametrize("dim", [1, 10, 16, 64, 128, 130, 256, 260, 1000, 1023, 4096])
def test_row_widths(dim):
    """Row groups of 1..64 lanes, the vector and the scalar row path, one to sixteen row pieces per
    lane (the widest rows the library takes: 4096 floats, or 1024 if the width is no multiple of 4)."""
    w = wl.WORKLOADS[1].scaled(dim=dim, optimizer=wl.ADAGRAD, eps=1e-8, policy=wl.LFU, s=2)
    run_workload(w, 12, state_every=3, values_every=3)


@pytest.mark.parametrize("cap,host", [(1, False), (4, False), (4, True), (16, False)])
def test_light_weight_lfu(cap, host):
    """HET_POLICY_LFU_LIGHT (Section 4.3): rows used `cap` times are no longer kept track of.  The
    oracle applies the same rule, so the comparison is as exact as for the other policies."""
    w = wl.WORKLOADS[1].scaled(policy=wl.LFU_LIGHT, s=3, optimizer=wl.ADAGRAD, eps=1e-8, capacity=700,
                               backing="host" if host else "hbm")
    st = run_workload(w, 40, state_every=1, values_every=8, prefetch="before", lfu_cap=cap)
    assert st["total"]["evicted"] > 0 and (cap == 1 or st["total"]["stale"] > 0)      # (cap 1 is first in, first out: nothing stays long enough)


def test_light_weight_lfu_config2_full_size():
    w = wl.WORKLOADS[2].scaled(policy=wl.LFU_LIGHT, s=5)
    st = run_workload(w, 20, state_every=5, values_every=10, prefetch="before", lfu_cap=4)
    assert st["total"]["evicted_dirty"] > 0


def test_config2_shape_reduced():
    """Config 2's structure (26 fields, Zipf 1.05, LFU, Adagrad, s = 100) at a tenth of its
    size, long enough for rows to go stale: several sort tiles, ragged last tile."""
    w = wl.WORKLOADS[2].scaled(vocab=100_000, batch=411, capacity=10_000, s=20)
    st = run_workload(w, 120, state_every=10, values_every=40)
    assert st["total"]["stale"] > 0


def test_config2_full_size():
    """Config 2 at full size in the launch configuration the benchmark times: 1M ids, dim 64,
    4096 x 26 lookups, LFU cache of 100k, Adagrad, the next batch's ids announced ahead."""
    w = wl.WORKLOADS[2].scaled(s=5)
    st = run_workload(w, 24, state_every=6, values_every=12, prefetch="before")
    assert st["total"]["stale"] > 0 and st["total"]["evicted"] > 0


def test_two_runs_are_bit_identical():
    """No ordering decision and no floating-point sum depends on the arrival order of atomics:
    two runs of the same stream (config 2 at full size, batches announced ahead) end with the
    same bits in every cached row and accumulator, every slot's state and the whole global table."""
    w = wl.WORKLOADS[2].scaled(s=5)
    T = 12
    table = wl.table_init(w)
    ids = wl.IdStream(w).batches(T)
    grads = wl.grad_pool(w)
    dev = torch.device("cuda:0")
    ids_dev = torch.from_numpy(ids).to(dev)
    gdev = [torch.from_numpy(g).to(dev) for g in grads]
    results = []
    for _ in range(2):
        W = torch.from_numpy(table.astype(np.float32)).to(dev)
        A = torch.zeros_like(W)
        Cg = torch.zeros(w.vocab, dtype=torch.int32, device=dev)
        cache = hc.HetCache(w.capacity, w.dim, w.s, w.policy, w.n, w.optimizer, w.eps)
        try:
            cache.attach_backing(W, A, Cg, hc.BACKING_HBM)
            out = torch.empty(w.n, w.dim, device=dev)
            outs = []
            for t in range(T):
                if t == 0:
                    cache.prefetch(ids_dev[1])
                if t + 2 < T:
                    cache.prefetch(ids_dev[t + 2])
                cache.lookup(ids_dev[t], out)
                outs.append(out.cpu().numpy().copy())
                cache.update(ids_dev[t], gdev[t % len(gdev)], w.lr)
            st = cache.export_state()
            rows, acc = cache.export_rows()
            assert cache.flush() == 0
            results.append((outs, st, rows, acc, W.cpu().numpy(), A.cpu().numpy(), Cg.cpu().numpy()))
        finally:
            cache.close()
    a, b = results
    for x, y in zip(a[0], b[0]):
        assert np.array_equal(x.view(np.uint32), y.view(np.uint32)), "lookup outputs differ between runs"
    for col in a[1]:
        assert np.array_equal(a[1][col], b[1][col]), f"cache column {col} differs between runs"
    for i, what in ((2, "cached rows"), (3, "cached accumulators"), (4, "global table"), (5, "global accumulators")):
        assert np.array_equal(a[i].view(np.uint32), b[i].view(np.uint32)), f"{what} differ between runs"
    assert np.array_equal(a[6], b[6])


@pytest.mark.parametrize("cfg", [4, 5])
def test_configs_4_and_5_full_size(cfg):
    """Configs 4 (skip-gram, 4M nodes, dim 128) and 5 (bag-of-words, pooled, dim 256, more unique ids
    than cache rows) at full size, in the benchmark's launch configuration, for a few iterations."""
    w = wl.WORKLOADS[cfg]
    w = w.scaled(s=2) if cfg == 4 else w.scaled(s=3)
    st = run_workload(w, 8, state_every=4, values_every=4, prefetch="before")
    assert st["total"]["evicted_dirty"] > 0


def test_config3_full_batch_and_cache_host_backed():
    """Config 3's launch shapes (8192 x 26 ids, dim 128, cache of 2M rows, LRU, table in pinned host
    memory), with the vocabulary cut to 4M so that the oracle's fp64 table fits in host memory.
    (The cache starts cold and holds every row for the length of this run; evictions over the
    host link are covered by the smaller host-backed cases.)"""
    w = wl.WORKLOADS[3].scaled(vocab=4_000_000, s=2)
    run_workload(w, 6, state_every=3, values_every=3, prefetch="before")


def test_config4_shape_reduced():
    w = wl.WORKLOADS[4].scaled(vocab=400_000, batch=2048, capacity=40_000, s=4)
    run_workload(w, 30, state_every=5, values_every=10)


def test_config5_pooled_more_uniques_than_capacity():
    """Bag-of-words shape: pooled lookup, and more unique ids per batch than cache rows, so
    rows of the current batch are evicted at the end of the update."""
    w = wl.WORKLOADS[5].scaled(vocab=100_000, batch=256, capacity=5_000, s=3)
    st = run_workload(w, 20, state_every=4, values_every=8)
    assert st["total"]["unique"] // 40 > w.capacity        # 20 lookups + 20 updates


def test_config3_pinned_host_backing_reduced():
    """Config 3's structure with the global table in pinned host memory."""
    w = wl.WORKLOADS[3].scaled(vocab=2_000_000, batch=2048, capacity=100_000, s=5)
    run_workload(w, 16, state_every=4, values_every=8)


def test_announcements_far_ahead_out_of_order_and_too_many():
    """Up to three batches stand announced; a fourth replaces the oldest; lookups may come in another
    order than the announcements, or with ids never announced.  Nothing of it changes a result."""
    w = wl.WORKLOADS[1].scaled(vocab=100_000, batch=300, capacity=2_000, s=1, policy=wl.LFU)   # 17-bit ids: three passes
    ids_np = wl.IdStream(w).batches(10)
    g = wl.grad_pool(w)
    p = Pair(w, wl.table_init(w))
    try:
        d = torch.from_numpy(ids_np).cuda()
        for t in (1, 2, 3, 4):                      # four announcements: the one for batch 1 is dropped
            p.cache.prefetch(d[t])
        order = [0, 1, 3, 2, 4, 5]                  # 0 never announced, 1 dropped, 3 before 2 (which voids 2's announcement)
        for i, t in enumerate(order):
            if t == 4:
                p.cache.prefetch(d[5])
            p.lookup(ids_np[t], ids_dev=d[t])
            p.update(ids_np[t], g[i % len(g)], ids_dev=d[t])
            p.compare_state(values=True); p.compare_counters()
        p.flush_and_compare()
    finally:
        p.close()


@pytest.mark.parametrize("policy,opt", [(wl.LRU, wl.SGD), (wl.LFU, wl.ADAGRAD)])
def test_host_backed_table_rows_evicted_and_fetched_again_at_once(policy, opt):
    """A small vocabulary behind a small cache in pinned host memory: keys evicted by one update are
    missed again by the next lookup, while their write-back is still on its way to the table."""
    w = wl.WORKLOADS[1].scaled(vocab=3000, capacity=150, s=2, policy=policy, optimizer=opt, backing="host")
    st = run_workload(w, 30, state_every=1, values_every=3, prefetch="before")
    assert st["total"]["evicted_dirty"] > 1000
    # Read after Read, and a waiting call between update and lookup (it sends the staged rows itself)
    ids_np = wl.IdStream(w).batches(6)
    g = wl.grad_pool(w)
    p = Pair(w, wl.table_init(w))
    try:
        for t in range(6):
            p.lookup(ids_np[t])
            if t % 2 == 0:
                p.lookup(ids_np[(t + 3) % 6])
                p.update(ids_np[(t + 3) % 6], g[t % len(g)])
            else:
                p.update(ids_np[t], g[t % len(g)])
            if t == 3:
                p.cache.stats()
            p.compare_state(values=True); p.compare_counters()
        p.flush_and_compare()
    finally:
        p.close()


@pytest.mark.parametrize("cfg,opt,host", [(1, wl.SGD, False), (1, wl.ADAGRAD, True), (5, wl.ADAGRAD, False)])
def test_no_cache_mode_is_uncached_training(cfg, opt, host):
    """HET_POLICY_NONE reads and writes the global table itself.  The oracle's cache is
    transparent (its pins: every Read equals uncached training, and after a flush so does the
    table), so its outputs and its flushed table are what uncached training gives."""
    from oracle.het_oracle import Oracle
    w = wl.WORKLOADS[cfg].scaled(optimizer=opt)
    if cfg == 5:
        w = w.scaled(vocab=50_000, batch=128, capacity=2_000)
    table = wl.table_init(w)
    ids_np = wl.IdStream(w).batches(12)
    g_np = wl.grad_pool(w)
    oracle = Oracle(w.capacity, w.dim, w.s, w.policy, w.n, w.optimizer, w.eps, table)
    cache = hc.HetCache(1, w.dim, 0, hc.POLICY_NONE, w.n, w.optimizer, w.eps)
    dev = torch.device("cuda:0")
    V = table.shape[0]
    W = torch.from_numpy(table.astype(np.float32))
    W = W.pin_memory() if host else W.to(dev)
    A = None
    if w.optimizer:
        A = torch.zeros(V, w.dim).pin_memory() if host else torch.zeros(V, w.dim, device=dev)
    Cg = torch.zeros(V, dtype=torch.int32).pin_memory() if host else torch.zeros(V, dtype=torch.int32, device=dev)
    cache.attach_backing(W, A, Cg, hc.BACKING_PINNED_HOST if host else hc.BACKING_HBM)
    offs_np = wl.bag_offsets(w) if w.pooled else None
    offs = torch.from_numpy(offs_np).to(dev) if w.pooled else None
    try:
        d = torch.from_numpy(ids_np).to(dev)
        for t in range(12):
            out = torch.full((w.n_grad_rows, w.dim), float("nan"), device=dev)
            g = torch.from_numpy(g_np[t % len(g_np)]).to(dev)
            if t + 1 < 12:
                cache.prefetch(d[t + 1])
            if w.pooled:
                cache.lookup_pooled(d[t], offs, out)
                want, _ = oracle.lookup_pooled(ids_np[t], offs_np)
            else:
                cache.lookup(d[t], out)
                want, _ = oracle.lookup(ids_np[t])
            close(out.cpu().numpy(), want, "lookup output")
            keys, cls, slots = cache.last_lookup()
            assert np.array_equal(keys, oracle.last_lookup()[0]) and np.array_equal(slots, keys)
            # every other update hands over a copy of the ids: the path that sorts for itself
            ids_for_update = d[t] if t % 2 == 0 else d[t].clone()
            if w.pooled:
                cache.update_pooled(ids_for_update, offs, g, w.lr)
                oracle.update_pooled(ids_np[t], offs_np, g_np[t % len(g_np)], w.lr)
            else:
                cache.update(ids_for_update, g, w.lr)
                oracle.update(ids_np[t], g_np[t % len(g_np)], w.lr)
        st = cache.stats()
        assert st["resident"] == 0 and st["error_bits"] == 0 and st["total"]["unique"] == oracle.stats()[1]["U"]
        assert cache.flush() == 0
        oracle.flush()
        close(W.cpu().numpy(), oracle.W, "global table")
        if A is not None:
            close(A.cpu().numpy(), oracle.A, "global accumulators")
    finally:
        cache.close(); oracle.close()


def test_ragged_and_degenerate_batches():
    """Batches of 1, 63, 64, 65, 1023, 1025, 2047, 2049 ids, all-equal ids, already-unique ids."""
    w = wl.WORKLOADS[1].scaled(capacity=300, s=1)
    table = wl.table_init(w)
    rng = np.random.default_rng(5)
    p = Pair(w, table, max_ids=4096)
    try:
        for n in (1, 63, 64, 65, 1023, 1025, 2047, 2049, 4096):
            for kind in ("zipf", "same", "unique"):
                if kind == "zipf":
                    ids = (rng.zipf(1.3, size=n) % w.vocab).astype(np.int64)
                elif kind == "same":
                    ids = np.full(n, int(rng.integers(w.vocab)), dtype=np.int64)
                else:
                    ids = rng.permutation(w.vocab)[:n].astype(np.int64)
                g = rng.standard_normal((n, w.dim)).astype(np.float32)
                p.lookup(ids)
                p.update(ids, g)
                p.compare_state(values=True)
                p.compare_counters()
        p.flush_and_compare()
    finally:
        p.close()


@pytest.mark.parametrize("dim,tile", [(64, 64), (128, 64), (256, 128), (520, 128)])
def test_two_very_long_runs_next_to_each_other(dim, tile):
    """Two neighbouring keys that each fill dozens of the update's tiles (sums of such runs are added
    up in groups of tiles first).  The second run starts in the middle of the tile in which the first
    ends, and that tile is the first of a group of the first run: both runs' group sums meet there."""
    w = wl.WORKLOADS[1].scaled(dim=dim, capacity=300, s=2, optimizer=wl.ADAGRAD, eps=1e-8, policy=wl.LFU)
    table = wl.table_init(w)
    rng = np.random.default_rng(17)
    a, b = 500, 501
    before = rng.integers(0, a, size=tile // 2)                 # keys below both: the first run starts in the middle of tile 0
    n_a, n_b, n_rest = tile * 32, tile * 20 + 7, 300
    n = len(before) + n_a + n_b + n_rest
    p = Pair(w, table, max_ids=n)
    try:
        for it in range(3):
            ids = np.concatenate([before, np.full(n_a, a), np.full(n_b, b), rng.integers(b + 1, w.vocab, size=n_rest)]).astype(np.int64)
            ids = ids[rng.permutation(n)]
            g = rng.standard_normal((n, w.dim)).astype(np.float32)
            p.lookup(ids)
            p.update(ids, g)
            p.compare_state(values=True)
            p.compare_counters()
        p.flush_and_compare()
    finally:
        p.close()


@pytest.mark.parametrize("dim,n", [(10, 3000), (64, 3000), (260, 2000), (260, 40_000), (64, 300_000)])
def test_long_runs_that_cover_whole_workgroups(dim, n):
    """A few keys hold most of the batch: the optimizer step's workgroups that lie inside one run
    leave one partial sum each (row groups of 1, 16 and 64 lanes; both chunk sizes)."""
    w = wl.WORKLOADS[1].scaled(dim=dim, capacity=400, s=2, optimizer=wl.ADAGRAD, eps=1e-8, policy=wl.LFU)
    table = wl.table_init(w)
    rng = np.random.default_rng(11)
    p = Pair(w, table, max_ids=n)
    try:
        hot = rng.permutation(w.vocab)[:3]
        for it in range(3):
            u = rng.random(n)
            ids = rng.integers(0, w.vocab, size=n)
            ids[u < 0.85] = hot[2]; ids[u < 0.65] = hot[1]; ids[u < 0.45] = hot[0]
            ids = ids.astype(np.int64)
            g = rng.standard_normal((n, w.dim)).astype(np.float32)
            p.lookup(ids)
            p.update(ids, g)
            p.compare_state(values=True)
            p.compare_counters()
        p.flush_and_compare()
    finally:
        p.close()


FUZZ_ITERATIONS = 36


@pytest.mark.parametrize("seed,host", [(1, False), (2, False), (3, True), (4, False), (5, False), (6, False), (7, False)])
def test_random_call_sequences(seed, host):
    """Seeded random mixes of the calls: batches of random size and skew, announcements of coming
    (and of never used) batches, lookups that no update follows, updates that sort their own ids,
    flushes in between.  State and counters are compared after every iteration."""
    rng = np.random.default_rng(100 + seed)
    N = 6000
    w = wl.WORKLOADS[1].scaled(dim=int(rng.choice([8, 16, 48, 128])), capacity=int(rng.choice([150, 700, 3000])),
                               s=int(rng.choice([0, 2, 50])), policy=int(rng.choice([wl.LRU, wl.LFU])),
                               optimizer=int(rng.choice([wl.SGD, wl.ADAGRAD])), eps=1e-8)
    table = wl.table_init(w)

    def batch():
        n = int(rng.choice([1, 7, 64, 255, 1024, 1025, 2500, 4097, N]))
        kind = rng.integers(4)
        if kind == 0:
            ids = rng.zipf(1.2, size=n) % w.vocab
        elif kind == 1:
            ids = rng.integers(0, w.vocab, size=n)
        elif kind == 2:
            ids = rng.integers(0, w.vocab, size=n)
            ids[rng.random(n) < 0.7] = int(rng.integers(w.vocab))
        else:
            ids = rng.permutation(w.vocab)[:n]
        return ids.astype(np.int64)

    T = FUZZ_ITERATIONS
    p = Pair(w, table, max_ids=N, host_backing=host)
    try:
        batches = [batch() for _ in range(T)]
        dev = [torch.from_numpy(b).to(p.dev) for b in batches]
        extra = [batch() for _ in range(6)]
        extra_dev = [torch.from_numpy(b).to(p.dev) for b in extra]
        for t in range(T):
            for _ in range(int(rng.integers(0, 3))):
                k = t + int(rng.integers(0, 4))
                if k < T:
                    p.cache.prefetch(dev[k])
            if rng.random() < 0.15:
                p.cache.prefetch(extra_dev[int(rng.integers(3))])          # never looked up
            if rng.random() < 0.15:
                e = 3 + int(rng.integers(3))
                p.lookup(extra[e], ids_dev=extra_dev[e])                   # a lookup that no update follows
            p.lookup(batches[t], ids_dev=dev[t])
            g = rng.standard_normal((len(batches[t]), w.dim)).astype(np.float32)
            mode = rng.random()
            if mode < 0.7:
                p.update(batches[t], g, ids_dev=dev[t])
            elif mode < 0.85:
                p.update(batches[t], g)                                    # same ids elsewhere: sorted again
            p.compare_state(values=t % 4 == 0)
            p.compare_counters()
            if rng.random() < 0.1:
                p.flush_and_compare()
        p.flush_and_compare()
    finally:
        p.close()


@pytest.mark.parametrize("policy", [wl.LRU, wl.LFU])
def test_beyond_2048_iterations_the_select_takes_more_passes(policy):
    """The policy keys grow with the iteration count: past iteration 2047 they need one more
    select pass (LRU two, LFU three), and more stages than the update's kernels can carry."""
    w = wl.WORKLOADS[1].scaled(batch=40, capacity=600, s=5, policy=policy, optimizer=wl.ADAGRAD, eps=1e-8)
    T = 2120
    table = wl.table_init(w)
    ids = wl.IdStream(w).batches(T)
    grads = wl.grad_pool(w)
    p = Pair(w, table)
    try:
        ids_dev = torch.from_numpy(ids).to(p.dev)
        for t in range(T):
            if t + 2 < T:
                p.cache.prefetch(ids_dev[t + 2])
            p.lookup(ids[t], check_values=t % 64 == 0 or t >= 2040, ids_dev=ids_dev[t])
            p.update(ids[t], grads[t % len(grads)], ids_dev=ids_dev[t])
            if t % 128 == 0 or t >= 2040:
                p.compare_state(values=t % 16 == 0)
                p.compare_counters()
        p.flush_and_compare()
    finally:
        p.close()


def test_beyond_65536_iterations_lfu_select_of_four_passes():
    """LFU keys are twice as wide as the iteration count: from iteration 65536 the select has four
    passes, one stage more than the update's kernels carry.  Most iterations run unchecked (both
    sides get the same calls); the integers of the state (keys, slots, clocks, policy fields,
    evicted ids, counters) are compared now and then and over the last 200 iterations.  Row values
    are not: fp32 rounding against the fp64 oracle adds up over 65 000 optimizer steps."""
    w = wl.WORKLOADS[1].scaled(batch=8, capacity=300, s=5, policy=wl.LFU, optimizer=wl.SGD)
    T = 65_700
    table = wl.table_init(w)
    ids = wl.IdStream(w).batches(T)
    grads = wl.grad_pool(w)
    p = Pair(w, table)
    try:
        ids_dev = torch.from_numpy(ids).to(p.dev)
        gdev = [torch.from_numpy(g).to(p.dev) for g in grads]
        out = torch.empty(ids.shape[1], w.dim, device=p.dev)
        for t in range(T):
            checked = t % 8192 == 0 or t >= T - 200
            if checked:
                p.lookup(ids[t], check_values=False, ids_dev=ids_dev[t])
                p.update(ids[t], grads[t % len(grads)], ids_dev=ids_dev[t])
                p.compare_state(values=False)
                p.compare_counters()
            else:
                p.cache.lookup(ids_dev[t], out)
                p.oracle.lookup(ids[t])
                p.cache.update(ids_dev[t], gdev[t % len(grads)], w.lr)
                p.oracle.update(ids[t], grads[t % len(grads)], w.lr)
        assert p.cache.flush() == 0
        p.oracle.flush()
        assert np.array_equal(p.Cg.cpu().numpy().view(np.uint32), p.oracle.Cg), "global clocks differ"
        p.compare_state(values=False)
        p.compare_counters()
    finally:
        p.close()


def test_largest_batch_the_library_accepts():
    """2^20 ids in one call (1024 probe tiles, 1024 sort tiles, the long-chunk optimizer step), one
    id more is refused at configuration."""
    n = 1 << 20
    w = wl.WORKLOADS[1].scaled(vocab=300_000, dim=8, capacity=50_000, s=1, policy=wl.LFU, optimizer=wl.ADAGRAD, eps=1e-8)
    table = wl.table_init(w)
    rng = np.random.default_rng(21)
    p = Pair(w, table, max_ids=n)
    try:
        for it in range(2):
            ids = (rng.zipf(1.1, size=n) % w.vocab).astype(np.int64)
            ids[: n // 8] = rng.integers(0, w.vocab, size=n // 8)
            g = rng.standard_normal((n, w.dim)).astype(np.float32)
            p.lookup(ids)
            p.update(ids, g)
            p.compare_state(values=True)
            p.compare_counters()
        p.flush_and_compare()
    finally:
        p.close()
    with pytest.raises(Exception):
        hc.HetCache(w.capacity, w.dim, w.s, w.policy, n + 1, w.optimizer, w.eps)


@pytest.mark.parametrize("dim", [24, 7, 320])
def test_pooled_with_bags_of_uneven_size_and_empty_bags(dim):
    """Bags of 0 to several hundred ids (the regular layouts have equal bags): pooled gather in bag
    order, bag gradients spread to the bag's ids.  Rows narrower than their row group (24 floats: six
    pieces for eight lanes), rows moved float by float (7), rows of more pieces than a wave has lanes (320)."""
    w = wl.WORKLOADS[5].scaled(vocab=20_000, dim=dim, batch=300, width=10, capacity=1_500, s=3)
    n = w.n
    table = wl.table_init(w)
    rng = np.random.default_rng(31)
    p = Pair(w, table)
    try:
        for it in range(6):
            cuts = np.sort(rng.integers(0, n + 1, size=w.batch - 1))
            cuts[rng.random(w.batch - 1) < 0.2] = cuts[0]                   # a fifth of the cuts coincide: empty bags
            offsets = np.concatenate([[0], np.sort(cuts), [n]]).astype(np.int64)
            p.offsets_np = offsets
            p.offsets = torch.from_numpy(offsets).to(p.dev)
            ids = (rng.zipf(1.2, size=n) % w.vocab).astype(np.int64)
            g = rng.standard_normal((w.batch, w.dim)).astype(np.float32)
            p.lookup(ids)
            p.update(ids, g)
            p.compare_state(values=True)
            p.compare_counters()
        p.flush_and_compare()
    finally:
        p.close()


@pytest.mark.parametrize("vocab,capacity", [(1, 1), (2, 1), (7, 3), (7, 100), (300, 1)])
def test_smallest_tables_and_caches(vocab, capacity):
    """A table of one row, a cache of one row, a cache larger than the table."""
    w = wl.WORKLOADS[1].scaled(vocab=vocab, dim=5, capacity=capacity, s=1, policy=wl.LRU, optimizer=wl.ADAGRAD, eps=1e-8)
    table = wl.table_init(w)
    rng = np.random.default_rng(41)
    p = Pair(w, table, max_ids=700)
    try:
        for n in (1, 2, 65, 700, 3):
            ids = rng.integers(0, vocab, size=n).astype(np.int64)
            g = rng.standard_normal((n, w.dim)).astype(np.float32)
            p.lookup(ids)
            p.update(ids, g)
            p.compare_state(values=True)
            p.compare_counters()
        p.flush_and_compare()
    finally:
        p.close()


def test_ids_of_25_bits_sort_in_four_passes():
    """A vocabulary of 20 M ids: the radix sort takes four passes (the configurations up to 4 M ids
    take three at most)."""
    w = wl.WORKLOADS[1].scaled(vocab=20_000_000, dim=4, batch=300, capacity=3_000, s=2, policy=wl.LFU,
                               optimizer=wl.ADAGRAD, eps=1e-8)
    st = run_workload(w, 10, state_every=2, values_every=5, prefetch="before")
    assert st["total"]["evicted"] > 0


@pytest.mark.parametrize("opt", [wl.SGD, wl.ADAGRAD])
def test_update_with_part_or_a_reordering_of_the_looked_up_ids(opt):
    """The update's ids need not be the lookup's list: a permutation of it, a part of it, its
    unique keys, each in a buffer of its own (the lookup's buffer stays alive, so that no other
    buffer can get its address and be taken for it)."""
    w = wl.WORKLOADS[1].scaled(vocab=5_000, capacity=700, s=3, policy=wl.LFU, optimizer=opt, eps=1e-8)
    table = wl.table_init(w)
    rng = np.random.default_rng(51)
    p = Pair(w, table, max_ids=3000)
    try:
        for t in range(24):
            n = int(rng.choice([17, 256, 1025, 3000]))
            ids = (rng.zipf(1.15, size=n) % w.vocab).astype(np.int64)
            keep = torch.from_numpy(ids).to(p.dev)
            p.lookup(ids, ids_dev=keep)
            uids = [rng.permutation(ids), ids[rng.random(n) < 0.5], np.unique(ids), ids[::-1].copy()][t % 4]
            if len(uids) == 0:
                uids = ids[:1]
            g = rng.standard_normal((len(uids), w.dim)).astype(np.float32)
            p.update(uids, g)
            p.compare_state(values=True)
            p.compare_counters()
        p.flush_and_compare()
    finally:
        p.close()


@pytest.mark.parametrize("dim", [16, 128])
@pytest.mark.parametrize("opt", [wl.SGD, wl.ADAGRAD])
def test_checkvalid_condition_two_after_another_writers_pushes(opt, dim):
    """CheckValid's second condition (c_g <= c_c + s, Section 3.1) never fails with one worker.
    Another worker's pushes are emulated by changing global rows and advancing their c_g behind
    the cache's back: cached rows without updates of their own are refetched and show the new
    values, rows with updates are pushed first.  (With rows of 128 floats the update pushes the
    rows it fetches early; a row the other worker has overwritten since must still be pushed at
    its eviction.)"""
    w = wl.WORKLOADS[1].scaled(dim=dim, capacity=600, s=2, policy=wl.LFU, optimizer=opt, eps=1e-8)
    T = 18
    table = wl.table_init(w)
    ids = wl.IdStream(w).batches(T)
    grads = wl.grad_pool(w)
    rng = np.random.default_rng(61)
    p = Pair(w, table)
    try:
        stale_seen = 0
        for t in range(T):
            p.lookup(ids[t])
            stale_seen += int((p.oracle.last_lookup()[1] == 1).sum())
            if t % 2 == 0:
                p.update(ids[t], grads[t % len(grads)])
            p.compare_state(values=True)
            p.compare_counters()
            cached = p.oracle.export_state()["key"]
            pick = rng.choice(cached, size=min(80, len(cached)), replace=False).astype(np.int64)
            bump = rng.integers(1, 7, size=len(pick)).astype(np.uint32)
            rows = rng.standard_normal((len(pick), w.dim)).astype(np.float32)
            p.oracle.Cg[pick] += bump
            p.oracle.W[pick] = rows
            pick_t = torch.from_numpy(pick).to(p.dev)
            p.Cg[pick_t] += torch.from_numpy(bump.astype(np.int32)).to(p.dev)
            p.W[pick_t] = torch.from_numpy(rows).to(p.dev)
        assert stale_seen > 0
        p.flush_and_compare()
    finally:
        p.close()


def test_per_kernel_timing_counts_the_launches_and_changes_nothing():
    """het_profile_begin / het_profile_end (what the benchmark's roofline figures are made of):
    one launch of each of the step's kernels per iteration, positive durations, same results."""
    w = wl.WORKLOADS[1].scaled(capacity=400, s=3, policy=wl.LFU, optimizer=wl.ADAGRAD, eps=1e-8)
    T = 6
    ids = wl.IdStream(w).batches(T)
    grads = wl.grad_pool(w)
    p = Pair(w, wl.table_init(w))
    try:
        dev = [torch.from_numpy(b).to(p.dev) for b in ids]
        for t in range(2):                       # fill the cache first: from here on every update trims
            p.lookup(ids[t], ids_dev=dev[t]); p.update(ids[t], grads[t], ids_dev=dev[t])
        p.cache.profile_begin()
        for t in range(2, T):
            p.lookup(ids[t], ids_dev=dev[t]); p.update(ids[t], grads[t], ids_dev=dev[t])
        prof = p.cache.profile_end()
        for name in ("probe_kernel", "fill_gather_kernel", "apply_kernel", "trim_evict_kernel"):
            ms, launches = prof[name]
            assert launches == T - 2 and ms > 0, (name, prof[name])
        p.compare_state(values=True)
        p.compare_counters()
        p.flush_and_compare()
    finally:
        p.close()


def test_on_a_stream_of_the_callers():
    """All work is enqueued on the stream given at configuration: here a stream of the test's own
    (default priority), on which the test's tensor operations run as well."""
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        w = wl.WORKLOADS[1].scaled(capacity=500, s=2, policy=wl.LFU, optimizer=wl.ADAGRAD, eps=1e-8)
        st = run_workload(w, 16, state_every=2, values_every=4, prefetch="before")
        assert st["total"]["evicted"] > 0
    stream.synchronize()


def test_two_caches_side_by_side():
    """Two caches of different shape in one process, their calls interleaved: nothing is shared."""
    wa = wl.WORKLOADS[1].scaled(capacity=300, s=1, policy=wl.LRU, optimizer=wl.SGD)
    wb = wl.WORKLOADS[1].scaled(vocab=3_000, dim=40, batch=50, capacity=900, s=4, policy=wl.LFU, optimizer=wl.ADAGRAD, eps=1e-8)
    ia, ib = wl.IdStream(wa).batches(12), wl.IdStream(wb).batches(12)
    ga, gb = wl.grad_pool(wa), wl.grad_pool(wb)
    pa, pb = Pair(wa, wl.table_init(wa)), Pair(wb, wl.table_init(wb))
    try:
        da = [torch.from_numpy(b).to(pa.dev) for b in ia]
        db = [torch.from_numpy(b).to(pb.dev) for b in ib]
        for t in range(12):
            if t + 1 < 12:
                pa.cache.prefetch(da[t + 1]); pb.cache.prefetch(db[t + 1])
            pa.lookup(ia[t], ids_dev=da[t])
            pb.lookup(ib[t], ids_dev=db[t])
            pb.update(ib[t], gb[t % len(gb)], ids_dev=db[t])
            pa.update(ia[t], ga[t % len(ga)], ids_dev=da[t])
            pa.compare_state(values=t % 3 == 0); pb.compare_state(values=t % 3 == 0)
            pa.compare_counters(); pb.compare_counters()
        pa.flush_and_compare(); pb.flush_and_compare()
    finally:
        pa.close(); pb.close()


def test_lookup_after_lookup_trims_first_and_empty_batch_is_a_no_op():
    w = wl.WORKLOADS[1].scaled(capacity=200, s=2)
    ids = wl.IdStream(w).batches(6)
    g = wl.grad_pool(w)
    p = Pair(w, wl.table_init(w))
    try:
        p.lookup(ids[0]); p.update(ids[0], g[0])
        p.lookup(ids[1])
        p.lookup(ids[2])                      # overflow of the first lookup is trimmed here
        assert np.array_equal(np.sort(p.cache.last_evicted()), np.sort(p.oracle.last_evicted()))
        p.compare_state(values=True); p.compare_counters()
        p.update(ids[2], g[2])
        empty = torch.zeros(0, dtype=torch.int64, device="cuda")
        p.cache.lookup(empty, torch.zeros(0, w.dim, device="cuda"))
        p.cache.update(empty, torch.zeros(0, w.dim, device="cuda"), 0.1)
        p.oracle.lookup(np.zeros(0, np.int64))
        p.compare_state(values=True); p.compare_counters()
        p.lookup(ids[3]); p.update(ids[3], g[3])
        p.flush_and_compare()
    finally:
        p.close()


def test_bad_ids_and_update_without_lookup_are_reported_not_fatal():
    w = wl.WORKLOADS[1].scaled(capacity=100)
    p = Pair(w, wl.table_init(w), max_ids=64)
    try:
        ids = np.array([5, -1, 7, w.vocab, 5, 2**40, 9], dtype=np.int64)
        out = p.lookup(ids, expect_rc=1)
        assert torch.all(out[[1, 3, 5]] == 0)
        st = p.cache.stats()
        assert st["error_bits"] & 1 and st["last"]["unique"] == 3
        assert p.cache.flush() == hc.HET_ERANGE
        p.oracle.flush()
        p.cache.clear_error(); p.oracle.clear_error()
        g = np.ones((len(ids), w.dim), np.float32)
        p.update(ids, g)
        assert p.cache.stats()["error_bits"] & 1
        p.cache.clear_error(); p.oracle.clear_error()
        # an id that was never looked up: skipped and flagged
        ids2 = np.array([5, 11], dtype=np.int64)
        p.cache.update(torch.from_numpy(ids2).cuda(), torch.ones(2, w.dim, device="cuda"), w.lr)
        p.oracle.update(ids2, np.ones((2, w.dim)), w.lr)
        assert p.cache.stats()["error_bits"] & 2
        assert p.cache.flush() == hc.HET_ESTATE
        p.oracle.flush()
        p.cache.clear_error(); p.oracle.clear_error()
        p.flush_and_compare()
        # host-visible argument errors change nothing
        too_many = torch.zeros(65, dtype=torch.int64, device="cuda")
        with pytest.raises(hc.HetError):
            p.cache.lookup(too_many, torch.zeros(65, w.dim, device="cuda"))
        p.compare_counters()
    finally:
        p.close()


def test_everything_fits_no_eviction():
    """Capacity >= vocabulary: misses are first touches only and nothing is ever evicted."""
    w = wl.WORKLOADS[1].scaled(vocab=2000, capacity=2000, s=1)
    st = run_workload(w, 25, state_every=5, values_every=5)
    assert st["total"]["evicted"] == 0


def test_an_announced_buffer_that_changed_is_flagged_at_the_lookup():
    """An announcement promises that the ids stay as they are until their lookup; if they do not,
    the order sorted ahead no longer fits them and the lookup says so."""
    w = wl.WORKLOADS[1].scaled(capacity=400, s=3)
    ids_np = wl.IdStream(w).batches(4)
    g_np = wl.grad_pool(w)
    p = Pair(w, wl.table_init(w))
    try:
        dev = [torch.from_numpy(b).cuda() for b in ids_np]
        g = torch.from_numpy(g_np[0]).cuda()
        out = torch.empty(w.n, w.dim, device="cuda")
        p.cache.prefetch(dev[1]); p.cache.prefetch(dev[2])
        p.cache.lookup(dev[0], out); p.cache.update(dev[0], g, w.lr)       # these carry the announced sorts
        p.cache.lookup(dev[1], out); p.cache.update(dev[1], g, w.lr)       # unchanged: fine
        assert p.cache.stats()["error_bits"] == 0
        dev[2][:50] = (dev[2][:50] + 1) % w.vocab                          # changed after it was announced (and sorted)
        p.cache.lookup(dev[2], out)
        assert p.cache.stats()["error_bits"] & 2
    finally:
        p.close()


def test_update_reuses_the_lookup_order_only_for_the_same_ids():
    """An update handed the lookup's own id buffer reuses its sorted order and checks every id
    against it on the device; a buffer whose contents changed in between is flagged, not
    silently misapplied; a different buffer with the same ids is sorted afresh."""
    w = wl.WORKLOADS[1].scaled(capacity=400, s=3)
    ids_np = wl.IdStream(w).batches(3)
    g_np = wl.grad_pool(w)
    p = Pair(w, wl.table_init(w))
    try:
        ids = torch.from_numpy(ids_np[0]).cuda()
        out = torch.empty(w.n, w.dim, device="cuda")
        g = torch.from_numpy(g_np[0]).cuda()
        # same buffer: fast path
        p.cache.lookup(ids, out); p.oracle.lookup(ids_np[0])
        p.cache.update(ids, g, w.lr); p.oracle.update(ids_np[0], g_np[0], w.lr)
        p.compare_state(values=True); p.compare_counters()
        # a copy of the buffer: sorted again, same result
        ids1 = torch.from_numpy(ids_np[1]).cuda()
        p.cache.lookup(ids1, out); p.oracle.lookup(ids_np[1])
        p.cache.update(ids1.clone(), g, w.lr); p.oracle.update(ids_np[1], g_np[0], w.lr)
        p.compare_state(values=True); p.compare_counters()
        # same buffer, contents overwritten after the lookup: flagged
        ids2 = torch.from_numpy(ids_np[2]).cuda()
        p.cache.lookup(ids2, out)
        ids2[:100] = (ids2[:100] + 1) % w.vocab
        p.cache.update(ids2, g, w.lr)
        assert p.cache.stats()["error_bits"] & 2
    finally:
        p.close()


@pytest.mark.parametrize("dim", [1, 4, 10, 16, 64, 256])
def test_rowwise_adagrad_row_widths(dim):
    """HET_OPT_ADAGRAD_ROWWISE: one accumulator per row (a += mean of the squared gradient), the row
    group adding up the squares; rows narrower than their row group (dim 10: six idle lanes)."""
    w = wl.WORKLOADS[1].scaled(dim=dim, optimizer=wl.ADAGRAD_ROWWISE, eps=1e-8, policy=wl.LFU, s=2)
    st = run_workload(w, 14, state_every=2, values_every=2, prefetch="before")
    assert st["total"]["stale_dirty"] > 0 and st["total"]["evicted_dirty"] > 0


def test_rowwise_adagrad_config2_full_size_and_long_runs():
    w = wl.WORKLOADS[2].scaled(optimizer=wl.ADAGRAD_ROWWISE, s=3)
    st = run_workload(w, 10, state_every=5, values_every=5, prefetch="before")
    assert st["total"]["stale_dirty"] > 0
    # a few keys hold most of the batch: segments summed by the whole workgroup, and runs that cross tiles
    w = wl.WORKLOADS[1].scaled(dim=64, capacity=400, s=2, optimizer=wl.ADAGRAD_ROWWISE, eps=1e-8, policy=wl.LFU)
    rng = np.random.default_rng(13)
    n = 3000
    p = Pair(w, wl.table_init(w), max_ids=n)
    try:
        hot = rng.permutation(w.vocab)[:3]
        for it in range(3):
            u = rng.random(n)
            ids = rng.integers(0, w.vocab, size=n)
            ids[u < 0.85] = hot[2]; ids[u < 0.65] = hot[1]; ids[u < 0.45] = hot[0]
            ids = ids.astype(np.int64)
            g = rng.standard_normal((n, w.dim)).astype(np.float32)
            p.lookup(ids); p.update(ids, g)
            p.compare_state(values=True); p.compare_counters()
        p.flush_and_compare()
    finally:
        p.close()


def test_rowwise_adagrad_pooled_and_without_a_cache():
    w = wl.WORKLOADS[5].scaled(vocab=50_000, dim=64, batch=128, capacity=3_000, s=3, optimizer=wl.ADAGRAD_ROWWISE)
    st = run_workload(w, 12, state_every=3, values_every=3)
    assert st["total"]["evicted_dirty"] > 0
    # HET_POLICY_NONE: the step goes straight to the global table and its per-row accumulators
    from oracle.het_oracle import Oracle
    w = wl.WORKLOADS[1].scaled(optimizer=wl.ADAGRAD_ROWWISE, eps=1e-8)
    table, ids_np, g_np = wl.table_init(w), wl.IdStream(w).batches(8), wl.grad_pool(w)
    oracle = Oracle(w.capacity, w.dim, w.s, w.policy, w.n, w.optimizer, w.eps, table)
    cache = hc.HetCache(1, w.dim, 0, hc.POLICY_NONE, w.n, w.optimizer, w.eps)
    dev = torch.device("cuda:0")
    W = torch.from_numpy(table).to(dev); A = torch.zeros(w.vocab, device=dev); Cg = torch.zeros(w.vocab, dtype=torch.int32, device=dev)
    cache.attach_backing(W, A, Cg)
    try:
        out = torch.empty(w.n, w.dim, device=dev)
        for t in range(8):
            d = torch.from_numpy(ids_np[t]).to(dev)
            cache.lookup(d, out)
            want, _ = oracle.lookup(ids_np[t])
            close(out.cpu().numpy(), want, "lookup output")
            cache.update(d, torch.from_numpy(g_np[t]).to(dev), w.lr)
            oracle.update(ids_np[t], g_np[t], w.lr)
        oracle.flush()
        close(W.cpu().numpy(), oracle.W, "global table")
        close(A.cpu().numpy(), oracle.A[:, 0], "global accumulators")
    finally:
        cache.close(); oracle.close()


def test_rowwise_adagrad_is_refused_where_it_is_not_built():
    with pytest.raises(hc.HetError):                       # rows of more than one piece per lane
        hc.HetCache(100, 512, 1, hc.POLICY_LFU, 64, hc.OPT_ADAGRAD_ROWWISE, 1e-8)
    with pytest.raises(hc.HetError):                       # several workers
        hc.HetCache(100, 16, 1, hc.POLICY_LFU, 64, hc.OPT_ADAGRAD_ROWWISE, 1e-8, many_writers=True)
    c = hc.HetCache(100, 16, 1, hc.POLICY_LFU, 64, hc.OPT_ADAGRAD_ROWWISE, 1e-8)
    try:
        with pytest.raises(hc.HetError):                   # table in host memory
            c.attach_backing(torch.zeros(50, 16).pin_memory(), torch.zeros(50).pin_memory(),
                             torch.zeros(50, dtype=torch.int32).pin_memory(), hc.BACKING_PINNED_HOST)
    finally:
        c.close()


@pytest.mark.gpu
def test_reference_pattern_kernels_do_what_the_header_says():
    """het_profile_rows' plain kernels (reference points for the roofline, not part of the path):
    the copy copies, the gather gathers, the update changes exactly the rows it is given."""
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(5)
    for dim in (4, 64, 128, 256, 520):
        V, n = 3000, 1237
        src = torch.randn(V, dim, device=dev)
        out = torch.zeros(n, dim, device=dev)
        assert hc.profile_rows(hc.PATTERN_COPY, out, src=src, n=n, reps=1) > 0
        assert torch.equal(out, src[:n])
        idx = torch.from_numpy(rng.integers(0, V, n).astype(np.int32)).to(dev)
        hc.profile_rows(hc.PATTERN_GATHER, out, src=src, idx=idx, reps=1)
        assert torch.equal(out, src[idx.long()])
        # the update: a += 1 + sum of the row's gradients, x -= a, three launches in all (two untimed)
        rows = torch.from_numpy(rng.choice(V, n, replace=False).astype(np.int32)).to(dev)
        for per in (0, 2, 3):
            x = torch.zeros(V, dim, device=dev); a = torch.zeros(V, dim, device=dev)
            g = torch.randn(n * 3, dim, device=dev)
            gidx = torch.from_numpy(rng.permutation(n * 3)[: n * per].astype(np.int32)).to(dev) if per else None
            hc.profile_rows(hc.PATTERN_UPDATE, x, a=a, src=g if per else None, idx=rows, gidx=gidx, per=per, reps=1)
            d = torch.ones(n, dim, device=dev, dtype=torch.float64)
            if per:
                d = d + g[gidx.long()].double().view(n, per, dim).sum(1)
            want_a = torch.zeros(V, dim, device=dev, dtype=torch.float64); want_a[rows.long()] = 3 * d
            want_x = torch.zeros(V, dim, device=dev, dtype=torch.float64); want_x[rows.long()] = -6 * d
            assert torch.allclose(a.double(), want_a, rtol=1e-5, atol=1e-5)
            assert torch.allclose(x.double(), want_x, rtol=1e-5, atol=1e-5)
    with pytest.raises(RuntimeError):
        hc.profile_rows(hc.PATTERN_GATHER, torch.zeros(4, 12, device=dev), src=torch.zeros(4, 12, device=dev),
                        idx=torch.zeros(4, dtype=torch.int32, device=dev))        # row groups of three lanes


@pytest.mark.gpu
def test_time_stamps_inside_the_kernels_change_nothing():
    """het_profile_trace: with the stamps on, a step gives the same cache as without, every
    workgroup of the two kernels leaves a record with start <= end, and switching them off stops them."""
    dev = torch.device("cuda:0")
    w = wl.WORKLOADS[1].scaled(capacity=600, s=2, optimizer=wl.ADAGRAD, eps=1e-8)
    table = wl.table_init(w)
    ids = wl.IdStream(w).batches(6)
    grads = wl.grad_pool(w)
    p = Pair(w, table)
    kernels = ("apply_kernel", "fill_gather_kernel")
    try:
        rec = {k: torch.zeros(4096, hc.TRACE_WORDS, dtype=torch.int64, device=dev) for k in kernels}
        seen = {}
        for t in range(6):
            if t == 3:
                for k in kernels:
                    p.cache.profile_trace(rec[k], k)
            if t == 4:
                for k in kernels:
                    p.cache.profile_trace(None, k)
                    seen[k] = rec[k].cpu().numpy().copy()
                    rec[k].zero_()
            p.lookup(ids[t])
            p.update(ids[t], grads[t % len(grads)])
            p.compare_state(values=True)
        for k in kernels:
            used = seen[k][:, 6] > 0
            assert used.sum() >= 1 and (seen[k][used, 6] <= 6).all()
            assert (seen[k][used, 5] >= seen[k][used, 0]).all() and (seen[k][used, 0] > 0).all()
            assert not rec[k].cpu().numpy().any()
        p.flush_and_compare()
    finally:
        p.close()


@pytest.mark.gpu
@pytest.mark.parametrize("dim", [16, 128])
@pytest.mark.parametrize("opt", [wl.SGD, wl.ADAGRAD])
def test_rows_a_lookup_leaves_to_the_update_are_fetched_by_whoever_needs_them_first(opt, dim):
    """With the table in HBM a lookup leaves the fetch of its missed keys' rows to the update that
    reuses its order.  Whatever comes instead (a flush, an export of the rows, another lookup, an
    update with other ids or with the same ids in another buffer) must find the rows in their slots."""
    w = wl.WORKLOADS[1].scaled(dim=dim, capacity=500, s=2, optimizer=opt, eps=1e-8, policy=wl.LFU)     # (dim 128: with the early push)
    table = wl.table_init(w)
    ids = wl.IdStream(w).batches(12)
    grads = wl.grad_pool(w)
    p = Pair(w, table)
    try:
        g = lambda t: grads[t % len(grads)]
        p.lookup(ids[0]); p.update(ids[0], g(0))                       # the ordinary case: the update fetches
        p.compare_state(values=True)
        p.lookup(ids[1]); p.compare_state(values=True)                 # an export of the rows comes first
        p.update(ids[1], g(1)); p.compare_state(values=True)
        p.lookup(ids[2]); p.flush_and_compare()                        # a flush comes first
        p.update(ids[2], g(2)); p.compare_state(values=True)
        p.lookup(ids[3]); p.lookup(ids[4])                             # another lookup comes first
        p.update(ids[4], g(4)); p.compare_state(values=True)
        p.lookup(ids[5])                                               # an update of a part of the ids comes first
        half = len(ids[5]) // 2
        p.update(ids[5][:half].copy(), g(5)[:half].copy()); p.compare_state(values=True)
        a = torch.from_numpy(ids[7]).to(p.dev); b = a.clone()          # the same ids in another buffer: sorted afresh
        p.lookup(ids[7], ids_dev=a)
        p.update(ids[7], g(7), ids_dev=b); p.compare_state(values=True)
        # and the ordinary case again, free-running
        for t in range(8, 12):
            dev_ids = torch.from_numpy(ids[t]).to(p.dev)
            p.lookup(ids[t], ids_dev=dev_ids)
            p.update(ids[t], g(t), ids_dev=dev_ids)
        p.compare_state(values=True)
        p.compare_counters()
        p.flush_and_compare()
    finally:
        p.close()
