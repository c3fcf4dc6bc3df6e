"""Pins of the CPU oracle against things other than itself: a brute-force twin on tiny inputs,
a dense uncached trainer, closed forms, a library optimizer, and invariants of the protocol
(Section 3.1, Algorithms 2 and 3 of the paper)."""
import itertools

import numpy as np
import pytest
import torch

from oracle import brute
from oracle.het_oracle import ERR_RANGE, HIT, MISS, S_INF, STALE, Oracle

CLS = {0: "hit", 1: "stale", 2: "miss"}


def skewed_ids(rng, vocab, n, alpha=1.0):
    """n IDs with Zipf(alpha) popularity; the popular IDs are scattered by a fixed permutation."""
    p = np.arange(1, vocab + 1, dtype=np.float64) ** (-alpha)
    p /= p.sum()
    perm = np.random.default_rng(vocab).permutation(vocab)
    return perm[rng.choice(vocab, size=n, p=p)].astype(np.int64)


def stream(seed, vocab, n, iters, dim, alpha=1.0):
    rng = np.random.default_rng(seed)
    ids = [skewed_ids(rng, vocab, int(rng.integers(1, n + 1)), alpha) for _ in range(iters)]
    grads = [rng.standard_normal((len(i), dim)) for i in ids]
    table = rng.standard_normal((vocab, dim)) * 0.01
    return ids, grads, table


# ---------------------------------------------------------------- brute force on tiny inputs
@pytest.mark.parametrize("policy,opt,s", list(itertools.product((0, 1), (0, 1), (0, 1, 3, S_INF))))
def test_matches_brute_force_twin(policy, opt, s):
    V, C, D, N = 50, 5, 3, 12
    ids, grads, table = stream(7 + policy + 2 * opt, V, N, 120, D)
    o = Oracle(C, D, s, policy, N, opt, 1e-8, table)
    b = brute.BruteCache(C, D, s, policy, N, opt, 1e-8, table)
    for t, (i, g) in enumerate(zip(ids, grads)):
        out, rc = o.lookup(i)
        assert rc == 0
        bout = b.read(i.tolist())
        assert np.array_equal(out, np.asarray(bout)), t
        keys, cls, slots = o.last_lookup()
        assert {k: CLS[c] for k, c in zip(keys.tolist(), cls.tolist())} == b.classes
        assert all(b.find(k).slot == sl for k, sl in zip(keys.tolist(), slots.tolist()))
        if t % 7 == 6:                      # a Read that follows a Read: trims first
            out2, _ = o.lookup(ids[t - 1])
            bout2 = b.read(ids[t - 1].tolist())
            assert np.array_equal(out2, np.asarray(bout2))
            assert sorted(o.last_evicted().tolist()) == sorted(b.evicted)
            out, _ = o.lookup(i)
            b.read(i.tolist())
        assert o.update(i, g, 0.05) == 0
        b.write(i.tolist(), g.tolist(), 0.05)
        assert o.last_evicted().tolist() == b.evicted
        st = o.export_state()
        got = list(zip(*(st[c].tolist() for c in ("key", "slot", "cs", "cc", "last_use", "freq"))))
        assert got == b.state()
        assert o.Cg.tolist() == b.c_g
        assert np.array_equal(o.W, np.asarray(b.W))
    o.flush()
    b.flush()
    _, tot = o.stats()
    assert tot["evicted_dirty"] + tot["stale_dirty"] + tot["flushed"] == b.pushes
    assert np.array_equal(o.W, np.asarray(b.W)) and o.Cg.tolist() == b.c_g
    if opt:
        assert np.array_equal(o.A, np.asarray(b.A))


# ---------------------------------------------------------------- dense uncached trainer
def dense_step(W, A, ids, grads, lr, opt, eps):
    """Plain embedding training on the full table: per unique key, the summed gradient (in
    order of position) applied once."""
    G = {}
    for i, k in enumerate(ids.tolist()):
        G[k] = G.get(k, np.zeros(W.shape[1], W.dtype)) + grads[i].astype(W.dtype)
    for k, g in G.items():
        if opt == 0:
            W[k] = W[k] - W.dtype.type(lr) * g
        else:
            A[k] = A[k] + g * g
            W[k] = W[k] - (W.dtype.type(lr) * g) / (np.sqrt(A[k]) + W.dtype.type(eps))


@pytest.mark.parametrize("real", ["f64", "f32"])
@pytest.mark.parametrize("policy,opt,s,C", [(0, 0, 0, 8), (1, 1, 2, 8), (0, 1, 10, 40),
                                            (1, 0, S_INF, 3), (1, 1, 0, 200)])
def test_cache_is_transparent_to_training(real, policy, opt, s, C):
    """Every Read returns exactly what uncached training would hold for that key (the s = 0
    case is the paper's fully consistent setting; with one worker it holds for every s), and
    after flush the global table equals the uncached one everywhere."""
    V, D, N = 120, 4, 30
    dt = np.float64 if real == "f64" else np.float32
    ids, grads, table = stream(11 + C, V, N, 150, D, alpha=1.1)
    table = table.astype(np.float32)
    grads = [g.astype(np.float32) for g in grads]
    o = Oracle(C, D, s, policy, N, opt, 1e-8, table, real=real)
    W, A = table.astype(dt), np.zeros((V, D), dt)
    touched = np.zeros(V, np.int64)
    for i, g in zip(ids, grads):
        out, _ = o.lookup(i)
        assert np.array_equal(out, W[i])
        o.update(i, g, 0.05)
        dense_step(W, A, i, g, 0.05, opt, 1e-8)
        touched[np.unique(i)] += 1
        assert o.size <= C
    o.flush()
    assert np.array_equal(o.W, W)
    if opt:
        assert np.array_equal(o.A, A)
    # c_g counts the updates of the row (Section 3.1): one per iteration whose key set has it
    assert np.array_equal(o.Cg.astype(np.int64), touched)
    st = o.export_state()
    assert np.array_equal(st["cs"], st["cc"])
    assert np.array_equal(st["cc"].astype(np.int64), touched[st["key"]])


def test_sgd_closed_form():
    """x_k(T) = x_k(0) - lr * sum of all gradients of k."""
    V, D, N = 80, 5, 25
    ids, grads, table = stream(3, V, N, 100, D)
    o = Oracle(10, D, 2, 0, N, 0, 0.0, table)
    total = np.zeros((V, D))
    for i, g in zip(ids, grads):
        o.lookup(i)
        o.update(i, g, 0.1)
        np.add.at(total, i, g)
    o.flush()
    np.testing.assert_allclose(o.W, table - 0.1 * total, rtol=1e-12, atol=1e-13)


def test_adagrad_matches_library_optimizer():
    """The per-row Adagrad step against torch.optim.Adagrad fed the coalesced dense gradient."""
    V, D, N = 60, 4, 20
    ids, grads, table = stream(5, V, N, 80, D)
    eps, lr = 1e-8, 0.05
    o = Oracle(7, D, 3, 1, N, 1, eps, table)
    w = torch.tensor(table, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adagrad([w], lr=lr, eps=eps, lr_decay=0, weight_decay=0,
                              initial_accumulator_value=0)
    for i, g in zip(ids, grads):
        o.lookup(i)
        o.update(i, g, lr)
        dense = torch.zeros(V, D, dtype=torch.float64)
        dense.index_add_(0, torch.tensor(i), torch.tensor(g))
        w.grad = dense
        opt.step()
    o.flush()
    np.testing.assert_allclose(o.W, w.detach().numpy(), rtol=1e-12, atol=1e-14)


# ---------------------------------------------------------------- clocks and staleness
@pytest.mark.parametrize("s", [0, 1, 4, 25])
def test_clock_drift_is_bounded(s):
    """Condition (1) of CheckValid: after a Read every key of the batch has c_c - c_s <= s;
    after a Write every cached row has drift <= s + 1; the global clock never passes c_s."""
    V, D, N = 100, 2, 30
    ids, grads, table = stream(21, V, N, 200, D, alpha=1.2)
    o = Oracle(20, D, s, 1, N, 0, 0.0, table)
    for i, g in zip(ids, grads):
        o.lookup(i)
        st = o.export_state()
        drift = st["cc"].astype(np.int64) - st["cs"].astype(np.int64)
        in_batch = np.isin(st["key"], i)
        assert drift.min() >= 0 and drift[in_batch].max() <= s
        assert np.all(o.Cg[st["key"]] <= st["cs"])
        assert o.size <= 20 + len(np.unique(i))
        o.update(i, g, 0.1)
        st = o.export_state()
        drift = st["cc"].astype(np.int64) - st["cs"].astype(np.int64)
        assert drift.max() <= s + 1
        assert o.size <= 20


@pytest.mark.parametrize("s", [0, 1, 3, 10, S_INF])
def test_refresh_count_closed_form_when_nothing_is_evicted(s):
    """With capacity >= vocabulary nothing is evicted: misses are first touches, and a key
    updated u times has been refreshed floor((u-1)/(s+1)) times once u-th update's successor
    Read has happened.  Counted here right after each key's Reads."""
    V, D, N = 40, 2, 15
    ids, grads, table = stream(33, V, N, 150, D)
    o = Oracle(V, D, s, 0, N, 0, 0.0, table)
    reads = np.zeros(V, np.int64)
    seen = set()
    for i, g in zip(ids, grads):
        o.lookup(i)
        keys, cls, _ = o.last_lookup()
        for k, c in zip(keys.tolist(), cls.tolist()):
            # before this Read the key had reads[k] updates since its first fetch
            if k not in seen:
                assert c == MISS
            elif s == S_INF:
                assert c == HIT
            else:
                assert (c == STALE) == (reads[k] % (s + 1) == 0), (k, reads[k], c)
            seen.add(k)
            reads[k] += 1
        o.update(i, g, 0.1)
        assert len(o.last_evicted()) == 0
    last, total = o.stats()
    assert total["miss"] == len(seen) and total["evicted"] == 0
    if s != S_INF:
        assert total["stale"] == sum(int((u - 1) // (s + 1)) for u in reads[reads > 0])
        assert total["stale_dirty"] == total["stale"]
    else:
        assert total["stale"] == 0


def test_residency_does_not_depend_on_s():
    """A refresh happens in place, so which rows are cached, where, and which are evicted is
    the same for every staleness bound."""
    V, D, N = 90, 2, 25
    ids, grads, table = stream(44, V, N, 120, D)
    runs = [Oracle(12, D, s, 1, N, 0, 0.0, table) for s in (0, 2, S_INF)]
    for i, g in zip(ids, grads):
        snaps = []
        for o in runs:
            o.lookup(i)
            o.update(i, g, 0.1)
            st = o.export_state()
            snaps.append((st["key"].tolist(), st["slot"].tolist(), st["last_use"].tolist(),
                          st["freq"].tolist(), o.last_evicted().tolist()))
        assert snaps[0] == snaps[1] == snaps[2]


def test_condition_two_of_checkvalid():
    """A global clock more than s ahead of the local clock makes the row invalid (condition (2)
    of CheckValid).  Another worker's pushes are emulated by raising c_g and the global row."""
    table = np.zeros((4, 1))
    o = Oracle(4, 1, 2, 0, 4, 0, 0.0, table)
    o.lookup([1])
    o.update([1], [[1.0]], 1.0)            # row = -1, c_s = 0, c_c = 1
    o.Cg[1] = 3                            # c_g <= c_c + s  (3 <= 3): still valid
    o.lookup([1])
    assert o.last_lookup()[1].tolist() == [HIT]
    o.Cg[1] = 4                            # 4 > 1 + 2: invalid
    o.W[1] = 7.0
    out, _ = o.lookup([1])
    assert o.last_lookup()[1].tolist() == [STALE]
    # Evict pushed the local row and c_g = max(4, 1); Fetch read it back with c_s = c_c = 4
    assert out[0, 0] == -1.0 and o.W[1, 0] == -1.0 and o.Cg[1] == 4
    st = o.export_state()
    assert st["cs"].tolist() == [4] and st["cc"].tolist() == [4]


# ---------------------------------------------------------------- policies
def test_lfu_misses_no_more_than_lru_and_bigger_cache_misses_less():
    """Section 5.2 reports LFU below LRU in miss rate and the miss rate falling as the cache
    grows; on a skewed stream the oracle must show the same ordering."""
    V, D, N = 2000, 1, 200
    ids, grads, table = stream(55, V, N, 150, D, alpha=1.1)
    miss = {}
    for policy in (0, 1):
        for frac in (0.03, 0.05, 0.10, 0.15):
            o = Oracle(int(V * frac), D, 100, policy, N, 0, 0.0, table)
            for i, g in zip(ids, grads):
                o.lookup(i)
                o.update(i, g, 0.1)
            _, tot = o.stats()
            miss[policy, frac] = tot["miss"] / tot["U"]
    for frac in (0.03, 0.05, 0.10, 0.15):
        assert miss[1, frac] <= miss[0, frac]
    for policy in (0, 1):
        r = [miss[policy, f] for f in (0.03, 0.05, 0.10, 0.15)]
        assert r[0] > r[1] > r[2] > r[3]


def test_lru_evicts_exactly_the_least_recent():
    """Capacity 3, unit batches 0,1,2,0,3: LRU evicts 1 (0 was used again); LFU evicts 1 too
    (freq 1, older than 2); after a further 4: LRU evicts 2, LFU evicts 2."""
    for policy in (0, 1):
        o = Oracle(3, 1, 100, policy, 1, 0, 0.0, np.zeros((6, 1)))
        ev = []
        for k in (0, 1, 2, 0, 3, 4):
            o.lookup([k])
            o.update([k], [[0.0]], 0.0)
            ev += o.last_evicted().tolist()
        assert ev == [1, 2]
    # LRU and LFU part ways once frequency outweighs recency: 0,0,0,1,2,3 with capacity 3
    got = {}
    for policy in (0, 1):
        o = Oracle(3, 1, 100, policy, 1, 0, 0.0, np.zeros((6, 1)))
        ev = []
        for k in (0, 0, 0, 1, 2, 3, 4):
            o.lookup([k])
            o.update([k], [[0.0]], 0.0)
            ev += o.last_evicted().tolist()
        got[policy] = ev
    assert got[0] == [0, 1] and got[1] == [1, 2]


# ---------------------------------------------------------------- pooled form, edges, errors
def test_pooled_read_and_write_reduce_to_the_plain_ones():
    """A pooled Read is the bag-wise sum of a plain Read; a pooled Write is a plain Write whose
    per-position gradient is its bag's gradient."""
    V, D = 70, 3
    rng = np.random.default_rng(9)
    table = rng.standard_normal((V, D)) * 0.01
    a = Oracle(9, D, 2, 1, 64, 1, 1e-8, table)
    b = Oracle(9, D, 2, 1, 64, 1, 1e-8, table)
    for _ in range(60):
        lens = rng.integers(0, 6, size=8)
        offs = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
        ids = skewed_ids(rng, V, int(offs[-1]))
        if ids.size == 0:
            continue
        bag_g = rng.standard_normal((8, D))
        pooled, _ = a.lookup_pooled(ids, offs)
        plain, _ = b.lookup(ids)
        expect = np.zeros((8, D))
        for bag in range(8):
            for r in plain[offs[bag]:offs[bag + 1]]:
                expect[bag] = expect[bag] + r
        assert np.array_equal(pooled, expect)
        a.update_pooled(ids, offs, bag_g, 0.05)
        b.update(ids, np.repeat(bag_g, lens, axis=0), 0.05)
        sa, sb = a.export_state(), b.export_state()
        assert all(np.array_equal(sa[c], sb[c]) for c in sa)
        assert np.array_equal(a.export_rows()[0], b.export_rows()[0])
    a.flush(); b.flush()
    assert np.array_equal(a.W, b.W) and np.array_equal(a.A, b.A)


def test_empty_batch_is_a_no_op_and_bad_ids_are_reported():
    table = np.arange(10, dtype=np.float64).reshape(5, 2)
    o = Oracle(2, 2, 1, 0, 8, 0, 0.0, table)
    out, rc = o.lookup(np.zeros(0, np.int64))
    assert rc == 0 and o.iteration == 0 and o.size == 0
    assert o.update(np.zeros(0, np.int64), np.zeros((0, 2)), 0.1) == 0
    out, rc = o.lookup([1, -1, 5, 4])
    assert rc & ERR_RANGE
    assert np.array_equal(out, [[2, 3], [0, 0], [0, 0], [8, 9]])
    assert o.last_lookup()[0].tolist() == [1, 4]
    o.clear_error()
    rc = o.update([1, 7, 4], [[1, 1], [5, 5], [2, 2]], 1.0)
    assert rc & ERR_RANGE
    o.flush()
    assert np.array_equal(o.W, [[0, 1], [1, 2], [4, 5], [6, 7], [6, 7]])
    # more ids than the configured maximum is refused before any state change
    it = o.iteration
    _, rc = o.lookup(np.zeros(9, np.int64))
    assert rc != 0 and o.iteration == it


def test_rows_that_accumulated_nothing_are_not_pushed():
    """Evict pushes accumulated updates (Section 3.1): a row that was only read has none."""
    V, D, N = 60, 2, 20
    ids, _, table = stream(66, V, N, 80, D)
    o = Oracle(6, D, 0, 0, N, 0, 0.0, table)
    for i in ids:
        o.lookup(i)
    o.flush()
    _, tot = o.stats()
    assert tot["evicted"] > 0
    assert tot["evicted_dirty"] == 0 and tot["stale_dirty"] == 0 and tot["flushed"] == 0
    assert tot["stale"] == 0 and not o.Cg.any()


def test_write_of_a_key_that_was_never_read_is_skipped_and_flagged():
    o = Oracle(2, 1, 1, 0, 4, 0, 0.0, np.zeros((5, 1)))
    o.lookup([1])
    rc = o.update([1, 3], [[1.0], [1.0]], 1.0)
    assert rc & 2
    o.flush()
    assert o.W[:, 0].tolist() == [0, -1, 0, 0, 0]


# ---------------------------------------------------------------- light-weight LFU (Section 4.3)
@pytest.mark.parametrize("opt,s,cap", [(0, 0, 1), (1, 2, 3), (0, S_INF, 6)])
def test_light_lfu_matches_brute_force_twin(opt, s, cap):
    """LFU whose use counter stops at a cap (a row used that often is left alone by Reads), against
    the list-based twin: classes, slots, evicted ids, every cached row's clocks and policy fields."""
    V, C, D, N = 50, 6, 2, 12
    ids, grads, table = stream(23 + cap, V, N, 150, D, alpha=1.2)
    o = Oracle(C, D, s, 3, N, opt, 1e-8, table, lfu_cap=cap)
    b = brute.BruteCache(C, D, s, 3, N, opt, 1e-8, table, lfu_cap=cap)
    capped = 0
    for i, g in zip(ids, grads):
        out, _ = o.lookup(i)
        assert np.array_equal(out, np.asarray(b.read(i.tolist())))
        keys, cls, slots = o.last_lookup()
        assert {k: CLS[c] for k, c in zip(keys.tolist(), cls.tolist())} == b.classes
        o.update(i, g, 0.05)
        b.write(i.tolist(), g.tolist(), 0.05)
        assert o.last_evicted().tolist() == b.evicted
        st = o.export_state()
        assert list(zip(*(st[c].tolist() for c in ("key", "slot", "cs", "cc", "last_use", "freq")))) == b.state()
        assert st["freq"].max() <= cap
        capped += int((st["freq"] == cap).sum())
    assert capped > 0
    o.flush(); b.flush()
    assert np.array_equal(o.W, np.asarray(b.W))


def test_light_lfu_with_a_cap_never_reached_is_lfu():
    V, C, D, N = 200, 20, 2, 40
    ids, grads, table = stream(29, V, N, 120, D, alpha=1.1)
    exact = Oracle(C, D, 3, 1, N, 0, 0.0, table)
    light = Oracle(C, D, 3, 3, N, 0, 0.0, table, lfu_cap=10**9)
    for i, g in zip(ids, grads):
        a, _ = exact.lookup(i)
        b, _ = light.lookup(i)
        assert np.array_equal(a, b)
        exact.update(i, g, 0.1); light.update(i, g, 0.1)
        assert exact.last_evicted().tolist() == light.last_evicted().tolist()
    se, sl = exact.export_state(), light.export_state()
    assert all(np.array_equal(se[c], sl[c]) for c in se)


def test_light_lfu_misses_about_as_often_as_lfu():
    """Section 4.3: under the same workload the light-weight version has a similar miss rate."""
    V, D, N, T = 3000, 2, 200, 300
    ids, grads, table = stream(37, V, N, T, D, alpha=1.05)
    miss = {}
    for name, policy, cap in (("lru", 0, None), ("lfu", 1, None), ("light", 3, 8)):
        o = Oracle(300, D, 5, policy, N, 0, 0.0, table, lfu_cap=cap)
        for t, (i, g) in enumerate(zip(ids, grads)):
            o.lookup(i)
            o.update(i, g, 0.1)
            if t == T // 3:
                warm = o.stats()[1]["miss"]
        miss[name] = o.stats()[1]["miss"] - warm
    assert abs(miss["light"] - miss["lfu"]) <= 0.05 * miss["lfu"]
    assert miss["light"] < miss["lru"]


# ---------------------------------------------------------------- row-wise Adagrad (one accumulator per row)
def test_rowwise_adagrad_with_rows_of_one_float_is_adagrad():
    """dim = 1: the mean of the squares is the square, so the row-wise form is the element-wise one
    (itself pinned to the library optimizer above)."""
    V, C, N = 80, 10, 25
    ids, grads, table = stream(43, V, N, 120, 1, alpha=1.1)
    a = Oracle(C, 1, 2, 1, N, 1, 1e-8, table)
    b = Oracle(C, 1, 2, 1, N, 2, 1e-8, table)
    for i, g in zip(ids, grads):
        x, _ = a.lookup(i); y, _ = b.lookup(i)
        assert np.array_equal(x, y)
        a.update(i, g, 0.05); b.update(i, g, 0.05)
    a.flush(); b.flush()
    assert np.array_equal(a.W, b.W) and np.array_equal(a.A, b.A)


def test_rowwise_adagrad_matches_library_adagrad_on_rows_of_equal_gradients():
    """If every component of a row's gradient is the same number c, the mean of the squares is c^2 and
    every component follows plain Adagrad with gradient c: the library optimizer on the dense table."""
    V, D, C, N, lr, eps = 40, 5, 40, 12, 0.1, 1e-10
    rng = np.random.default_rng(47)
    table = rng.standard_normal((V, D)) * 0.01
    o = Oracle(C, D, 3, 1, N, 2, eps, table)
    Wt = torch.tensor(table.copy(), dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adagrad([Wt], lr=lr, eps=eps)
    for t in range(60):
        ids = rng.integers(0, V, size=N).astype(np.int64)
        c = rng.standard_normal(N)
        grads = np.repeat(c[:, None], D, axis=1)
        out, _ = o.lookup(ids)
        np.testing.assert_allclose(out, Wt.detach().numpy()[ids], rtol=1e-12, atol=1e-15)
        o.update(ids, grads, lr)
        dense = np.zeros((V, D))
        np.add.at(dense, ids, grads)
        # rows that were not touched must not move: give them no gradient at all
        Wt.grad = torch.tensor(dense)
        before = Wt.detach().clone()
        opt.step()
        untouched = np.setdiff1d(np.arange(V), ids)
        assert torch.equal(Wt.detach()[untouched], before[untouched])
    o.flush()
    np.testing.assert_allclose(o.W, Wt.detach().numpy(), rtol=1e-12, atol=1e-15)


@pytest.mark.parametrize("policy,s,many", [(0, 0, False), (1, 2, False), (1, 3, True)])
def test_rowwise_adagrad_matches_brute_force_twin(policy, s, many):
    V, C, D, N = 50, 6, 4, 12
    ids, grads, table = stream(53 + policy, V, N, 100, D)
    o = Oracle(C, D, s, policy, N, 2, 1e-8, table, many_writers=many)
    b = brute.BruteCache(C, D, s, policy, N, 2, 1e-8, table, many=many)
    for i, g in zip(ids, grads):
        out, _ = o.lookup(i)
        assert np.array_equal(out, np.asarray(b.read(i.tolist())))
        o.update(i, g, 0.05)
        b.write(i.tolist(), g.tolist(), 0.05)
        assert o.last_evicted().tolist() == b.evicted
        assert np.array_equal(o.W, np.asarray(b.W))
        assert np.array_equal(o.A[:, 0], np.asarray(b.A)[:, 0])
    o.flush(); b.flush()
    assert np.array_equal(o.W, np.asarray(b.W)) and np.array_equal(o.A[:, 0], np.asarray(b.A)[:, 0])
