"""Pins of the oracle's several-workers mode (the literal Evict of Section 3.1: a worker pushes
what it accumulated since its Fetch and the server adds it; CheckValid's second condition;
Lemma 1) against things other than itself: the single-writer oracle, a closed form, the bounds
CheckValid enforces, and a two-worker brute-force twin."""
import itertools

import numpy as np
import pytest

from oracle import brute
from oracle.het_oracle import S_INF, Oracle
from test_oracle_pins import CLS, stream


def two_workers(C, D, s, policy, N, opt, table):
    a = Oracle(C, D, s, policy, N, opt, 1e-8, table, many_writers=True)
    b = Oracle(C, D, s, policy, N, opt, 1e-8, None, many_writers=True, share_with=a)
    return a, b


@pytest.mark.parametrize("policy,opt,s", [(0, 0, 0), (1, 0, 3), (0, 1, 2), (1, 1, S_INF)])
def test_with_one_worker_the_delta_push_equals_the_write_back(policy, opt, s):
    """One writer: adding (row - row as fetched) to the global row gives the row itself, up to the
    rounding of that one addition; every integer of the protocol is the same."""
    V, C, D, N = 120, 9, 4, 30
    ids, grads, table = stream(31 + policy, V, N, 150, D, alpha=1.1)
    one = Oracle(C, D, s, policy, N, opt, 1e-8, table)
    many = Oracle(C, D, s, policy, N, opt, 1e-8, table, many_writers=True)
    for i, g in zip(ids, grads):
        o1, _ = one.lookup(i)
        o2, _ = many.lookup(i)
        np.testing.assert_allclose(o2, o1, rtol=1e-12, atol=1e-15)
        assert all(np.array_equal(x, y) for x, y in zip(one.last_lookup(), many.last_lookup()))
        one.update(i, g, 0.05)
        many.update(i, g, 0.05)
        assert one.last_evicted().tolist() == many.last_evicted().tolist()
        s1, s2 = one.export_state(), many.export_state()
        assert all(np.array_equal(s1[c], s2[c]) for c in s1)
        assert np.array_equal(one.Cg, many.Cg)
    one.flush(); many.flush()
    np.testing.assert_allclose(many.W, one.W, rtol=1e-12, atol=1e-15)
    if opt:
        np.testing.assert_allclose(many.A, one.A, rtol=1e-12, atol=1e-15)
    assert one.stats()[1] == many.stats()[1]


@pytest.mark.parametrize("policy,s,C", [(0, 0, 6), (1, 2, 6), (0, 7, 25), (1, S_INF, 4), (1, 1, 300)])
def test_two_workers_sgd_closed_form(policy, s, C):
    """SGD's step does not depend on the row, so whatever the staleness, the policy and the order in
    which pushes reach the server, once both workers have flushed the global table is the initial
    one minus lr times the sum of every gradient either of them wrote."""
    V, D, N, lr = 150, 3, 24, 0.05
    ids_a, g_a, table = stream(41 + C, V, N, 140, D, alpha=1.05)
    ids_b, g_b, _ = stream(97 + C, V, N, 140, D, alpha=1.05)
    a, b = two_workers(C, D, s, policy, N, 0, table)
    total = np.zeros((V, D))
    for t in range(140):
        for w, ids, g in ((a, ids_a[t], g_a[t]), (b, ids_b[t], g_b[t])):
            w.lookup(ids)
            w.update(ids, g, lr)
            np.add.at(total, ids, g)
        if t % 3 == 0:                      # the workers do not run in lockstep
            b.lookup(ids_b[(t * 7) % 140])
    a.flush(); b.flush()
    np.testing.assert_allclose(a.W, table - lr * total, rtol=1e-10, atol=1e-12)
    # and a second flush has nothing left to push
    before = a.W.copy()
    a.flush(); b.flush()
    assert np.array_equal(a.W, before)


@pytest.mark.parametrize("s", [0, 1, 3, 8])
def test_checkvalid_bounds_after_every_read_and_lemma_one(s):
    """Right after a worker's Read, every key of the batch satisfies both conditions of CheckValid
    against the global clock as it is then: c_c <= c_s + s and c_g <= c_c + s, with c_s <= c_g.
    Lemma 1: two replicas that are both valid against one global clock differ by at most 2s."""
    V, C, D, N, lr = 60, 30, 2, 20, 0.1
    ids_a, g_a, table = stream(51 + s, V, N, 200, D, alpha=0.9)
    ids_b, g_b, _ = stream(151 + s, V, N, 200, D, alpha=0.9)
    a, b = two_workers(C, D, s, 1, N, 0, table)
    compared = 0

    def clocks(w, keys):
        st = w.export_state()
        at = {k: i for i, k in enumerate(st["key"].tolist())}
        idx = [at[k] for k in keys]
        return st["cs"][idx].astype(np.int64), st["cc"][idx].astype(np.int64)

    for t in range(200):
        a.lookup(ids_a[t])
        ka = np.unique(ids_a[t])
        cs, cc = clocks(a, ka.tolist())
        cg = a.Cg[ka].astype(np.int64)
        assert np.all(cc - cs <= s) and np.all(cg - cc <= s) and np.all(cs <= cg)
        cg_at_a = a.Cg.copy()
        b.lookup(ids_b[t])
        kb = np.unique(ids_b[t])
        cs, cc = clocks(b, kb.tolist())
        cg = b.Cg[kb].astype(np.int64)
        assert np.all(cc - cs <= s) and np.all(cg - cc <= s) and np.all(cs <= cg)
        # keys both have just validated against the same global clock
        both = [k for k in np.intersect1d(ka, kb).tolist() if cg_at_a[k] == a.Cg[k]]
        if both:
            _, cca = clocks(a, both)
            _, ccb = clocks(b, both)
            assert np.all(np.abs(cca - ccb) <= 2 * s)
            compared += len(both)
        a.update(ids_a[t], g_a[t], lr)
        b.update(ids_b[t], g_b[t], lr)
    assert compared > 200


@pytest.mark.parametrize("policy,opt,s", list(itertools.product((0, 1), (0, 1), (0, 2, S_INF))))
def test_two_workers_match_the_brute_force_twin(policy, opt, s):
    """Two caches over one global table, calls interleaved unevenly, against the list-based twin:
    Read values, classes, slots, evicted ids, every cached row's clocks and the global table."""
    V, C, D, N = 40, 5, 3, 10
    ids_a, g_a, table = stream(61 + policy + 2 * opt, V, N, 90, D)
    ids_b, g_b, _ = stream(161 + policy + 2 * opt, V, N, 90, D)
    oa, ob = two_workers(C, D, s, policy, N, opt, table)
    ba = brute.BruteCache(C, D, s, policy, N, opt, 1e-8, table, many=True)
    bb = brute.BruteCache(C, D, s, policy, N, opt, 1e-8, None, many=True, server=ba)

    def read(o, b, i):
        out, rc = o.lookup(i)
        assert rc == 0
        assert np.array_equal(out, np.asarray(b.read(i.tolist())))
        keys, cls, slots = o.last_lookup()
        assert {k: CLS[c] for k, c in zip(keys.tolist(), cls.tolist())} == b.classes
        assert all(b.find(k).slot == sl for k, sl in zip(keys.tolist(), slots.tolist()))

    def write(o, b, i, g):
        assert o.update(i, g, 0.05) == 0
        b.write(i.tolist(), g.tolist(), 0.05)
        assert o.last_evicted().tolist() == b.evicted

    for t in range(90):
        read(oa, ba, ids_a[t])
        read(ob, bb, ids_b[t])
        if t % 4 == 1:
            read(oa, ba, ids_a[t])            # a Read that follows a Read
        write(ob, bb, ids_b[t], g_b[t])
        write(oa, ba, ids_a[t], g_a[t])
        if t % 5 == 2:                        # a worker that is not modelled pushes too
            k = np.unique(ids_a[t])[:3]
            d = np.full((len(k), D), 0.25)
            oa.foreign_update(k, d)
            for kk in k.tolist():
                ba.W[kk] = [x + 0.25 for x in ba.W[kk]]
                ba.c_g[kk] += 1
        for o, b in ((oa, ba), (ob, bb)):
            st = o.export_state()
            got = list(zip(*(st[c].tolist() for c in ("key", "slot", "cs", "cc", "last_use", "freq"))))
            assert got == b.state()
        assert oa.Cg.tolist() == ba.c_g
        assert np.array_equal(oa.W, np.asarray(ba.W))
    for o, b in ((oa, ba), (ob, bb)):
        o.flush(); b.flush()
    assert np.array_equal(oa.W, np.asarray(ba.W)) and oa.Cg.tolist() == ba.c_g
    if opt:
        assert np.array_equal(oa.A, np.asarray(ba.A))


def test_a_foreign_push_makes_clean_replicas_refetch():
    """The server's side of another worker's Evict: the global row moves and its clock advances.  A
    cached row without updates of its own whose clock falls more than s behind is fetched again at
    the next Read and shows the new value."""
    V, C, D, N, s = 30, 30, 2, 30, 1
    table = np.arange(V * D, dtype=np.float64).reshape(V, D)
    o = Oracle(C, D, s, 0, N, 0, 0.0, table, many_writers=True)
    keys = np.arange(10, dtype=np.int64)
    o.lookup(keys)
    d = np.ones((3, D))
    o.foreign_update(keys[:3], d)                 # c_g = 1 <= c_c + s = 1: still valid
    out, _ = o.lookup(keys)
    assert np.array_equal(out, table[:10]) and (o.last_lookup()[1] == 0).all()
    o.foreign_update(keys[:3], d)                 # c_g = 2 > c_c + s: stale
    out, _ = o.lookup(keys)
    assert (o.last_lookup()[1][:3] == 1).all() and (o.last_lookup()[1][3:] == 0).all()
    assert np.array_equal(out[:3], table[:3] + 2.0) and np.array_equal(out[3:], table[3:10])
    assert o.stats()[1]["stale_dirty"] == 0
