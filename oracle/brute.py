"""List-based brute-force twin of the cache protocol, for tiny inputs.  Test infrastructure only.

Written separately from `het_oracle.c` and as naively as possible (a Python list of cached
entries, linear search, a full sort of all entries at every trim) so that the two can be
compared on small random cases.  Follows Section 3.1 (Fetch, Evict, CheckValid), Algorithm 2
(Read) and Algorithm 3 (Write) of the paper, with the same single-worker readings as the C file.
Values are Python floats (fp64).
"""
from __future__ import annotations

import math

HIT, STALE, MISS = "hit", "stale", "miss"
S_INF = (1 << 63) - 1


class Entry:
    def __init__(self, key, slot, row, acc, clock):
        self.key, self.slot = key, slot
        self.row, self.acc = list(row), list(acc)
        self.row0, self.acc0 = list(row), list(acc)      # as fetched (several workers: deltas are pushed)
        self.c_s = self.c_c = clock
        self.last_use, self.freq = 0, 0


class BruteCache:
    def __init__(self, capacity, dim, s, policy, max_batch_ids, optimizer, eps, table, many=False, server=None, lfu_cap=16):
        """`many`: one of several workers over one server (Evict pushes what was accumulated since
        the Fetch, and the server adds it); `server`: another BruteCache whose global table is used."""
        self.C, self.D, self.s = capacity, dim, s
        self.policy, self.opt, self.eps = policy, optimizer, float(eps)
        self.P = capacity + max_batch_ids
        self.many = many
        self.lfu_cap = lfu_cap         # policy 3, light-weight LFU: rows used this often are no longer kept track of
        if server is not None:
            self.W, self.A, self.c_g = server.W, server.A, server.c_g
        else:
            self.W = [[float(x) for x in r] for r in table]      # global table
            self.A = [[0.0] * dim for _ in table]         # (row-wise Adagrad, optimizer 2, uses the first entry only)
            self.c_g = [0] * len(table)
        self.entries = []                                      # the cache embedding table
        self.t = 0
        self.evicted = []
        self.classes = {}
        self.pushes = 0            # rows actually sent to the server

    def find(self, k):
        for e in self.entries:
            if e.key == k:
                return e
        return None

    def push(self, e):
        """Evict's message to the server: accumulated updates and the local clock."""
        if e.c_c == e.c_s:
            return False
        self.pushes += 1
        if self.many:
            for j in range(self.D):
                self.W[e.key][j] = self.W[e.key][j] + (e.row[j] - e.row0[j])
                if self.opt == 1 or (self.opt == 2 and j == 0):
                    self.A[e.key][j] = self.A[e.key][j] + (e.acc[j] - e.acc0[j])
        else:
            self.W[e.key] = list(e.row)
            self.A[e.key] = list(e.acc)
        self.c_g[e.key] = max(self.c_g[e.key], e.c_c)
        return True

    def check_valid(self, e):
        return e.c_c <= e.c_s + self.s and self.c_g[e.key] <= e.c_c + self.s

    def evict_overflow(self):
        self.evicted = []
        m = len(self.entries) - self.C
        if m <= 0:
            return
        if self.policy == 0:
            order = sorted(self.entries, key=lambda e: (e.last_use, e.slot))
        else:
            order = sorted(self.entries, key=lambda e: (e.freq, e.last_use, e.slot))
        for e in order[:m]:
            self.push(e)
            self.evicted.append(e.key)
            self.entries.remove(e)

    def read(self, ids):
        if len(ids) == 0:
            return []
        self.t += 1
        if len(self.entries) > self.C:
            self.evict_overflow()
        self.classes = {}
        for k in sorted(set(ids)):
            e = self.find(k)
            if e is not None:
                if not self.check_valid(e):
                    self.push(e)
                    e.row, e.acc = list(self.W[k]), list(self.A[k])
                    e.row0, e.acc0 = list(e.row), list(e.acc)
                    e.c_s = e.c_c = self.c_g[k]
                    self.classes[k] = STALE
                else:
                    self.classes[k] = HIT
            else:
                used = {x.slot for x in self.entries}
                slot = min(set(range(self.P)) - used)
                self.entries.append(Entry(k, slot, self.W[k], self.A[k], self.c_g[k]))
                self.classes[k] = MISS
        for k in set(ids):
            e = self.find(k)
            if self.policy == 3 and e.freq >= self.lfu_cap:
                continue
            e.last_use = self.t
            e.freq += 1
        return [list(self.find(k).row) for k in ids]

    def write(self, ids, grads, lr):
        if len(ids) == 0:
            return
        G = {}
        for i, k in enumerate(ids):
            g = G.setdefault(k, [0.0] * self.D)
            for j in range(self.D):
                g[j] = g[j] + float(grads[i][j])
        for k in sorted(G):
            e = self.find(k)
            if self.opt == 2:
                e.acc[0] = e.acc[0] + self._mean_sq(G[k])
            for j in range(self.D):
                g = G[k][j]
                if self.opt == 2:
                    e.row[j] = e.row[j] - (lr * g) / (math.sqrt(e.acc[0]) + self.eps)
                elif self.opt == 0:
                    e.row[j] = e.row[j] - lr * g
                else:
                    e.acc[j] = e.acc[j] + g * g
                    e.row[j] = e.row[j] - (lr * g) / (math.sqrt(e.acc[j]) + self.eps)
            e.c_c += 1
        self.evict_overflow()

    def _mean_sq(self, g):
        ss = 0.0
        for v in g:
            ss = ss + v * v
        return ss / self.D

    def flush(self):
        for e in self.entries:
            if self.push(e):
                e.c_s = e.c_c = self.c_g[e.key]
                e.row0, e.acc0 = list(e.row), list(e.acc)

    def state(self):
        """(key, slot, c_s, c_c, last_use, freq) of every cached row, ascending slot."""
        return sorted(((e.key, e.slot, e.c_s, e.c_c, e.last_use, e.freq) for e in self.entries),
                      key=lambda r: r[1])
