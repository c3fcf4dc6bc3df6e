"""The C oracle and the brute-force twin against a trace worked by hand from the paper's rules
(tests/golden/hand_trace.json; Section 3.1, Algorithms 2 and 3, Section 4.3)."""
import json
import os

import numpy as np
import pytest

from oracle import brute
from oracle.het_oracle import Oracle

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "hand_trace.json")))
CLS = {0: "hit", 1: "stale", 2: "miss"}


def _table():
    return np.asarray(GOLD["table"], dtype=np.float64).reshape(-1, 1)


@pytest.mark.parametrize("policy", ["lru", "lfu"])
@pytest.mark.parametrize("real", ["f64", "f32"])
def test_c_oracle_follows_hand_trace(policy, real):
    o = Oracle(GOLD["capacity"], 1, GOLD["s"], {"lru": 0, "lfu": 1}[policy],
               GOLD["max_batch_ids"], 0, 0.0, _table(), real=real)
    for step in GOLD["steps"]:
        out, rc = o.lookup(step["ids"])
        assert rc == 0
        assert out[:, 0].tolist() == step["out"]
        keys, cls, _ = o.last_lookup()
        assert {str(k): CLS[c] for k, c in zip(keys.tolist(), cls.tolist())} == step["classes"]
        assert o.update(step["ids"], np.asarray(step["grads"], float).reshape(-1, 1),
                        GOLD["lr"]) == 0
        assert o.last_evicted().tolist() == step["evicted"][policy]
        st = o.export_state()
        rows, _ = o.export_rows()
        got = [[int(st["key"][i]), int(st["slot"][i]), int(st["cs"][i]), int(st["cc"][i]),
                int(st["last_use"][i]), int(st["freq"][i]), float(rows[i, 0])]
               for i in range(len(st["key"]))]
        assert got == step["state_after_update"][policy]
    assert o.W[:, 0].tolist() == GOLD["global_before_flush"][policy]["W"]
    assert o.Cg.tolist() == GOLD["global_before_flush"][policy]["c_g"]
    assert o.flush() == 0
    assert o.W[:, 0].tolist() == GOLD["global_after_flush"]["W"]
    assert o.Cg.tolist() == GOLD["global_after_flush"]["c_g"]
    st = o.export_state()
    assert np.array_equal(st["cs"], st["cc"])


@pytest.mark.parametrize("policy", ["lru", "lfu"])
def test_brute_twin_follows_hand_trace(policy):
    b = brute.BruteCache(GOLD["capacity"], 1, GOLD["s"], {"lru": 0, "lfu": 1}[policy],
                         GOLD["max_batch_ids"], 0, 0.0, _table())
    for step in GOLD["steps"]:
        out = b.read(step["ids"])
        assert [r[0] for r in out] == step["out"]
        assert {str(k): v for k, v in b.classes.items()} == step["classes"]
        b.write(step["ids"], [[g] for g in step["grads"]], GOLD["lr"])
        assert b.evicted == step["evicted"][policy]
        got = [[k, sl, cs, cc, lu, fr, b.find(k).row[0]] for k, sl, cs, cc, lu, fr in b.state()]
        assert got == step["state_after_update"][policy]
    assert [r[0] for r in b.W] == GOLD["global_before_flush"][policy]["W"]
    assert b.c_g == GOLD["global_before_flush"][policy]["c_g"]
    b.flush()
    assert [r[0] for r in b.W] == GOLD["global_after_flush"]["W"]
    assert b.c_g == GOLD["global_after_flush"]["c_g"]
