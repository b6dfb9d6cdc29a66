"""Chunk prefix tree with LFU eviction (Sec. 4.1.1, Sec. 4.2.2, App. B.2): host logic, no GPU.

The C library is checked against (a) the worked example the paper gives in App. B.2, (b) hand-computed eviction
orders, (c) an independent plain-Python reference on long random query streams (every returned slot, length and
evicted slot must agree), (d) invariants."""
import os

import numpy as np
import pytest

from oracle.cache_tree_ref import TreeRef
from paper_2601_11553_amd.binding import CacheTree, PercacheError

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "cache_tree_appendix_b2.txt")
TOK = 100


def both(n_slots=16, limit=10**9, bpt=1, tail=0):
    return CacheTree(n_slots, limit, bpt, tail), TreeRef(n_slots, limit, bpt, tail)


def test_appendix_b2_example():
    for impl in both(tail=7):
        is_c = isinstance(impl, CacheTree)
        ins = impl.percache_tree_insert if is_c else impl.insert
        mat = impl.percache_tree_match if is_c else impl.match
        slot_of = {}
        for line in open(GOLDEN):
            if line.startswith("#") or not line.strip():
                continue
            op, ids, expect = [p.strip() for p in line.split(";")]
            chunks = [f"chunk {i}" for i in ids.split()]
            e = expect.split()
            if op == "insert":
                shared, slots, new, ev = ins(chunks, [TOK] * len(chunks))
                assert shared == int(e[1]) and sum(new) == int(e[3]) and ev == []
                slot_of[ids] = slots
            elif op == "nodes":
                assert (impl.percache_tree_nodes() if is_c else impl.n_nodes()) == int(e[0])
            else:
                slots, used = mat(chunks)
                assert len(slots) == int(e[1])
                assert used == [TOK] * (len(slots) - 1) + [TOK - 7]          # tail of the final node is not reused
                if "last_node_is_child_of_second_5" in e:
                    assert slots == slot_of["1 5 9"] and slots[1] != slot_of["1 5 7"][1] and slots[0] == slot_of["1 5 7"][0]


def test_lfu_order_by_hand():
    t = CacheTree(4, 10**9, 1, 0)
    assert t.percache_tree_insert(["a"], [10])[1] == [0]
    assert t.percache_tree_insert(["b"], [10])[1] == [1]
    assert t.percache_tree_insert(["c"], [10])[1] == [2]
    assert t.percache_tree_insert(["d"], [10])[1] == [3]
    for q in (["a"], ["a"], ["c"], ["d"], ["d"], ["d"]):
        t.percache_tree_match(q)
    # counts: a 2, b 0, c 1, d 3 -> b goes first; e (never retrieved) takes its slot and is the next to go, then c
    assert t.percache_tree_insert(["e"], [10])[3] == [1]
    assert t.percache_tree_insert(["f", "g"], [10, 10])[3] == [1, 2]
    assert t.percache_tree_match(["d"])[0] == [3] and t.percache_tree_match(["a"])[0] == [0]
    assert t.percache_tree_match(["c"])[0] == [] and t.percache_tree_match(["f", "g"])[0] == [1, 2]
    # byte limit: 35 bytes hold three 10-token chunks
    t = CacheTree(8, 35, 1, 0)
    t.percache_tree_insert(["x", "y", "z"], [10, 10, 10])
    s, slots, new, ev = t.percache_tree_insert(["x", "w"], [10, 10])
    # common prefix is (x): nothing shared (App. B.2), two new nodes, 50 bytes > 35: leaves z then y are evicted
    assert s == 0 and new == [True, True] and ev == [2, 1] and t.percache_tree_bytes() == 30
    with pytest.raises(PercacheError) as e:
        t.percache_tree_insert(["p", "q", "r", "s"], [10, 10, 10, 10])    # 40 bytes can never fit
    assert e.value.status == -5 and e.value.evicted == []


@pytest.mark.parametrize("seed,n_slots,limit,tail", [(0, 12, 10**9, 0), (1, 40, 900, 3), (2, 6, 10**9, 5), (3, 25, 2000, 0)])
def test_random_streams_agree_with_reference(seed, n_slots, limit, tail):
    g = np.random.default_rng(seed)
    c, r = both(n_slots, limit, 1, tail)
    universe = [f"chunk-{i}" for i in range(14)]
    tokens = {u: int(g.integers(20, 120)) for u in universe}
    live = {}
    for step in range(600):
        k = int(g.integers(1, 5))
        # popular chunks first so that prefixes repeat
        q = [universe[min(13, int(g.exponential(3.0)))] for _ in range(k)]
        sc, uc = c.percache_tree_match(q)
        sr, ur = r.match(q)
        assert (sc, uc) == (sr, ur), (step, q)
        if len(sc) < k:
            tk = [tokens[x] for x in q]
            try:
                out_r = r.insert(q, tk)
            except MemoryError:
                with pytest.raises(PercacheError):
                    c.percache_tree_insert(q, tk)
                continue
            out_c = c.percache_tree_insert(q, tk)
            assert out_c == out_r, (step, q)
            for s in out_c[3]:
                live.pop(s)
            for s, nw, x in zip(out_c[1], out_c[2], q):
                if nw:
                    assert s not in live                      # a slot is never handed out twice
                    live[s] = x
                else:
                    assert live[s] == x                       # a shared slot holds that chunk
        assert c.percache_tree_nodes() == r.n_nodes() == len(live)
        assert c.percache_tree_bytes() == r.bytes <= limit and len(live) <= n_slots


def test_bad_arguments():
    with pytest.raises(PercacheError):
        CacheTree(0, 10, 1, 0)
    t = CacheTree(2, 100, 1, 0)
    with pytest.raises(PercacheError):
        t.percache_tree_insert(["a"], [0])
    with pytest.raises(PercacheError) as e:
        t.percache_tree_insert(["a", "b", "c"], [1, 1, 1])      # more new nodes than slots
    assert e.value.status == -5
    assert t.percache_tree_match([]) == ([], [])
