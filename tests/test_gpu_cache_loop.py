"""End to end on the GPU: the paper's online loop for a stream of queries (Sec. 3, Sec. 4.1.1, Sec. 4.2.2, App. B.2) --
match the retrieved chunk list in the cache tree, run the layer stack on the rows that are not covered, slice the
new chunks' K/V into the slots the tree hands out, clear what the tree evicts -- against a plain full prefill of the
same prompt (GPU, same kernels, no cache) and, for the first queries, the CPU oracle's stack.

Synthetic stand-in for text: a chunk is a fixed block of hidden-state rows drawn from its id (so the same chunk is
the same rows wherever it appears, and tokenization is always consistent)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2601_11553_amd import workloads as wl
from paper_2601_11553_amd.binding import CacheTree, Percache

from gpu_util import DEV, bf16, host
from test_gpu_stack import EPS, check_hidden, dev_layers, oracle_block

pytestmark = pytest.mark.gpu

H, HQ, HKV, D, F, L, C = 256, 4, 2, 64, 384, 2, 64
TAIL = 4


def chunk_rows(cid: int) -> np.ndarray:
    g = np.random.default_rng([77, cid])
    n = int(g.integers(20, C + 1))
    return wl.round_bf16(g.standard_normal((n, H)).astype(np.float32))


def run_stream(n_slots, byte_limit, queries, check_oracle=2):
    Ws = [wl.stack_weights(5, l, H, HQ, HKV, D, F) for l in range(L)]
    layers = dev_layers(Ws)
    pc = Percache(n_layers=L, hidden=H, n_q_heads=HQ, n_kv_heads=HKV, head_dim=D, n_slots=n_slots, slot_capacity=C,
                  max_pos=8 * C, device=DEV)
    plain = Percache(n_layers=L, hidden=H, n_q_heads=HQ, n_kv_heads=HKV, head_dim=D, n_slots=1, slot_capacity=C,
                     max_pos=8 * C, device=DEV)
    bytes_per_token = L * 2 * HKV * D * 2
    tree = CacheTree(n_slots, byte_limit, bytes_per_token, TAIL)
    stats = dict(reused_tokens=0, total_tokens=0, evictions=0)
    for qi, (cids, tq) in enumerate(queries):
        texts = [f"chunk {c}" for c in cids]
        rows = [chunk_rows(c) for c in cids]
        toks = [r.shape[0] for r in rows]
        query = wl.round_bf16(np.random.default_rng([78, qi]).standard_normal((tq, H)).astype(np.float32))
        prompt = np.concatenate(rows + [query])
        starts = np.concatenate([[0], np.cumsum(toks)])
        # ---- match, then make room / get slots for the chain
        slots, used = tree.percache_tree_match(texts)
        shared, ins_slots, is_new, evicted = tree.percache_tree_insert(texts, toks)
        stats["evictions"] += len(evicted)
        # a matched node that the insertion evicted (it was not part of the shared prefix) can no longer be read
        for i, s in enumerate(slots):
            if s in evicted:
                slots, used = slots[:i], used[:i]
                break
        m = len(slots)
        l_pre = int(sum(used))
        # new nodes that lie inside the reused region (the re-stored end of the common prefix, App. B.2): their
        # tensors are the cached ones; copy slot to slot before anything is cleared
        for i in range(shared, len(cids)):
            if is_new[i] and i < m:
                for l in range(L):
                    k, v = pc.percache_kv_get(l, slots[i])
                    pc.percache_kv_put(l, ins_slots[i], k, v)
                is_new[i] = False
        for s in evicted:
            if s not in ins_slots:
                for l in range(L):
                    pc.percache_kv_evict(l, s)
        # ---- reuse pass over the uncovered rows; new chunks that start in the fresh part are sliced on the way
        fresh = prompt[l_pre:]
        bounds, save = [0], []
        for i in range(len(cids)):
            if is_new[i]:
                assert starts[i] >= l_pre, "a new chunk must lie in the recomputed part"
                if bounds[-1] != starts[i] - l_pre:
                    bounds.append(int(starts[i] - l_pre)); save.append(-1)
                bounds.append(int(starts[i + 1] - l_pre)); save.append(ins_slots[i])
        if bounds[-1] != fresh.shape[0]:
            bounds.append(fresh.shape[0]); save.append(-1)
        out = pc.percache_stack_reuse(layers, F, EPS, bf16(fresh[None]), [slots] if m else None, [used] if m else None,
                                      save_bounds=bounds, save_slots=[save])
        ref = plain.percache_stack_reuse(layers, F, EPS, bf16(prompt[None]))
        torch.cuda.synchronize()
        check_hidden(host(out[0, -tq:]), host(ref[0, -tq:]), f"query {qi}: chunks {cids}, {m} matched, L_pre {l_pre}", rel_max=2.0 ** -5)
        if qi < check_oracle:
            h = prompt
            for W in Ws:
                h, _, _ = oracle_block(h, W, HQ, HKV, D, 10000.0)
            check_hidden(host(out[0, -tq:]), h[-tq:], f"query {qi} vs oracle stack")
        for i, s in enumerate(ins_slots):
            for l in range(L):
                assert pc.percache_kv_len(l, s) == toks[i], (qi, i, s)
        stats["reused_tokens"] += l_pre
        stats["total_tokens"] += prompt.shape[0]
    return stats


def test_query_stream_with_room_for_everything():
    queries = [([1, 5, 7], 9), ([1, 5, 9], 12), ([1, 5, 9, 12], 8), ([1, 5, 7], 16), ([2], 5), ([1, 5, 9, 12], 11), ([2, 5], 7)]
    st = run_stream(24, 10 ** 9, queries)
    print(st, flush=True)
    assert st["evictions"] == 0 and st["reused_tokens"] > 0.3 * st["total_tokens"]


def test_query_stream_under_a_tight_limit():
    g = np.random.default_rng(11)
    queries = [([int(min(9, g.exponential(2.5))) for _ in range(int(g.integers(1, 4)))], int(g.integers(4, 20))) for _ in range(14)]
    st = run_stream(5, 10 ** 9, queries, check_oracle=0)
    print(st, flush=True)
    assert st["evictions"] > 0
