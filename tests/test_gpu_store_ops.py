"""The K/V store as a state machine (Sec. 4.1.1: one slot per chunk and layer; Sec. 2.1: a sequence's own K/V grows token
by token): seeded random sequences of put, batched put, append, slice, evict and get on a store with bf16 and 8-bit
slots, against a model on the host that keeps, per (layer, slot), what the slot must read back -- the bf16 input bit
for bit, or the oracle's quantiser (`oracle.kv_fp8`) for an 8-bit slot.  After every call the slots it names are read
back, and at the end every slot of every layer, so a write that strays into a neighbour shows too."""
import numpy as np
import pytest
import torch

from oracle import kv_fp8
from paper_2601_11553_amd import workloads as wl
from paper_2601_11553_amd.binding import Percache

from gpu_util import DEV, bf16, host

pytestmark = pytest.mark.gpu


def _tokens(g, Hkv, n, D, spread):
    return wl.round_bf16((g.standard_normal((Hkv, n, D)) * spread).astype(np.float32))


@pytest.mark.parametrize("seed", list(range(12)))
def test_seeded_random_store_ops(seed):
    g = np.random.default_rng(7000 + seed)
    D = int(g.choice([64, 128]))
    Hkv = int(g.choice([1, 2, 3]))
    C = int(g.choice([64, 128, 192, 320]))
    L = int(g.integers(1, 3))
    S = int(g.integers(3, 9))
    mode = seed % 3                                    # 0: bf16 slots, 1: 8-bit slots, 2: the last n8 slots 8-bit
    n8 = {0: 0, 1: 0, 2: int(g.integers(1, S))}[mode]
    pc = Percache(n_layers=L, hidden=128, n_q_heads=2 * Hkv, n_kv_heads=Hkv, head_dim=D, n_slots=S, slot_capacity=C,
                  max_pos=4 * C, kv_fp8=mode == 1, n_slots_8bit=n8, device=DEV)
    is8 = (lambda s: True) if mode == 1 else (lambda s: s >= S - n8)
    keep = lambda x, s: kv_fp8.round_trip(x) if is8(s) else x
    model = {(l, s): None for l in range(L) for s in range(S)}

    def check(l, s, what):
        want = model[(l, s)]
        n = pc.percache_kv_len(l, s)
        assert n == (0 if want is None else want[0].shape[1]), (what, l, s, n)
        if want is not None:
            k, v = pc.percache_kv_get(l, s)
            torch.cuda.synchronize()
            assert np.array_equal(host(k), want[0]), (what, "K", l, s)
            assert np.array_equal(host(v), want[1]), (what, "V", l, s)

    for step in range(40):
        l = int(g.integers(0, L))
        op = g.choice(["put", "put_batch", "append", "slice", "evict"], p=[0.25, 0.15, 0.3, 0.15, 0.15])
        spread = float(g.choice([0.01, 1.0, 30.0]))
        what = f"seed {seed} step {step} {op}"
        if op == "put":
            s, n = int(g.integers(0, S)), int(g.integers(1, C + 1))
            k, v = _tokens(g, Hkv, n, D, spread), _tokens(g, Hkv, n, D, 1.0)
            pc.percache_kv_put(l, s, bf16(k), bf16(v))
            model[(l, s)] = (keep(k, s), keep(v, s))
            touched = [s]
        elif op == "put_batch":
            m, n = int(g.integers(1, S + 1)), int(g.integers(1, C + 1))
            slots = [int(x) for x in g.permutation(S)[:m]]
            k = np.stack([_tokens(g, Hkv, n, D, spread) for _ in slots])
            v = np.stack([_tokens(g, Hkv, n, D, 1.0) for _ in slots])
            pc.percache_kv_put_batch(l, slots, bf16(k), bf16(v))
            for i, s in enumerate(slots):
                model[(l, s)] = (keep(k[i], s), keep(v[i], s))
            touched = slots
        elif op == "append":
            s = int(g.integers(0, S))
            have = 0 if model[(l, s)] is None else model[(l, s)][0].shape[1]
            if have == C:
                continue
            n = int(g.integers(1, min(C - have, 70) + 1))
            k, v = _tokens(g, Hkv, n, D, spread), _tokens(g, Hkv, n, D, 1.0)
            pc.percache_kv_append(l, s, bf16(k), bf16(v))
            if model[(l, s)] is None:
                model[(l, s)] = (keep(k, s), keep(v, s))
            elif is8(s):
                model[(l, s)] = (kv_fp8.append(model[(l, s)][0], k), kv_fp8.append(model[(l, s)][1], v))
            else:
                model[(l, s)] = (np.concatenate([model[(l, s)][0], k], axis=1), np.concatenate([model[(l, s)][1], v], axis=1))
            touched = [s]
        elif op == "slice":
            m = int(g.integers(1, min(S, 4) + 1))
            lens = [int(x) for x in g.integers(1, C + 1, size=m)]
            bounds = [0] + [int(x) for x in np.cumsum(lens)]
            slots = [int(x) for x in g.permutation(S)[:m]]
            if m > 1 and g.random() < 0.5:
                slots[int(g.integers(0, m))] = -1              # a piece that is not kept
            k, v = _tokens(g, Hkv, bounds[-1], D, spread), _tokens(g, Hkv, bounds[-1], D, 1.0)
            pc.percache_kv_slice(l, bf16(k), bf16(v), bounds, slots)
            for j, s in enumerate(slots):
                if s >= 0:
                    model[(l, s)] = (keep(k[:, bounds[j]:bounds[j + 1]], s), keep(v[:, bounds[j]:bounds[j + 1]], s))
            touched = [s for s in slots if s >= 0]
        else:
            s = int(g.integers(0, S))
            pc.percache_kv_evict(l, s)
            model[(l, s)] = None
            touched = [s]
        for s in touched:
            check(l, s, what)
    for (l, s) in model:
        check(l, s, f"seed {seed} final")
    pc.close()
