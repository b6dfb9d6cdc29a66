"""Decoding steps over [reused chunks ; the prompt's own K/V ; generated tokens] through the slot gather, and the slot
append they rely on, through the C ABI.

There is no language-model head here: the "generated token" fed to step i is a seeded row of hidden state.  The reference
for every step is a plain prefill of the whole sequence so far (GPU, no cache) and, at the last step, the CPU oracle's stack for every query of the batch."""
import numpy as np
import pytest
import torch

from paper_2601_11553_amd import workloads as wl
from paper_2601_11553_amd.binding import Percache, PercacheError

from gpu_util import DEV, bf16, host
from test_gpu_stack import EPS, check_hidden, dev_layers, oracle_block

pytestmark = pytest.mark.gpu


def test_kv_append_equals_put_of_the_concatenation():
    Hkv, D, C = 2, 128, 192
    pc = Percache(n_layers=1, hidden=256, n_q_heads=2, n_kv_heads=Hkv, head_dim=D, n_slots=3, slot_capacity=C, max_pos=256, device=DEV)
    g = np.random.default_rng(1)
    k = bf16(g.standard_normal((Hkv, 150, D)))
    v = bf16(g.standard_normal((Hkv, 150, D)))
    pc.percache_kv_put(0, 0, k, v)
    cuts = [0, 37, 38, 64, 65, 129, 150]                      # appends that start / end inside and on block borders
    for lo, hi in zip(cuts[:-1], cuts[1:]):
        pc.percache_kv_append(0, 1, k[:, lo:hi].contiguous(), v[:, lo:hi].contiguous())
        assert pc.percache_kv_len(0, 1) == hi
    ka, va = pc.percache_kv_get(0, 1)
    torch.cuda.synchronize()
    assert torch.equal(ka, k) and torch.equal(va, v)
    with pytest.raises(PercacheError) as e:
        pc.percache_kv_append(0, 1, k[:, :43].contiguous(), v[:, :43].contiguous())   # 150 + 43 > 192
    assert e.value.status == -4 and pc.percache_kv_len(0, 1) == 150
    with pytest.raises(PercacheError) as e:                                           # tensors that are not 16-byte aligned
        pc.percache_kv_append(0, 2, k.reshape(-1)[1:1 + Hkv * 2 * D].view(Hkv, 2, D), v[:, :2].contiguous())
    assert e.value.status == -1 and pc.percache_kv_len(0, 2) == 0
    # attention over the appended slot equals attention over the slot written at once (same padding behaviour)
    q = bf16(g.standard_normal((1, 2, 5, D)))
    kf = bf16(g.standard_normal((1, Hkv, 5, D)))
    vf = bf16(g.standard_normal((1, Hkv, 5, D)))
    a0 = pc.percache_attention_reuse(0, q, kf, vf, [[0]])
    a1 = pc.percache_attention_reuse(0, q, kf, vf, [[1]])
    torch.cuda.synchronize()
    assert torch.equal(a0, a1)


@pytest.mark.parametrize("batch,D,Hq", [(1, 64, 4), (3, 64, 4), (2, 128, 8), (1, 128, 2)])
def test_decode_steps_match_full_prefill(batch, D, Hq):
    _decode_case(batch, D, Hq, 2, 256, 384, 2, 64, 2, 20, 6, 40 + batch, full_slot=True)


@pytest.mark.parametrize("seed", list(range(12)))
def test_seeded_random_decode_shapes(seed):
    """Shapes drawn from a seed: batch, head size, GQA ratio, widths, layers, chunk count (none included) and capacity,
    prompt length, number of steps (the sequence slot ends exactly full in some draws)."""
    g = np.random.default_rng(9000 + seed)
    D = int(g.choice([64, 128]))
    Hkv = int(g.choice([1, 2, 4]))
    Hq = Hkv * int(g.choice([1, 2, 4]))
    while ((Hq + 2 * Hkv) * D) % 128:
        Hq += Hkv
    C = int(g.choice([64, 128]))
    n_steps = int(g.integers(1, 6))
    t_prompt = int(g.choice([1, 2, 31, C - n_steps]))
    _decode_case(int(g.integers(1, 4)), D, Hq, Hkv, int(g.choice([128, 256, 384])), int(g.choice([192, 448])),
                 int(g.integers(1, 3)), C, int(g.integers(0, 4)), t_prompt, n_steps, 9100 + seed, full_slot=False)


def _decode_case(batch, D, Hq, Hkv, H, F, L, C, n_c, t_prompt, n_steps, seed, full_slot):
    Ws = [wl.stack_weights(31, l, H, Hq, Hkv, D, F) for l in range(L)]
    layers = dev_layers(Ws)
    n_slots = batch * (n_c + 1)
    pc = Percache(n_layers=L, hidden=H, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=D, n_slots=n_slots, slot_capacity=C,
                  max_pos=n_c * C + C, device=DEV)
    plain = Percache(n_layers=L, hidden=H, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=D, n_slots=1, slot_capacity=C,
                     max_pos=n_c * C + C, device=DEV)
    g = np.random.default_rng(seed)
    total = n_c * C + t_prompt + n_steps
    seqs = wl.round_bf16(g.standard_normal((batch, total, H)).astype(np.float32))   # chunks, prompt, then the fed tokens
    chunk_slots = [[b * (n_c + 1) + c for c in range(n_c)] for b in range(batch)]
    seq_slots = [b * (n_c + 1) + n_c for b in range(batch)]
    # population: each query's chunks and prompt are prefilled once; chunk K/V -> chunk slots, prompt K/V -> the sequence slot
    bounds = [c * C for c in range(n_c + 1)] + [n_c * C + t_prompt]
    pc.percache_stack_reuse(layers, F, EPS, bf16(seqs[:, :n_c * C + t_prompt]), save_bounds=bounds,
                            save_slots=[chunk_slots[b] + [seq_slots[b]] for b in range(batch)])
    for step in range(n_steps):
        pos = n_c * C + t_prompt + step
        x = bf16(seqs[:, pos:pos + 1])
        chains = [chunk_slots[b] + [seq_slots[b]] for b in range(batch)]
        out = pc.percache_stack_decode(layers, F, EPS, x, chains, seq_slots)
        ref = plain.percache_stack_reuse(layers, F, EPS, bf16(seqs[:, :pos + 1]))
        torch.cuda.synchronize()
        for b in range(batch):
            assert pc.percache_kv_len(0, seq_slots[b]) == t_prompt + step + 1 == pc.percache_kv_len(L - 1, seq_slots[b])
        check_hidden(host(out[:, 0]), host(ref[:, -1]), f"decode step {step} (batch {batch} D {D} heads {Hq}/{Hkv} H {H} layers {L} "
                     f"chunks {n_c}x{C} prompt {t_prompt}) vs full prefill", rel_max=2.0 ** -5)
    for b in range(batch):
        h = seqs[b]
        for W in Ws:
            h, _, _ = oracle_block(h, W, Hq, Hkv, D, 10000.0)
        check_hidden(host(out[b, 0]), h[-1], f"last decode step vs oracle stack, query {b}")
    if not full_slot:
        return
    # a sequence slot that is full refuses the step and nothing changes
    filler = bf16(g.standard_normal((Hkv, C - t_prompt - n_steps, D)))
    for l in range(L):
        pc.percache_kv_append(l, seq_slots[0], filler, filler)
    with pytest.raises(PercacheError) as e:
        pc.percache_stack_decode(layers, F, EPS, x, chains, seq_slots)
    assert e.value.status == -4 and pc.percache_kv_len(0, seq_slots[-1]) == t_prompt + n_steps + (C - t_prompt - n_steps if batch == 1 else 0)
