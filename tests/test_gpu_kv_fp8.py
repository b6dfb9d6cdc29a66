"""8-bit K/V slots through the C ABI: the codes and scales the GPU stores must be the oracle's bit for bit (checked on
the values read back, which are exact products code * 2^e), and attention over such slots must match the oracle's
attention over the same read-back values to the bf16 bar."""
import numpy as np
import pytest
import torch

import oracle
from oracle import kv_fp8
from oracle import kv_fp8 as kv_fp8_mod
from paper_2601_11553_amd import workloads as wl
from paper_2601_11553_amd.binding import Percache, PercacheError

from gpu_util import DEV, bf16, check_close, host

pytestmark = pytest.mark.gpu


def _ctx(D, C, n_slots=4, Hkv=2, **kw):
    args = dict(n_layers=1, hidden=256, n_q_heads=2 * Hkv, n_kv_heads=Hkv, head_dim=D, n_slots=n_slots, slot_capacity=C,
                max_pos=4 * C + 512, kv_fp8=True, device=DEV)
    args.update(kw)
    return Percache(**args)


@pytest.mark.parametrize("D", [64, 128])
def test_round_trip_is_the_oracles_quantiser(D):
    g = np.random.default_rng(D)
    Hkv, n, C = 2, 150, 192
    k = wl.round_bf16((g.standard_normal((Hkv, n, D)) * np.exp2(g.integers(-6, 7, (Hkv, n, 1)))).astype(np.float32))
    v = wl.round_bf16((g.standard_normal((Hkv, n, D)) * 0.3).astype(np.float32))
    v[1, 64:128] = 0.0                                    # an all-zero block
    k[0, 130:] *= 2.0 ** -100                              # tiny values: the exponent floor
    k = wl.round_bf16(k)
    pc = _ctx(D, C)
    pc.percache_kv_put(0, 2, bf16(k), bf16(v))
    kk, vv = pc.percache_kv_get(0, 2)
    torch.cuda.synchronize()
    assert pc.percache_kv_len(0, 2) == n
    assert np.array_equal(host(kk), kv_fp8.round_trip(k)), "K read back differs from the oracle's quantiser"
    assert np.array_equal(host(vv), kv_fp8.round_trip(v)), "V read back differs from the oracle's quantiser"
    pc.close()


def test_every_bf16_value_in_range_gets_the_oracles_code():
    """All finite bf16 values up to 448 in blocks whose largest element is 448 (scale 1), and again scaled by 2^-5 in
    blocks whose largest element is 448 * 2^-5 ... 1.75 * 2^3 = 14: every rounding case of the element conversion."""
    bits = np.arange(1 << 16, dtype=np.uint32)
    vals = (bits << 16).view(np.float32)
    vals = vals[np.isfinite(vals) & (np.abs(vals) <= 448.0)]
    D, Hkv = 64, 1
    n = -(-len(vals) // (D - 1))                           # one element of every row is the planted maximum
    n = -(-n // 64) * 64
    x = np.zeros((Hkv, n, D), np.float32)
    x[0, :, 1:].reshape(-1)[:len(vals)] = vals
    x[0, :, 0] = 448.0
    for scale in (1.0, 2.0 ** -5):
        xs = (x * scale).astype(np.float32)                # exact: powers of two
        pc = _ctx(D, n, n_slots=1, Hkv=1, max_pos=n + 64)
        pc.percache_kv_put(0, 0, bf16(xs), bf16(xs[:, ::-1].copy()))
        kk, vv = pc.percache_kv_get(0, 0)
        torch.cuda.synchronize()
        want = kv_fp8.round_trip(wl.round_bf16(xs))
        assert np.array_equal(host(kk), want)
        assert np.array_equal(host(vv), want[:, ::-1])
        pc.close()


def test_put_batch_slice_and_errors():
    g = np.random.default_rng(7)
    D, Hkv, C = 128, 2, 128
    pc = _ctx(D, C, n_slots=6)
    kb = wl.round_bf16(g.standard_normal((3, Hkv, 100, D)).astype(np.float32))
    vb = wl.round_bf16(g.standard_normal((3, Hkv, 100, D)).astype(np.float32) * 4)
    pc.percache_kv_put_batch(0, [5, 0, 3], bf16(kb), bf16(vb), 100)
    for i, s in enumerate([5, 0, 3]):
        kk, vv = pc.percache_kv_get(0, s)
        torch.cuda.synchronize()
        assert np.array_equal(host(kk), kv_fp8.round_trip(kb[i])) and np.array_equal(host(vv), kv_fp8.round_trip(vb[i]))
    # slicer: token ranges of a longer sequence; the scales are taken over each piece's own blocks
    seq_k = wl.round_bf16(g.standard_normal((Hkv, 230, D)).astype(np.float32))
    seq_v = wl.round_bf16(g.standard_normal((Hkv, 230, D)).astype(np.float32))
    pc.percache_kv_slice(0, bf16(seq_k), bf16(seq_v), [0, 128, 230], [1, 2])
    for lo, hi, s in [(0, 128, 1), (128, 230, 2)]:
        kk, vv = pc.percache_kv_get(0, s)
        torch.cuda.synchronize()
        assert np.array_equal(host(kk), kv_fp8.round_trip(seq_k[:, lo:hi])) and np.array_equal(host(vv), kv_fp8.round_trip(seq_v[:, lo:hi]))
    pc.close()


def _fill_fp8(pc, w, scale_k=1.0):
    """Puts the workload's slots (scaled K) and returns what the oracle reads back from them."""
    store = {}
    for s in sorted(set(int(x) for x in w.slot_ids.reshape(-1))):
        k, v = w.slot_kv(s)
        k = wl.round_bf16(k * np.float32(scale_k))
        pc.percache_kv_put(0, s, bf16(k), bf16(v))
        store[s] = (kv_fp8.round_trip(k), kv_fp8.round_trip(v))
    return store


def _oracle_on(store, w, b, X=None):
    ids = [int(s) for s in w.slot_ids[b]]
    sk = np.stack([store[s][0] for s in ids])
    sv = np.stack([store[s][1] for s in ids])
    return oracle.prefill_reuse(w.X[b] if X is None else X, w.Wqkv, w.n_q_heads, w.n_kv_heads, w.head_dim, w.rope_theta, sk, sv,
                                np.arange(len(ids), dtype=np.int32), w.used_len[b])


@pytest.mark.parametrize("D,t_fresh", [(128, 70), (64, 70), (128, 1), (64, 3)])
def test_attention_over_8_bit_slots(D, t_fresh):
    """Ragged chunks, several tiles per chunk, a fresh part with its causal mask (bf16 tiles), 1 to 70 fresh rows."""
    w = wl.make_prefill("fp8", 40 + D, "bf16", 512, 6, 2, D, 2, t_fresh, 3, 192, 8)
    w.used_len[0] = [192, 100, 1]
    w.used_len[1] = [65, 0, 190]
    pc = _ctx(D, 192, n_slots=8, hidden=512, n_q_heads=6, max_pos=w.max_pos)
    store = _fill_fp8(pc, w)
    for n_splits in (0, 1, 3):
        q, kf, vf = pc.percache_qkv_rope(0, bf16(w.X), bf16(w.Wqkv), w.slot_ids, w.used_len)
        out = pc.percache_attention_reuse(0, q, kf, vf, w.slot_ids, w.used_len, n_splits=n_splits)
        torch.cuda.synchronize()
        for b in range(2):
            O, _, _, _ = _oracle_on(store, w, b)
            check_close(host(out[b]), O, f"fp8 slots D={D} T={t_fresh} splits={n_splits} b={b}")
    pc.close()


def test_attention_over_8_bit_slots_256_row_workgroups_and_peaked_scores():
    """Enough stacked rows for the 8-wavefront kernel; K scaled x12 so that the softmax is peaked (scores up to +-60):
    a wrong element order in the 8-bit operands would show at once."""
    w = wl.make_prefill("fp8w", 77, "bf16", 256, 32, 8, 128, 4, 80, 2, 128, 12)
    w.used_len[:, 1] = 100
    pc = _ctx(128, 128, n_slots=12, hidden=256, n_q_heads=32, Hkv=8, max_pos=w.max_pos)
    store = _fill_fp8(pc, w, scale_k=12.0)
    out = pc.percache_prefill_reuse(0, bf16(w.X), bf16(w.Wqkv), w.slot_ids, w.used_len)
    torch.cuda.synchronize()
    for b in range(4):
        O, _, _, _ = _oracle_on(store, w, b)
        check_close(host(out[b]), O, f"fp8 wide peaked b={b}", max_abs=6e-2, mean_abs=6e-3)
    pc.close()


def test_stack_population_then_reuse_on_8_bit_slots():
    """The population pass cuts the prompt's K/V of every layer into 8-bit slots on the way; the reuse pass on the fresh
    rows reads them.  The oracle does the same with its own numbers: full pass in exact arithmetic, K/V of the chunks
    rounded to the storage dtype and put through its quantiser, reuse pass over what it reads back.  (The two sides'
    codes may differ where an element sits at a rounding border: the bar is the hidden-state bar of the bf16 stack.)"""
    from test_gpu_stack import EPS, check_hidden, dev_layers, oracle_block
    H, Hq, Hkv, D, F, C, n_c, Tf, L = 256, 4, 2, 64, 384, 64, 3, 40, 2
    total = n_c * C + Tf
    h0 = wl.round_bf16(np.random.default_rng(19).standard_normal((total, H)).astype(np.float32))
    Ws = [wl.stack_weights(19, l, H, Hq, Hkv, D, F) for l in range(L)]
    layers = dev_layers(Ws)
    pc = Percache(n_layers=L, hidden=H, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=D, n_slots=8, slot_capacity=C, max_pos=total,
                  kv_fp8=True, device=DEV)
    slots = [6, 1, 4]
    bounds = [c * C for c in range(n_c + 1)] + [total]
    pc.percache_stack_reuse(layers, F, EPS, bf16(h0[None]), save_bounds=bounds, save_slots=[slots + [-1]])
    reuse = pc.percache_stack_reuse(layers, F, EPS, bf16(h0[None, n_c * C:]), [slots])
    torch.cuda.synchronize()
    # oracle: layer by layer, the reuse pass's fresh rows over the quantised K/V of the full pass's chunk rows
    h_full, h_fresh = h0, h0[n_c * C:]
    for W in Ws:
        h_next, K, V = oracle_block(h_full, W, Hq, Hkv, D, 10000.0)
        sk = np.stack([kv_fp8.round_trip(wl.round_bf16(K[:, c * C:(c + 1) * C])) for c in range(n_c)])
        sv = np.stack([kv_fp8.round_trip(wl.round_bf16(V[:, c * C:(c + 1) * C])) for c in range(n_c)])
        h_fresh, _, _ = oracle_block(h_fresh, W, Hq, Hkv, D, 10000.0, sk, sv, np.arange(n_c, dtype=np.int32), [C] * n_c)
        h_full = h_next
    check_hidden(host(reuse[0]), h_fresh, "reuse pass over 8-bit slots vs oracle")
    # and the quantisation itself stays small against the exact stack
    check_hidden(host(reuse[0]), h_full[n_c * C:], "reuse pass over 8-bit slots vs exact full recompute", rel_max=2.0 ** -4, rel_fro=3e-2)
    pc.close()


@pytest.mark.parametrize("D", [64, 128])
def test_append_to_8_bit_slots_follows_the_oracles_rule(D):
    """Appends that start and end inside blocks and on block borders; later tokens larger (the open block's scale
    rises and its old codes are re-rounded) and smaller."""
    g = np.random.default_rng(11 + D)
    Hkv, C = 2, 256
    pc = _ctx(D, C, n_slots=2)
    mag = np.exp2(g.integers(-2, 5, (1, 250, 1))).astype(np.float32)
    k = wl.round_bf16(g.standard_normal((Hkv, 250, D)).astype(np.float32) * mag)
    v = wl.round_bf16(g.standard_normal((Hkv, 250, D)).astype(np.float32) * mag[:, ::-1])
    cuts = [0, 37, 38, 64, 65, 129, 192, 250]
    want_k = want_v = None
    for lo, hi in zip(cuts[:-1], cuts[1:]):
        if lo == 0:
            pc.percache_kv_put(0, 1, bf16(k[:, :hi]), bf16(v[:, :hi]))
            want_k, want_v = kv_fp8.round_trip(k[:, :hi]), kv_fp8.round_trip(v[:, :hi])
        else:
            pc.percache_kv_append(0, 1, bf16(k[:, lo:hi]), bf16(v[:, lo:hi]))
            want_k, want_v = kv_fp8.append(want_k, k[:, lo:hi]), kv_fp8.append(want_v, v[:, lo:hi])
        assert pc.percache_kv_len(0, 1) == hi
        kk, vv = pc.percache_kv_get(0, 1)
        torch.cuda.synchronize()
        assert np.array_equal(host(kk), want_k), f"K after the append to {hi}"
        assert np.array_equal(host(vv), want_v), f"V after the append to {hi}"
    with pytest.raises(PercacheError) as e:
        pc.percache_kv_append(0, 1, bf16(k[:, :7]), bf16(v[:, :7]))      # 250 + 7 > 256
    assert e.value.status == -4 and pc.percache_kv_len(0, 1) == 250
    pc.close()


def test_decode_steps_on_8_bit_slots():
    """Decoding steps whose sequence slot and reused chunks are 8-bit slots, against the oracle doing the same thing
    with its own numbers: per layer, the step's K/V (rounded to the storage dtype) appended by the oracle's append rule,
    attention over what its slots read back."""
    from test_gpu_stack import EPS, check_hidden, dev_layers, oracle_block
    H, Hq, Hkv, D, F, L, C = 256, 4, 2, 64, 384, 2, 64
    n_c, t_prompt, n_steps = 2, 20, 5
    Ws = [wl.stack_weights(33, l, H, Hq, Hkv, D, F) for l in range(L)]
    layers = dev_layers(Ws)
    pc = Percache(n_layers=L, hidden=H, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=D, n_slots=3, slot_capacity=C,
                  max_pos=n_c * C + C, kv_fp8=True, device=DEV)
    g = np.random.default_rng(44)
    total = n_c * C + t_prompt + n_steps
    seq = wl.round_bf16(g.standard_normal((total, H)).astype(np.float32))
    chunk_slots, seq_slot = [0, 1], 2
    bounds = [c * C for c in range(n_c + 1)] + [n_c * C + t_prompt]
    pc.percache_stack_reuse(layers, F, EPS, bf16(seq[None, :n_c * C + t_prompt]), save_bounds=bounds, save_slots=[chunk_slots + [seq_slot]])
    # oracle population: exact full pass; slots = quantised (bf16-rounded) K/V of every layer
    store = []      # per layer: list of read-back (k, v) for [chunk 0, chunk 1, sequence slot]
    h = seq[:n_c * C + t_prompt]
    for W in Ws:
        h, K, V = oracle_block(h, W, Hq, Hkv, D, 10000.0)
        cuts = list(zip(bounds[:-1], bounds[1:]))
        store.append([(kv_fp8.round_trip(wl.round_bf16(K[:, lo:hi])), kv_fp8.round_trip(wl.round_bf16(V[:, lo:hi]))) for lo, hi in cuts])
    for step in range(n_steps):
        pos = n_c * C + t_prompt + step
        out = pc.percache_stack_decode(layers, F, EPS, bf16(seq[None, pos:pos + 1]), [chunk_slots + [seq_slot]], [seq_slot])
        torch.cuda.synchronize()
        hx = seq[pos:pos + 1]
        for l, W in enumerate(Ws):
            used = [C, C, store[l][2][0].shape[1]]
            sk = np.zeros((3, Hkv, C, D), np.float32)
            sv = np.zeros((3, Hkv, C, D), np.float32)
            for i, (k_, v_) in enumerate(store[l]):
                sk[i, :, :k_.shape[1]] = k_
                sv[i, :, :v_.shape[1]] = v_
            hx, Kn, Vn = oracle_block(hx, W, Hq, Hkv, D, 10000.0, sk, sv, np.arange(3, dtype=np.int32), used)
            store[l][2] = (kv_fp8.append(store[l][2][0], wl.round_bf16(Kn)), kv_fp8.append(store[l][2][1], wl.round_bf16(Vn)))
        assert pc.percache_kv_len(L - 1, seq_slot) == t_prompt + step + 1
        check_hidden(host(out[0]), hx, f"decode step {step} over 8-bit slots vs oracle", rel_max=2.0 ** -5)
    pc.close()


@pytest.mark.parametrize("kv_fp8", [False, True])
def test_config4_decode_step_shape_full_size(kv_fp8):
    """One new token per query over the 16 x 1024 cached tokens of config 4 (batch 8), over bf16 and over 8-bit slots: the
    launch configurations of the benchmark's decode-step lines.  One row per query and head: the oracle computes all."""
    w = wl.config4(t_fresh=1)
    pc = Percache(n_layers=1, hidden=w.hidden, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim,
                  n_slots=w.n_slots, slot_capacity=w.chunk_tokens, max_pos=w.max_pos, kv_fp8=kv_fp8, device=DEV)
    store = {}
    for s in sorted(set(int(x) for x in w.slot_ids.reshape(-1))):
        k, v = w.slot_kv(s)
        pc.percache_kv_put(0, s, bf16(k), bf16(v))
        store[s] = (kv_fp8_mod.round_trip(k), kv_fp8_mod.round_trip(v)) if kv_fp8 else (k, v)
    out = pc.percache_prefill_reuse(0, bf16(w.X), bf16(w.Wqkv), w.slot_ids, w.used_len)
    torch.cuda.synchronize()
    for b in range(w.batch):
        O, _, _, _ = _oracle_on(store, w, b)
        check_close(host(out[b]), O, f"cfg4 decode shape kv_fp8={kv_fp8} b={b}")
    pc.close()
