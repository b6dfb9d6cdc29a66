"""GPU parity of the cache-reusing prefill (Sec. 4.2.2, App. B.1/B.2) against the CPU oracle, through the C ABI.

Bar for bf16 inputs, against the unrounded oracle: max-abs 2e-2 and mean-abs 2e-3, plus a relative Frobenius
bound of 1e-2 (the outputs of flat softmaxes are small, so the absolute bounds alone constrain little).
Integer/byte work (slot store round trip, slot permutation) is bit-exact.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2601_11553_amd import workloads as wl
from paper_2601_11553_amd.binding import PercacheError

from gpu_util import DEV, bf16, check_close, fill_slots, host, make_ctx

pytestmark = pytest.mark.gpu


def _oracle_query(w, b, X=None, samples=None):
    sk, sv, ids = w.compact_store(b)
    return oracle.prefill_reuse(w.X[b] if X is None else X, w.Wqkv, w.n_q_heads, w.n_kv_heads, w.head_dim,
                                w.rope_theta, sk, sv, ids, w.used_len[b], samples=samples)


def _run_and_check(w, tag, rel_fro=1e-2, max_abs=2e-2, mean_abs=2e-3):
    pc = make_ctx(w)
    fill_slots(pc, w, w.slot_ids.reshape(-1))
    kf = torch.empty((w.batch, w.n_kv_heads, w.t_fresh, w.head_dim), dtype=torch.bfloat16, device=DEV)
    vf = torch.empty_like(kf)
    out = pc.percache_prefill_reuse(0, bf16(w.X), bf16(w.Wqkv), w.slot_ids, w.used_len, k_fresh_out=kf, v_fresh_out=vf)
    torch.cuda.synchronize()
    for b in range(w.batch):
        O, Kf, Vf, _ = _oracle_query(w, b)
        check_close(host(out[b]), O, f"{tag} attn b={b}", rel_fro=rel_fro, max_abs=max_abs, mean_abs=mean_abs)
        check_close(host(kf[b]), Kf, f"{tag} k_fresh b={b}")
        check_close(host(vf[b]), Vf, f"{tag} v_fresh b={b}")
    pc.close()
    return out


# --------------------------------------------------------------------------- K/V store
def test_kv_store_round_trip_and_errors():
    w = wl.make_prefill("kv", 3, "bf16", 256, 4, 2, 64, 1, 16, 2, 128, 6)
    pc = make_ctx(w, n_layers=2)
    g = np.random.default_rng(1)
    for layer, slot, n in [(0, 0, 128), (1, 5, 1), (0, 3, 77)]:
        k = bf16(g.standard_normal((2, n, 64)).astype(np.float32))
        v = bf16(g.standard_normal((2, n, 64)).astype(np.float32))
        pc.percache_kv_put(layer, slot, k, v)
        assert pc.percache_kv_len(layer, slot) == n
        k2, v2 = pc.percache_kv_get(layer, slot)
        torch.cuda.synchronize()
        assert torch.equal(k, k2) and torch.equal(v, v2)
    assert pc.percache_kv_len(1, 0) == 0
    # several chunks in one launch, then read back one by one
    kb = bf16(g.standard_normal((3, 2, 70, 64)).astype(np.float32))
    vb = bf16(g.standard_normal((3, 2, 70, 64)).astype(np.float32))
    pc.percache_kv_put_batch(1, [4, 0, 2], kb, vb)
    for i, s in enumerate([4, 0, 2]):
        k2, v2 = pc.percache_kv_get(1, s)
        torch.cuda.synchronize()
        assert torch.equal(kb[i], k2) and torch.equal(vb[i], v2)
    with pytest.raises(PercacheError) as e:
        pc.percache_kv_put_batch(1, [1, 1], kb[:2], vb[:2])
    assert e.value.status == -1
    # ... and read back in one launch: whole chunks in another order with a repeat, then a shorter prefix of each
    order = [2, 4, 4, 0]
    kg, vg = pc.percache_kv_get_batch(1, order, 70)
    kp, vp = pc.percache_kv_get_batch(1, order, 33)
    torch.cuda.synchronize()
    src = {4: 0, 0: 1, 2: 2}
    for i, s in enumerate(order):
        assert torch.equal(kg[i], kb[src[s]]) and torch.equal(vg[i], vb[src[s]])
        assert torch.equal(kp[i], kb[src[s]][:, :33]) and torch.equal(vp[i], vb[src[s]][:, :33])
    with pytest.raises(PercacheError) as e:
        pc.percache_kv_get_batch(1, [2, 4], 71)               # more tokens than the slots hold
    assert e.value.status == -4
    with pytest.raises(PercacheError) as e:
        pc.percache_kv_get_batch(1, [2, 3], 10)               # slot 3 of layer 1 is empty
    assert e.value.status == -3
    pc.percache_kv_evict(1, 0)
    k = bf16(np.zeros((2, 129, 64), np.float32))
    for args, status in [((0, 6, k[:, :8], k[:, :8]), -3), ((2, 0, k[:, :8], k[:, :8]), -3), ((0, 1, k, k), -4)]:
        with pytest.raises(PercacheError) as e:
            pc.percache_kv_put(*args)
        assert e.value.status == status
    with pytest.raises(PercacheError) as e:
        pc.percache_kv_get(1, 0)
    assert e.value.status == -3
    pc.percache_kv_evict(0, 3)
    assert pc.percache_kv_len(0, 3) == 0
    # a prefill that names an empty slot, a bad slot, or too long a used length is refused before any launch
    x, wq = bf16(w.X), bf16(w.Wqkv)
    for ids, ul, status in [([[0, 3]], None, -3), ([[0, 9]], None, -3), ([[0, 0]], [[128, 129]], -4)]:
        with pytest.raises(PercacheError) as e:
            pc.percache_prefill_reuse(0, x, wq, ids, ul)
        assert e.value.status == status
    pc.close()


# --------------------------------------------------------------------------- projection + RoPE
@pytest.mark.parametrize("shape", [
    dict(hidden=256, n_q_heads=4, n_kv_heads=2, head_dim=64, batch=1, t_fresh=16, n_chunks=2, chunk_tokens=64, n_slots=4),
    dict(hidden=1024, n_q_heads=16, n_kv_heads=8, head_dim=128, batch=1, t_fresh=64, n_chunks=4, chunk_tokens=512, n_slots=16),
    dict(hidden=512, n_q_heads=6, n_kv_heads=2, head_dim=128, batch=3, t_fresh=50, n_chunks=2, chunk_tokens=64, n_slots=8),
    dict(hidden=320, n_q_heads=4, n_kv_heads=4, head_dim=64, batch=2, t_fresh=131, n_chunks=1, chunk_tokens=192, n_slots=3),
    # enough tiles that the launcher takes its 192-token tiles (more than two workgroups per CU otherwise), ragged last tile
    dict(hidden=256, n_q_heads=24, n_kv_heads=8, head_dim=128, batch=13, t_fresh=131, n_chunks=1, chunk_tokens=64, n_slots=16),
    dict(hidden=192, n_q_heads=48, n_kv_heads=16, head_dim=64, batch=7, t_fresh=250, n_chunks=1, chunk_tokens=64, n_slots=8),
    # the two-head tiles of 8 wavefronts with 7 x 7 and 4 x 6 tile grids (other strip widths of the XCD patches), 2 and 6 k-steps
    dict(hidden=128, n_q_heads=10, n_kv_heads=2, head_dim=128, batch=6, t_fresh=200, n_chunks=1, chunk_tokens=64, n_slots=8),
    dict(hidden=384, n_q_heads=4, n_kv_heads=2, head_dim=128, batch=9, t_fresh=128, n_chunks=2, chunk_tokens=64, n_slots=20),
])
def test_qkv_rope_matches_oracle(shape):
    w = wl.make_prefill("proj", 5, "bf16", last_used_len=shape["chunk_tokens"] - 3, **shape)
    pc = make_ctx(w)
    fill_slots(pc, w, w.slot_ids.reshape(-1))
    q, k, v = pc.percache_qkv_rope(0, bf16(w.X), bf16(w.Wqkv), w.slot_ids, w.used_len)
    torch.cuda.synchronize()
    for b in range(w.batch):
        Q, K, V = oracle.qkv_rope(w.X[b], w.Wqkv, w.n_q_heads, w.n_kv_heads, w.head_dim, int(w.l_pre[b]), w.rope_theta)
        check_close(host(q[b]), Q, f"q b={b}")
        check_close(host(k[b]), K, f"k b={b}")
        check_close(host(v[b]), V, f"v b={b}")
    pc.close()


# --------------------------------------------------------------------------- config 0 (tiny layer, D = 64)
def _config0_store():
    w = wl.config0("bf16")
    _, K, V, _ = oracle.prefill_reuse(w.prompt[: w.l_pre], w.Wqkv, w.n_q_heads, w.n_kv_heads, w.head_dim, w.rope_theta)
    return w, wl.round_bf16(K), wl.round_bf16(V)


@pytest.mark.parametrize("variant", ["2x64", "last60", "1x128"])
def test_config0_reuse(variant):
    """Cached K/V come from running the same layer on the chunk tokens (rounded to bf16 for the store)."""
    w, K, V = _config0_store()
    from paper_2601_11553_amd.binding import Percache
    C = 128 if variant == "1x128" else 64
    pc = Percache(n_layers=1, hidden=w.hidden, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim,
                  n_slots=4, slot_capacity=C, max_pos=256, rope_theta=w.rope_theta, device=DEV)
    if variant == "1x128":
        sk, sv = K[None, :, :128], V[None, :, :128]
        ids, used, fresh_from = [2], [128], 128
    else:
        sk = np.stack([K[:, :64], K[:, 64:128]])
        sv = np.stack([V[:, :64], V[:, 64:128]])
        ids, used, fresh_from = [3, 1], ([64, 64] if variant == "2x64" else [64, 60]), (128 if variant == "2x64" else 124)
    for c, s in enumerate(ids):
        pc.percache_kv_put(0, s, bf16(sk[c]), bf16(sv[c]))
    X = w.prompt[fresh_from:]
    out = pc.percache_prefill_reuse(0, bf16(X)[None], bf16(w.Wqkv), [ids], [used])
    torch.cuda.synchronize()
    ref, _, _, _ = oracle.prefill_reuse(X, w.Wqkv, w.n_q_heads, w.n_kv_heads, w.head_dim, w.rope_theta, sk, sv,
                                        list(range(len(ids))), used)
    check_close(host(out[0]), ref, f"cfg0 {variant}")
    # the reuse result is also the full recomputation of the contiguous prompt (fresh rows)
    full, _, _, _ = oracle.prefill_reuse(w.prompt, w.Wqkv, w.n_q_heads, w.n_kv_heads, w.head_dim, w.rope_theta)
    check_close(host(out[0]), full[fresh_from:], f"cfg0 {variant} vs full recompute")
    pc.close()


# --------------------------------------------------------------------------- config 1 and variations
def test_config1_full():
    _run_and_check(wl.config1(), "cfg1")


def test_ragged_batch_with_partial_and_empty_chunks():
    """Several tiles per chunk plus ragged tails; per-query chunk counts differ; one chunk contributes nothing."""
    w = wl.make_prefill("ragged", 7, "bf16", 512, 6, 2, 128, 3, 83, 3, 192, 12)
    w.used_len[0] = [192, 100, 1]
    w.used_len[1] = [65, 0, 190]
    w.used_len[2] = [7, 192, 64]
    _run_and_check(w, "ragged")
    # explicit n_chunks smaller than the list width
    pc = make_ctx(w)
    fill_slots(pc, w, w.slot_ids.reshape(-1))
    out = pc.percache_prefill_reuse(0, bf16(w.X), bf16(w.Wqkv), w.slot_ids, w.used_len, n_chunks=[3, 1, 0])
    torch.cuda.synchronize()
    for b, nc in enumerate([3, 1, 0]):
        sk, sv, ids = w.compact_store(b)
        O, _, _, _ = oracle.prefill_reuse(w.X[b], w.Wqkv, w.n_q_heads, w.n_kv_heads, w.head_dim, w.rope_theta, sk, sv,
                                          ids[:nc], w.used_len[b][:nc])
        check_close(host(out[b]), O, f"n_chunks={nc} b={b}")
    pc.close()


@pytest.mark.parametrize("seed", list(range(24)))
def test_seeded_random_shapes(seed):
    """Shapes drawn from a seed: head size, GQA ratio, batch, fresh length (1 .. a few tiles), chunk count (0 .. 5),
    chunk capacity, ragged used lengths (zero included), over bf16 slots, 8-bit slots and a store of both (against the
    oracle run on what each slot reads back)."""
    g = np.random.default_rng(1000 + seed)
    D = int(g.choice([64, 128]))
    Hkv = int(g.choice([1, 2, 3, 4]))
    G = int(g.choice([1, 2, 3, 4]))
    while ((G + 2) * Hkv * D) % 128:
        Hkv += 1
    batch = int(g.integers(1, 4))
    t_fresh = int(g.choice([1, 2, 17, 31, 64, 65, 100, 129, 150]))
    n_chunks = int(g.integers(0, 6))
    C = int(g.choice([64, 128, 192]))
    hidden = int(g.choice([128, 192, 256, 320]))
    w = wl.make_prefill(f"rnd{seed}", 2000 + seed, "bf16", hidden, G * Hkv, Hkv, D, batch, t_fresh, n_chunks, C, max(8, n_chunks + 2))
    if n_chunks:
        w.used_len[:] = g.integers(0, C + 1, size=(batch, n_chunks))
    mode = seed % 3                                   # 0: bf16 slots, 1: 8-bit slots, 2: the upper half of the slots 8-bit
    n16 = {0: w.n_slots, 1: 0, 2: w.n_slots // 2}[mode]
    pc = make_ctx(w, kv_fp8=mode == 1, n_slots_8bit=w.n_slots - n16 if mode == 2 else 0)
    fill_slots(pc, w, w.slot_ids.reshape(-1))
    out = pc.percache_prefill_reuse(0, bf16(w.X), bf16(w.Wqkv), w.slot_ids if n_chunks else None, w.used_len if n_chunks else None)
    torch.cuda.synchronize()
    from oracle import kv_fp8
    for b in range(batch):
        sk, sv, ids = w.compact_store(b)
        if n_chunks:   # what each chunk's slot reads back
            is8 = [int(s_) >= n16 for s_ in w.slot_ids[b]]
            sk = np.stack([kv_fp8.round_trip(wl.round_bf16(x)) if e else x for x, e in zip(sk, is8)])
            sv = np.stack([kv_fp8.round_trip(wl.round_bf16(x)) if e else x for x, e in zip(sv, is8)])
        O, _, _, _ = oracle.prefill_reuse(w.X[b], w.Wqkv, w.n_q_heads, w.n_kv_heads, w.head_dim, w.rope_theta, sk, sv, ids, w.used_len[b])
        check_close(host(out[b]), O, f"seed {seed} (D={D} G={G} Hkv={Hkv} B={batch} T={t_fresh} chunks={n_chunks}x{C} slots mode {mode}) b={b}")
    pc.close()


@pytest.mark.parametrize("n_splits", [0, 1, 5])
def test_long_chunk_lists(n_splits):
    """70 and 64 short chunks per query (the kernel keeps the first 64 list entries in registers and reads the
    rest from memory), unused chunks before, at and after the 64th, ragged lengths; key-axis partitions that start
    inside either part of the list."""
    n_c, C = 70, 64
    w = wl.make_prefill("long_list", 17, "bf16", 256, 4, 2, 64, 2, 40, n_c, C, 80)
    g = np.random.default_rng(5)
    w.used_len[:] = g.integers(1, C + 1, size=(2, n_c))
    w.used_len[0, [0, 5, 62, 63, 64, 69]] = 0
    w.used_len[1, [63, 65, 66]] = 0
    pc = make_ctx(w)
    fill_slots(pc, w, w.slot_ids.reshape(-1))
    X, W = bf16(w.X), bf16(w.Wqkv)
    q, kf, vf = pc.percache_qkv_rope(0, X, W, w.slot_ids, w.used_len, n_chunks=[70, 64])
    out = pc.percache_attention_reuse(0, q, kf, vf, w.slot_ids, w.used_len, n_chunks=[70, 64], n_splits=n_splits)
    torch.cuda.synchronize()
    for b, nc in enumerate([70, 64]):
        sk, sv, ids = w.compact_store(b)
        O, _, _, _ = oracle.prefill_reuse(w.X[b], w.Wqkv, w.n_q_heads, w.n_kv_heads, w.head_dim, w.rope_theta, sk, sv,
                                          ids[:nc], w.used_len[b][:nc])
        check_close(host(out[b]), O, f"long list splits={n_splits} b={b}")
    pc.close()


@pytest.mark.parametrize("t_fresh,n_splits,head_dim", [(70, 0, 128), (70, 1, 128), (70, 3, 128), (100, 0, 128), (100, 4, 128),
                                                       (256, 2, 128), (70, 0, 64), (100, 3, 64), (192, 1, 64)])
def test_long_context_kernel_on_ragged_lists(t_fresh, n_splits, head_dim):
    """The launch shape that takes the 8-wavefront long-context kernel (head size 128, 64 batch x kv-head groups,
    more than 128 stacked rows per group), on everything its chunk walk has to get right: chunks that end inside a
    tile, chunks of one key, unused chunks at the start, in the middle and at the end of a list, a query without
    chunks, a fresh length that is no multiple of the tile, a last workgroup with rows to spare (3 x 70 = 210 of 256,
    3 x 100 = 300 of 512), row blocks that straddle two query heads, and key-axis partitions that begin inside a chunk,
    at a chunk boundary and in the fresh part."""
    n_c, C = 6, 192
    if head_dim == 128:
        w = wl.make_prefill("wide_ragged", 31, "bf16", 256, 24, 8, 128, 8, t_fresh, n_c, C, 20)
    else:   # 0.5B-shaped heads (7 query heads per kv head), 16 queries x 2 kv heads x at least 2 row blocks
        w = wl.make_prefill("wide_ragged64", 32, "bf16", 128, 14, 2, 64, 16, t_fresh, n_c, C, 24)
    g = np.random.default_rng(9)
    w.used_len[:] = g.integers(1, C + 1, size=(w.batch, n_c))
    w.used_len[0] = [192, 192, 192, 192, 192, 192]
    w.used_len[1] = [0, 65, 0, 1, 128, 0]
    w.used_len[2] = [1, 1, 1, 1, 1, 1]
    w.used_len[3] = [0, 0, 0, 0, 0, 0]
    w.used_len[4] = [191, 64, 63, 0, 0, 129]
    n_chunks = [6, 6, 6, 6, 6, 3, 0, 1] + [int(x) for x in g.integers(0, n_c + 1, size=w.batch - 8)]
    pc = make_ctx(w)
    fill_slots(pc, w, w.slot_ids.reshape(-1))
    X, W = bf16(w.X), bf16(w.Wqkv)
    q, kf, vf = pc.percache_qkv_rope(0, X, W, w.slot_ids, w.used_len, n_chunks=n_chunks)
    out = pc.percache_attention_reuse(0, q, kf, vf, w.slot_ids, w.used_len, n_chunks=n_chunks, n_splits=n_splits)
    torch.cuda.synchronize()
    for b, nc in enumerate(n_chunks):
        sk, sv, ids = w.compact_store(b)
        O, _, _, _ = oracle.prefill_reuse(w.X[b], w.Wqkv, w.n_q_heads, w.n_kv_heads, w.head_dim, w.rope_theta, sk, sv,
                                          ids[:nc], w.used_len[b][:nc])
        check_close(host(out[b]), O, f"long-context kernel T={t_fresh} splits={n_splits} b={b} chunks={list(w.used_len[b][:nc])}")
    pc.close()


@pytest.mark.parametrize("t_fresh,n_splits,n16", [(70, 0, 0), (100, 3, 0), (256, 1, 0), (70, 2, 3), (192, 0, 3)])
def test_long_context_kernel_over_8bit_slots(t_fresh, n_splits, n16):
    """The long-context launch shape over 8-bit slots: every chunk of the call in an 8-bit slot (a store of 8-bit slots
    only, and one whose first three slots are bf16 slots that the call does not name, so slot ids are offset), ragged and
    unused chunks, ranges that begin inside a chunk (the chunk's scales are picked by the tile's place in it), fresh
    tiles in bf16.  Reference: the oracle on what each slot reads back."""
    from oracle import kv_fp8
    n_c, C = 6, 192
    w = wl.make_prefill("wide_8bit", 51, "bf16", 256, 24, 8, 128, 8, t_fresh, n_c, C, 20)
    if n16:
        w.slot_ids[:] = n16 + w.slot_ids % (w.n_slots - n16)
    g = np.random.default_rng(13)
    w.used_len[:] = g.integers(1, C + 1, size=(8, n_c))
    w.used_len[1] = [0, 65, 0, 1, 128, 0]
    w.used_len[2] = [1, 1, 1, 1, 1, 1]
    w.used_len[3] = 0
    w.used_len[4] = [191, 64, 63, 0, 0, 129]
    n_chunks = [6, 6, 6, 6, 6, 3, 0, 1]
    pc = make_ctx(w, kv_fp8=n16 == 0, n_slots_8bit=w.n_slots - n16 if n16 else 0)
    fill_slots(pc, w, w.slot_ids.reshape(-1))
    X, W = bf16(w.X), bf16(w.Wqkv)
    q, kf, vf = pc.percache_qkv_rope(0, X, W, w.slot_ids, w.used_len, n_chunks=n_chunks)
    out = pc.percache_attention_reuse(0, q, kf, vf, w.slot_ids, w.used_len, n_chunks=n_chunks, n_splits=n_splits).clone()
    again = pc.percache_attention_reuse(0, q, kf, vf, w.slot_ids, w.used_len, n_chunks=n_chunks, n_splits=n_splits)
    torch.cuda.synchronize()
    assert torch.equal(out, again), "the same call twice gives other bits"
    for b, nc in enumerate(n_chunks):
        sk, sv, ids = w.compact_store(b)
        sk = np.stack([kv_fp8.round_trip(wl.round_bf16(x)) for x in sk]) if len(sk) else sk
        sv = np.stack([kv_fp8.round_trip(wl.round_bf16(x)) for x in sv]) if len(sv) else sv
        O, _, _, _ = oracle.prefill_reuse(w.X[b], w.Wqkv, w.n_q_heads, w.n_kv_heads, w.head_dim, w.rope_theta, sk, sv,
                                          ids[:nc], w.used_len[b][:nc])
        check_close(host(out[b]), O, f"long-context kernel, 8-bit slots, T={t_fresh} splits={n_splits} first 8-bit slot {n16} b={b}")
    pc.close()


@pytest.mark.parametrize("n_c,n_splits", [(64, 0), (64, 4), (40, 1), (66, 0)])
def test_long_context_kernel_on_full_width_lists(n_c, n_splits):
    """The same kernel with as many chunks as its register-held list takes (64) and with 40: one-tile chunks of ragged
    length, unused ones at both ends and in runs, per-query counts from none to all.  66 entries: the same launch shape
    falls back to the general 8-wavefront kernel, which reads entries past the 64th from memory."""
    C = 64
    w = wl.make_prefill("wide_lists", 41, "bf16", 256, 24, 8, 128, 8, 70, n_c, C, n_c + 8)
    g = np.random.default_rng(11)
    w.used_len[:] = g.integers(0, C + 1, size=(8, n_c))
    w.used_len[0, :3] = 0
    w.used_len[0, -2:] = 0
    w.used_len[1, 10:30] = 0
    w.used_len[2] = C
    n_chunks = [n_c, n_c, n_c, n_c - 1, 33 if n_c >= 33 else n_c, 1, 0, n_c]
    pc = make_ctx(w)
    fill_slots(pc, w, w.slot_ids.reshape(-1))
    X, W = bf16(w.X), bf16(w.Wqkv)
    q, kf, vf = pc.percache_qkv_rope(0, X, W, w.slot_ids, w.used_len, n_chunks=n_chunks)
    out = pc.percache_attention_reuse(0, q, kf, vf, w.slot_ids, w.used_len, n_chunks=n_chunks, n_splits=n_splits)
    torch.cuda.synchronize()
    for b, nc in enumerate(n_chunks):
        sk, sv, ids = w.compact_store(b)
        O, _, _, _ = oracle.prefill_reuse(w.X[b], w.Wqkv, w.n_q_heads, w.n_kv_heads, w.head_dim, w.rope_theta, sk, sv,
                                          ids[:nc], w.used_len[b][:nc])
        check_close(host(out[b]), O, f"long-context kernel, {n_c}-entry lists, splits={n_splits} b={b}")
    pc.close()


@pytest.mark.parametrize("head_dim,t_fresh", [(64, 320), (128, 320), (64, 300)])
def test_large_projection_tiles_lay_out_fresh_v_themselves(head_dim, t_fresh):
    """More token rows than the few-row kernels take: the large projection tiles write V token-major and, when the
    fresh length is a multiple of 64, as the 64-key blocks the attention kernel reads (no repack launch); a length
    that is not takes the repack kernel.  Both must give the oracle's attention output and fresh K/V."""
    hq, hkv = (8, 2) if head_dim == 64 else (6, 2)
    w = wl.make_prefill("v_blocks", 77, "bf16", 256, hq, hkv, head_dim, 2, t_fresh, 2, 128, 6)
    w.used_len[0] = [128, 70]
    w.used_len[1] = [1, 128]
    _run_and_check(w, f"v blocks D={head_dim} T={t_fresh}")


def test_kernel_timing_switch_selects_kernel_kinds():
    """The per-kernel event pairs: all kinds, a selection of kinds, off; a value outside the mask is refused."""
    from paper_2601_11553_amd import binding
    from paper_2601_11553_amd.binding import PercacheError
    w = wl.config1()
    pc = make_ctx(w)
    fill_slots(pc, w, w.slot_ids.reshape(-1))
    call = lambda: pc.percache_prefill_reuse(0, bf16(w.X), bf16(w.Wqkv), w.slot_ids, w.used_len)
    counts = lambda: [pc.percache_profile_read(k)[1] for k in (binding.KERNEL_LOOKUP, binding.KERNEL_QKV_ROPE, binding.KERNEL_ATTENTION)]
    pc.percache_profile_enable(True)
    call(); call()
    ms_attn, n_attn = pc.percache_profile_read(binding.KERNEL_ATTENTION)
    assert n_attn == 2 and 0.0 < ms_attn < 50.0
    assert counts() == [0, 2, 0]          # (the read above cleared the attention record)
    pc.percache_profile_enable(True, kernels=[binding.KERNEL_ATTENTION])
    call()
    assert counts() == [0, 0, 1]
    pc.percache_profile_enable(True, kernels=[binding.KERNEL_QKV_ROPE, binding.KERNEL_LOOKUP])
    call()
    assert counts() == [0, 1, 0]
    pc.percache_profile_enable(False)
    call()
    assert counts() == [0, 0, 0]
    with pytest.raises(PercacheError):
        pc._check(pc.lib.percache_profile_enable(pc.ctx, 16))
    pc.close()


def test_full_recompute_path_is_plain_causal_prefill():
    w = wl.make_prefill("causal", 8, "bf16", 256, 4, 2, 64, 2, 200, 0, 64, 1)
    pc = make_ctx(w, max_pos=256)
    out = pc.percache_prefill_reuse(0, bf16(w.X), bf16(w.Wqkv))
    torch.cuda.synchronize()
    for b in range(2):
        O, _, _, _ = oracle.prefill_reuse(w.X[b], w.Wqkv, w.n_q_heads, w.n_kv_heads, w.head_dim, w.rope_theta)
        check_close(host(out[b]), O, f"causal b={b}")
    pc.close()


def _oracle_qkv_bf16(w, b=0):
    """Oracle projection + RoPE of query b, rounded to the bf16 storage dtype: inputs for attention-only tests."""
    Q, K, V = oracle.qkv_rope(w.X[b], w.Wqkv, w.n_q_heads, w.n_kv_heads, w.head_dim, int(w.l_pre[b]), w.rope_theta)
    return wl.round_bf16(Q), wl.round_bf16(K), wl.round_bf16(V)


def test_peaked_softmax_stress():
    """Hidden states scaled x16 so that scores have a standard deviation of 10 and more (fresh-fresh scores reach
    +-100): mistakes in the running max / sum / rescale become O(1) errors.  At this scale the rounding of q and
    k to bf16 alone moves scores by ~0.4, so the attention step is tested on its own from the oracle's q, k, v
    rounded to bf16 (both sides get the same tensors); what remains is the rounding of probabilities to bf16."""
    w = wl.config1(x_scale=16.0, seed=21)
    pc = make_ctx(w)
    fill_slots(pc, w, w.slot_ids.reshape(-1))
    Q, K, V = _oracle_qkv_bf16(w)
    sk, sv, ids = w.compact_store(0)
    ref = oracle.attention_reuse(Q, K, V, sk, sv, ids, w.used_len[0])
    for ns in (1, 5):
        out = pc.percache_attention_reuse(0, bf16(Q)[None], bf16(K)[None], bf16(V)[None], w.slot_ids, w.used_len, n_splits=ns)
        torch.cuda.synchronize()
        check_close(host(out[0]), ref, f"peaked splits={ns}", max_abs=0.5, mean_abs=2e-2, rel_fro=6e-3)
    pc.close()


def test_split_count_and_slot_placement_do_not_change_results():
    w = wl.config1(seed=9, t_fresh=48)
    pc = make_ctx(w)
    kv = fill_slots(pc, w, w.slot_ids.reshape(-1))
    Qo, Ko, Vo = _oracle_qkv_bf16(w)
    q, k, v = bf16(Qo)[None], bf16(Ko)[None], bf16(Vo)[None]
    outs = {}
    for ns in (1, 2, 3, 8, 33):
        outs[ns] = pc.percache_attention_reuse(0, q, k, v, w.slot_ids, w.used_len, n_splits=ns).clone()
    auto = pc.percache_attention_reuse(0, q, k, v, w.slot_ids, w.used_len).clone()
    torch.cuda.synchronize()
    sk, sv, ids = w.compact_store(0)
    ref = oracle.attention_reuse(Qo, Ko, Vo, sk, sv, ids, w.used_len[0])
    for ns, o in outs.items():
        check_close(host(o[0]), ref, f"splits={ns}", max_abs=4e-3, mean_abs=4e-4, rel_fro=4e-3)
        assert (o.float() - outs[1].float()).abs().max().item() < 2e-3
    check_close(host(auto[0]), ref, "splits=auto", max_abs=4e-3, mean_abs=4e-4, rel_fro=4e-3)
    # same chunks placed in other slots and addressed by the permuted list: bit-identical output
    perm = [int(s) for s in w.slot_ids[0]]
    free = [s for s in range(w.n_slots) if s not in perm][: len(perm)]
    for old, new in zip(perm, free):
        pc.percache_kv_put(0, new, bf16(kv[old][0]), bf16(kv[old][1]))
    moved = pc.percache_attention_reuse(0, q, k, v, [free], w.used_len, n_splits=3)
    torch.cuda.synchronize()
    assert torch.equal(moved, outs[3])
    with pytest.raises(PercacheError):
        pc.percache_attention_reuse(0, q, k, v, w.slot_ids, w.used_len, n_splits=65)
    pc.close()


def test_gpu_full_prefill_populates_store_then_reuse_matches():
    """The GPU's own full prefill of a prompt, sliced into slots through kv_put (the cache slicer), then a
    reuse prefill of the suffix: the suffix rows must agree with the full pass."""
    H, Hq, Hkv, D, C, n_c, Tf = 512, 8, 4, 128, 128, 3, 40
    w = wl.make_prefill("self", 13, "bf16", H, Hq, Hkv, D, 1, C * n_c + Tf, 0, C, 4)
    pc = make_ctx(w, max_pos=512)
    x, wq = bf16(w.X), bf16(w.Wqkv)
    kf = torch.empty((1, Hkv, C * n_c + Tf, D), dtype=torch.bfloat16, device=DEV)
    vf = torch.empty_like(kf)
    full = pc.percache_prefill_reuse(0, x, wq, k_fresh_out=kf, v_fresh_out=vf).clone()
    for c in range(n_c):
        pc.percache_kv_put(0, c + 1, kf[0, :, c * C:(c + 1) * C].contiguous(), vf[0, :, c * C:(c + 1) * C].contiguous())
    reuse = pc.percache_prefill_reuse(0, x[:, C * n_c:].contiguous(), wq, [[1, 2, 3]])
    torch.cuda.synchronize()
    check_close(host(reuse[0]), host(full[0, C * n_c:]), "gpu reuse vs gpu full", max_abs=8e-3, mean_abs=8e-4, rel_fro=8e-3)
    O, _, _, _ = oracle.prefill_reuse(w.X[0], w.Wqkv, Hq, Hkv, D, w.rope_theta)
    check_close(host(full[0]), O, "gpu full vs oracle full")
    pc.close()


# --------------------------------------------------------------------------- config 4 shape
def test_config4_reduced():
    """The 3B-shaped GQA layer (G = 3, hidden 3072) at reduced batch / chunk count; full oracle check."""
    _run_and_check(wl.config4(batch=2, n_chunks=3, n_slots=8, t_fresh=256), "cfg4-reduced")


def test_repeated_calls_are_bit_identical():
    """No atomics, no order that depends on timing: the same call gives the same bits (split-KV merge included)."""
    w = wl.config4(batch=2, n_chunks=5, n_slots=12, t_fresh=200)
    pc = make_ctx(w)
    fill_slots(pc, w, w.slot_ids.reshape(-1))
    x, wq = bf16(w.X), bf16(w.Wqkv)
    first = pc.percache_prefill_reuse(0, x, wq, w.slot_ids, w.used_len).clone()
    for _ in range(3):
        again = pc.percache_prefill_reuse(0, x, wq, w.slot_ids, w.used_len)
        torch.cuda.synchronize()
        assert torch.equal(first, again)
    pc.close()


def test_config4_full_size_one_query_in_full_and_sampled_rows():
    """Full config 4 (batch 8, 16 x 1024 cached tokens, 256 fresh) in the launch configuration the benchmark
    times.  The oracle computes query 0 completely (all 256 rows x 24 heads, and its fresh K/V) and 70 sampled
    (query, row, head) outputs of the other seven queries, first and last row included."""
    w = wl.config4()
    pc = make_ctx(w)
    fill_slots(pc, w, w.slot_ids.reshape(-1))
    kf = torch.empty((w.batch, w.n_kv_heads, w.t_fresh, w.head_dim), dtype=torch.bfloat16, device=DEV)
    vf = torch.empty_like(kf)
    out = pc.percache_prefill_reuse(0, bf16(w.X), bf16(w.Wqkv), w.slot_ids, w.used_len, k_fresh_out=kf, v_fresh_out=vf)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all().item()
    O, Kf, Vf, _ = _oracle_query(w, 0)
    check_close(host(out[0]), O, "cfg4 query 0, every row and head")
    check_close(host(kf[0]), Kf, "cfg4 k_fresh b=0")
    check_close(host(vf[0]), Vf, "cfg4 v_fresh b=0")
    g = np.random.default_rng(4)
    out_h = host(out).reshape(w.batch, w.t_fresh, w.n_q_heads, w.head_dim)
    got, ref = [], []
    for b in range(1, w.batch):
        rows = g.integers(0, w.t_fresh, 10)
        heads = g.integers(0, w.n_q_heads, 10)
        rows[0], rows[1] = 0, w.t_fresh - 1
        O, _, _, _ = _oracle_query(w, b, samples=(rows, heads))
        got.append(np.stack([out_h[b, i, h] for i, h in zip(rows, heads)]))
        ref.append(O)
        print(f"cfg4 b={b} sampled", flush=True)
    check_close(np.concatenate(got), np.concatenate(ref), "cfg4 sampled rows of queries 1..7")
    pc.close()


def test_peaked_softmax_through_the_fused_path():
    """A peaked case through projection + RoPE + attention in one call (hidden states x4: scores up to about +-30).
    The GPU rounds q and k to bf16 once (relative error at most 2^-9 per element), the oracle does not, so a score
    moves by at most  eps_s(i, j) = (2 * 2^-9 + 2^-18) * sum_d |q_id k_jd| / sqrt(D).  With delta_i the largest
    eps_s of row i, every probability changes by a factor within [e^-2delta, e^2delta], the l1 distance of the two
    probability rows is at most e^(2 delta) - 1, and because both rows sum to one
        |o'_i - o_i| <= (e^(2 delta_i) - 1 + 2^-8) * max_j |v_j - o_i|      (2^-8: bf16 rounding of p and of v)
    element by element.  The bound is computed here from the oracle's own q, k, v, o; a mistake in the running
    maximum, the rescale or the row sum shows as an error of the size of |v| itself.  That bound is a worst case
    (every rounding error aligned); the typical score error is |score| 2^-9 sqrt(2), so on average over the output
    the error must also stay below (max|score| 2^-9 sqrt(2) + 2^-8) times the mean spread."""
    w = wl.config1(x_scale=4.0, seed=23, t_fresh=96)
    pc = make_ctx(w)
    fill_slots(pc, w, w.slot_ids.reshape(-1))
    out = host(pc.percache_prefill_reuse(0, bf16(w.X), bf16(w.Wqkv), w.slot_ids, w.used_len)[0])
    torch.cuda.synchronize()
    sk, sv, ids = w.compact_store(0)
    O, Kf, Vf, Q = oracle.prefill_reuse(w.X[0], w.Wqkv, w.n_q_heads, w.n_kv_heads, w.head_dim, w.rope_theta, sk, sv, ids, w.used_len[0])
    D, T, G = w.head_dim, w.t_fresh, w.n_q_heads // w.n_kv_heads
    worst_ratio, peak_score, err_sum, spread_sum, n_el = 0.0, 0.0, 0.0, 0.0, 0
    for h in range(w.n_q_heads):
        kv = h // G
        K_all = np.concatenate([sk[c, kv, :u] for c, u in zip(ids, w.used_len[0])] + [Kf[kv]]).astype(np.float64)
        V_all = np.concatenate([sv[c, kv, :u] for c, u in zip(ids, w.used_len[0])] + [Vf[kv]]).astype(np.float64)
        n_cached = K_all.shape[0] - T
        q = Q[h].astype(np.float64)
        eps_s = (2 * 2.0 ** -9 + 2.0 ** -18) * (np.abs(q) @ np.abs(K_all).T) / np.sqrt(D)
        vis = np.arange(K_all.shape[0])[None, :] < (n_cached + 1 + np.arange(T))[:, None]
        peak_score = max(peak_score, float(np.abs((q @ K_all.T) / np.sqrt(D))[vis].max()))
        delta = np.where(vis, eps_s, 0.0).max(axis=1)
        o = O[:, h * D:(h + 1) * D].astype(np.float64)
        for i in range(T):
            spread = np.abs(V_all[: n_cached + i + 1] - o[i]).max(axis=0)             # per output element
            bound = (np.expm1(2 * delta[i]) + 2.0 ** -8) * spread + 1e-6
            err = np.abs(out[i, h * D:(h + 1) * D] - o[i])
            worst_ratio = max(worst_ratio, float((err / bound).max()))
            err_sum += float(err.sum())
            spread_sum += float(spread.sum())
            n_el += D
    fro = np.linalg.norm(out - O) / np.linalg.norm(O)
    typical = (peak_score * 2.0 ** -9 * np.sqrt(2.0) + 2.0 ** -8) * spread_sum / n_el
    print(f"peaked fused path: largest |score| {peak_score:.1f}, worst error / bound {worst_ratio:.3f}, mean-abs error "
          f"{err_sum / n_el:.3e} (typical-error bar {typical:.3e}), rel-fro {fro:.3e}", flush=True)
    assert peak_score > 15.0 and worst_ratio <= 1.0 and err_sum / n_el <= typical
    pc.close()


def test_probabilities_far_above_the_reference_exponent():
    """The reference exponent of a row is refreshed only when the SUM of a lane's 32 probabilities of a tile exceeds
    32 * 2^8, so a single probability can reach 2^13 against a stale reference.  Rows whose first tile has scores 0
    meet, tiles later, one key whose score is 9 .. 12.9 log2 units higher (everything else stays at 0): no refresh
    happens, the probability is carried as a bf16 value up to 2^12.9, and the result must still match."""
    D, C, T = 128, 256, 40
    w = wl.make_prefill("hot", 31, "bf16", 256, 2, 1, D, 1, T, 1, C, 2)
    pc = make_ctx(w)
    g = np.random.default_rng(3)
    k = np.zeros((1, C, D), np.float32)
    v = wl.round_bf16(g.standard_normal((1, C, D)).astype(np.float32))
    hot = [64 + 7, 128 + 40, 192 + 63]
    k[0, hot, 0] = 1.0
    pc.percache_kv_put(0, 1, bf16(k), bf16(v))
    # q = a e_0: score of a hot key = a / sqrt(D), in log2 units a log2(e) / sqrt(D) = 9 .. 12.9 over the rows
    lifts = np.linspace(9.0, 12.9, T)
    Q = np.zeros((2, T, D), np.float32)
    Q[:, :, 0] = wl.round_bf16((lifts * np.sqrt(D) / np.log2(np.e)).astype(np.float32))[None, :]
    Kf = np.zeros((1, T, D), np.float32)
    Vf = wl.round_bf16(g.standard_normal((1, T, D)).astype(np.float32))
    out = pc.percache_attention_reuse(0, bf16(Q)[None], bf16(Kf)[None], bf16(Vf)[None], [[1]], n_splits=1)
    torch.cuda.synchronize()
    ref = oracle.attention_reuse(Q, Kf, Vf, k[None], v[None], [0], [C])
    check_close(host(out[0]), ref, "probabilities up to 2^12.9 against a stale reference", max_abs=2e-2, mean_abs=2e-3, rel_fro=6e-3)
    pc.close()
