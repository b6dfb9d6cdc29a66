"""GPU parity of the layer stack on the retained rows (App. B.1) and of the cache slicer (Sec. 4.1.1), through the C ABI.

Hidden states are O(1) and are stored in bf16 between the steps of a block, so the attention tolerance (absolute
2e-2) does not apply to them; the bar for hidden states is relative: max-abs error <= 2^-6 of the largest reference
magnitude (a few bf16 roundings of 2^-9 each per layer) and relative Frobenius error <= 1e-2.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2601_11553_amd import workloads as wl
from paper_2601_11553_amd.binding import Percache, PercacheError

from gpu_util import DEV, bf16, host

pytestmark = pytest.mark.gpu
EPS = 1e-6


def check_hidden(got, ref, what, rel_max=2.0 ** -6, rel_fro=1e-2):
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape and np.isfinite(got).all(), what
    err = np.abs(got - ref)
    fro = np.linalg.norm(got - ref) / np.linalg.norm(ref)
    msg = f"{what}: max-abs {err.max():.3e} (|ref| max {np.abs(ref).max():.3e}) rel-fro {fro:.3e}"
    print(msg, flush=True)
    assert err.max() <= rel_max * np.abs(ref).max() and fro <= rel_fro, msg


def dev_layers(Ws):
    return [dict(gain1=bf16(W.gain1), wqkv=bf16(W.Wqkv), wo=bf16(W.Wo), gain2=bf16(W.gain2), w_gate=bf16(W.Wgate),
                 w_up=bf16(W.Wup), w_down=bf16(W.Wdown)) for W in Ws]


def oracle_block(h, W, Hq, Hkv, D, theta, sk=None, sv=None, ids=(), used=(), extras=None):
    return oracle.block(h, W.gain1, W.Wqkv, Hq, Hkv, D, theta, W.Wo, W.gain2, W.Wgate, W.Wup, W.Wdown, EPS, sk, sv, ids, used,
                        extras=extras)


@pytest.mark.parametrize("D,t_fresh,used_last", [(64, 48, 64), (128, 70, 40), (128, 200, 64), (64, 64, 64), (128, 64, 33)])
def test_one_block_vs_oracle(D, t_fresh, used_last):
    """One block over two loaded chunks (random K/V) + a ragged fresh part, against the oracle's block."""
    H, Hq, Hkv, F, C = 256, 4, 2, 448, 64
    w = wl.make_prefill("blk", 21, "bf16", H, Hq, Hkv, D, 2, t_fresh, 2, C, 6, last_used_len=used_last)
    Ws = [wl.stack_weights(21, 0, H, Hq, Hkv, D, F)]
    pc = Percache(n_layers=1, hidden=H, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=D, n_slots=6, slot_capacity=C,
                  max_pos=w.max_pos, device=DEV)
    for s in sorted(set(int(x) for x in w.slot_ids.reshape(-1))):
        k, v = w.slot_kv(s)
        pc.percache_kv_put(0, s, bf16(k), bf16(v))
    h_out = pc.percache_stack_reuse(dev_layers(Ws), F, EPS, bf16(w.X), w.slot_ids, w.used_len)
    torch.cuda.synchronize()
    for b in range(2):
        sk, sv, ids = w.compact_store(b)
        ref, _, _ = oracle_block(w.X[b], Ws[0], Hq, Hkv, D, w.rope_theta, sk, sv, ids, w.used_len[b])
        check_hidden(host(h_out[b]), ref, f"block D={D} T={t_fresh} query {b}")


@pytest.mark.parametrize("seed", list(range(16)))
def test_seeded_random_block_shapes(seed):
    """One block with every size drawn from a seed: the token-row count decides which projection kernels run (slices
    of the contraction, the one-pass kernels for few rows, the 64/128-token tiles), the rest varies head size, GQA
    ratio, widths, chunk lists and the projection variants."""
    g = np.random.default_rng(4000 + seed)
    D = int(g.choice([64, 128]))
    Hkv = int(g.choice([1, 2, 4]))
    G = int(g.choice([1, 2, 4]))
    while ((G + 2) * Hkv * D) % 128:
        Hkv += 1
    Hq = G * Hkv
    H = int(g.choice([128, 256, 384]))
    F = int(g.choice([64, 192, 448, 640]))
    batch = int(g.integers(1, 4))
    t_fresh = int(g.choice([1, 3, 20, 33, 64, 70, 100, 130]))
    n_chunks = int(g.integers(0, 4))
    C = int(g.choice([64, 128]))
    w = wl.make_prefill(f"blk{seed}", 4100 + seed, "bf16", H, Hq, Hkv, D, batch, t_fresh, n_chunks, C, 6)
    if n_chunks:
        w.used_len[:] = g.integers(1, C + 1, size=(batch, n_chunks))
    W = wl.stack_weights(4100 + seed, 0, H, Hq, Hkv, D, F)
    layer = dev_layers([W])[0]
    extras = None
    if seed % 3 == 0:
        n_out = (Hq + 2 * Hkv) * D
        bias = wl.round_bf16(0.5 * g.standard_normal(n_out).astype(np.float32))
        qg = wl.round_bf16(1 + 0.2 * g.standard_normal(D).astype(np.float32))
        kg = wl.round_bf16(1 + 0.2 * g.standard_normal(D).astype(np.float32))
        layer.update(qkv_bias=bf16(bias), q_norm=bf16(qg), k_norm=bf16(kg))
        extras = dict(bias=bias, q_gain=qg, k_gain=kg, eps=EPS)
    pc = Percache(n_layers=1, hidden=H, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=D, n_slots=6, slot_capacity=C,
                  max_pos=w.max_pos, device=DEV)
    for s_ in sorted(set(int(x) for x in w.slot_ids.reshape(-1))):
        k, v = w.slot_kv(s_)
        pc.percache_kv_put(0, s_, bf16(k), bf16(v))
    h_out = pc.percache_stack_reuse([layer], F, EPS, bf16(w.X), w.slot_ids if n_chunks else None, w.used_len if n_chunks else None)
    torch.cuda.synchronize()
    for b in range(batch):
        sk, sv, ids = w.compact_store(b)
        ref, _, _ = oracle_block(w.X[b], W, Hq, Hkv, D, w.rope_theta, sk, sv, ids, w.used_len[b], extras=extras)
        check_hidden(host(h_out[b]), ref, f"seed {seed}: D={D} Hq={Hq} Hkv={Hkv} H={H} F={F} B={batch} T={t_fresh} chunks={n_chunks}x{C} variants={extras is not None} b={b}")


def test_kv_slice_round_trip_and_errors():
    Hkv, D, C, T = 2, 64, 64, 150
    pc = Percache(n_layers=2, hidden=256, n_q_heads=4, n_kv_heads=Hkv, head_dim=D, n_slots=8, slot_capacity=C,
                  max_pos=256, device=DEV)
    g = np.random.default_rng(3)
    k = bf16(g.standard_normal((Hkv, T, D)))
    v = bf16(g.standard_normal((Hkv, T, D)))
    bounds, slots = [0, 64, 100, 150], [5, -1, 2]
    pc.percache_kv_slice(1, k, v, bounds, slots)
    torch.cuda.synchronize()
    assert pc.percache_kv_len(1, 5) == 64 and pc.percache_kv_len(1, 2) == 50 and pc.percache_kv_len(0, 5) == 0
    for lo, hi, s in [(0, 64, 5), (100, 150, 2)]:
        kk, vv = pc.percache_kv_get(1, s)
        torch.cuda.synchronize()
        assert torch.equal(kk, k[:, lo:hi]) and torch.equal(vv, v[:, lo:hi])
    for bad_bounds, bad_slots, status in [([0, 65, 150], [1, -1], -4), ([0, 64, 151], [1, 2], -4), ([0, 64, 128], [1, 1], -1),
                                          ([0, 64, 128], [1, 8], -3)]:
        with pytest.raises(PercacheError) as e:
            pc.percache_kv_slice(0, k, v, bad_bounds, bad_slots)
        assert e.value.status == status
    assert pc.percache_kv_len(0, 1) == 0   # failed calls wrote nothing


def test_two_layer_stack_population_then_reuse():
    """The population pass (ordinary prefill of the whole prompt, K/V sliced into slots on the way) and the reuse pass
    on the last rows, both against the oracle's two-layer stack; then GPU reuse against GPU full on the same rows."""
    H, Hq, Hkv, D, F, C, n_c, Tf, L = 256, 4, 2, 64, 448, 64, 3, 40, 2
    total = n_c * C + Tf
    h0 = wl.round_bf16(np.random.default_rng(9).standard_normal((total, H)).astype(np.float32))
    Ws = [wl.stack_weights(9, l, H, Hq, Hkv, D, F) for l in range(L)]
    layers = dev_layers(Ws)
    pc = Percache(n_layers=L, hidden=H, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=D, n_slots=8, slot_capacity=C,
                  max_pos=total, device=DEV)
    # oracle: full pass, K/V per layer
    h = h0
    stores = []
    for W in Ws:
        h, K, V = oracle_block(h, W, Hq, Hkv, D, 10000.0)
        stores.append((np.stack([K[:, c * C:(c + 1) * C] for c in range(n_c)]), np.stack([V[:, c * C:(c + 1) * C] for c in range(n_c)])))
    ref_full = h
    # GPU population pass
    slots = [6, 1, 4]
    bounds = [c * C for c in range(n_c + 1)] + [total]
    full = pc.percache_stack_reuse(layers, F, EPS, bf16(h0[None]), save_bounds=bounds, save_slots=[slots + [-1]])
    torch.cuda.synchronize()
    check_hidden(host(full[0]), ref_full, "population pass, all rows")
    for l in range(L):
        for c, s in enumerate(slots):
            assert pc.percache_kv_len(l, s) == C
            kk, vv = pc.percache_kv_get(l, s)
            torch.cuda.synchronize()
            check_hidden(host(kk), stores[l][0][c], f"sliced K layer {l} chunk {c}", rel_max=2.0 ** -6)
            check_hidden(host(vv), stores[l][1][c], f"sliced V layer {l} chunk {c}", rel_max=2.0 ** -6)
    # GPU reuse pass on the fresh rows, from the GPU-made cache
    reuse = pc.percache_stack_reuse(layers, F, EPS, bf16(h0[None, n_c * C:]), [slots])
    torch.cuda.synchronize()
    check_hidden(host(reuse[0]), ref_full[n_c * C:], "reuse pass vs oracle full recompute")
    check_hidden(host(reuse[0]), host(full[0, n_c * C:]), "reuse pass vs population pass (GPU)")
    # error paths: a save slot that the call also reads; differing lengths between layers
    with pytest.raises(PercacheError) as e:
        pc.percache_stack_reuse(layers, F, EPS, bf16(h0[None, n_c * C:]), [slots], save_bounds=[0, Tf], save_slots=[[6]])
    assert e.value.status == -1
    pc.percache_kv_evict(1, 4)
    with pytest.raises(PercacheError) as e:
        pc.percache_stack_reuse(layers, F, EPS, bf16(h0[None, n_c * C:]), [slots])
    assert e.value.status == -3


def test_config2_full_size_reuse_equals_full_recompute():
    """28-layer Qwen3-0.6B-shaped stack, 8 chunks x 512 cached + 128 fresh tokens.  The GPU's own full prefill of the
    4224-token prompt fills the cache (slicer); the reuse pass over the last 128 rows must reproduce the full pass's
    rows.  The oracle checks layer 0 of the full pass on sampled rows (deeper layers are covered at reduced size)."""
    w = wl.config2(n_slots=16)
    F, L, C, n_c, Tf = 3072, w.n_layers, w.chunk_tokens, w.n_chunks, w.t_fresh
    total = n_c * C + Tf
    h0 = wl.round_bf16(np.random.default_rng(2).standard_normal((total, w.hidden)).astype(np.float32))
    Ws = [wl.stack_weights(2, l, w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, F) for l in range(L)]
    layers = dev_layers(Ws)
    pc = Percache(n_layers=L, hidden=w.hidden, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim,
                  n_slots=16, slot_capacity=C, max_pos=total, device=DEV)
    slots = [int(s) for s in w.slot_ids[0]]
    bounds = [c * C for c in range(n_c + 1)] + [total]
    h_dev = bf16(h0[None])
    one = pc.percache_stack_reuse(layers[:1], F, EPS, h_dev)
    full = pc.percache_stack_reuse(layers, F, EPS, h_dev, save_bounds=bounds, save_slots=[slots + [-1]])
    reuse = pc.percache_stack_reuse(layers, F, EPS, h_dev[:, n_c * C:].contiguous(), [slots])
    torch.cuda.synchronize()
    check_hidden(host(reuse[0]), host(full[0, n_c * C:]), "cfg2: reuse vs full recompute after 28 layers", rel_max=2.0 ** -5, rel_fro=2e-2)
    # layer 0 of the full pass against the oracle on the first 96 rows (causal: they depend on nothing later)
    ref, _, _ = oracle_block(h0[:96], Ws[0], w.n_q_heads, w.n_kv_heads, w.head_dim, w.rope_theta)
    check_hidden(host(one[0, :96]), ref, "cfg2: layer 0 of the full pass, rows 0..95")


def depth_bounds(n_layers):
    """Bar on the relative Frobenius error of the hidden state after ``n_layers`` blocks against the unrounded oracle.
    One bf16 rounding has a relative error of at most 2^-9, uniformly spread: rms u = 2^-9 / sqrt(3).  In a block two
    stored tensors have the residual's own size (h' and h''), the branch outputs carry a few more roundings at a
    fraction of it: about 2u per block (measured 2.3e-3 = 2.04u).  The errors of different blocks are independent and
    ride along the residual path with unit gain, so after L blocks the relative Frobenius error is 2u sqrt(L); the bar
    allows twice that for what the non-linear branches add.  Element by element the error is largely relative to the
    element's own size (the roundings of the residual stream itself), so the largest error sits on the largest
    elements: four standard deviations of the expected relative error bar/2 there, i.e. max-abs <= 2 bar max|ref|."""
    u = 2.0 ** -9 / np.sqrt(3.0)
    return 4.0 * u * np.sqrt(n_layers)


def test_config2_random_store_reuse_vs_oracle_at_depth():
    """Config 2 as worded: 28 layers, 8 chunks x 512 tokens gathered from a 256-slot store of N(0,1) K/V by random slot
    ids, 128 fresh tokens.  The oracle's blocks are chained over all 28 layers on the reuse path and compared with
    percache_stack_reuse after the last layer (and after layers 1, 2, 7, 14 of the same chain, from shorter GPU runs)."""
    w = wl.config2()
    F, L, C, n_c, Tf = 3072, w.n_layers, w.chunk_tokens, w.n_chunks, w.t_fresh
    Ws = [wl.stack_weights(2, l, w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, F) for l in range(L)]
    layers = dev_layers(Ws)
    pc = Percache(n_layers=L, hidden=w.hidden, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim,
                  n_slots=w.n_slots, slot_capacity=C, max_pos=n_c * C + Tf, device=DEV)
    slots = [int(s) for s in w.slot_ids[0]]
    for l in range(L):
        for s_, (k, v) in w.slots_kv(slots, l).items():
            pc.percache_kv_put(l, s_, bf16(k), bf16(v))
    x = bf16(w.X)
    got = {n: host(pc.percache_stack_reuse(layers[:n], F, EPS, x, w.slot_ids, w.used_len)[0]) for n in (1, 2, 7, 14, L)}
    torch.cuda.synchronize()
    h = w.X[0]
    for l in range(L):
        sk, sv, ids = w.compact_store(0, l)
        h, _, _ = oracle_block(h, Ws[l], w.n_q_heads, w.n_kv_heads, w.head_dim, w.rope_theta, sk, sv, ids, w.used_len[0])
        n = l + 1
        if n in got:
            bar = depth_bounds(n)
            top = float(np.abs(h).max())
            err = np.abs(got[n] - h)
            fro = np.linalg.norm(got[n] - h) / np.linalg.norm(h)
            print(f"cfg2 random store, after {n} layers: rel-fro {fro:.3e} (bar {bar:.3e}) max-abs {err.max():.3e} "
                  f"(bar {2 * bar * top:.3e}, max|ref| {top:.3f})", flush=True)
            assert np.isfinite(got[n]).all() and fro <= bar and err.max() <= 2 * bar * top
    pc.close()


@pytest.mark.parametrize("D,t_fresh,which,heads", [
    (128, 40, "all", (4, 2)), (64, 40, "all", (4, 2)), (128, 260, "all", (4, 2)), (64, 260, "all", (4, 2)),
    (128, 260, "bias", (4, 2)), (128, 40, "norm", (4, 2)), (64, 260, "qnorm", (4, 2)),
    (128, 1700, "all", (24, 8)),   # enough tiles for the launcher's 192-token tiles
])
def test_projection_variants_bias_and_head_norm(D, t_fresh, which, heads):
    """Qwen-family variants of the projection: bias, RMSNorm over the head dimension of q and k before RoPE; few rows
    (split-k path) and many rows (single-pass kernel, 128- and 192-token tiles), both head sizes, each part alone and
    together."""
    H, (Hq, Hkv), F, C = 256, heads, 384, 64
    w = wl.make_prefill("var", 23, "bf16", H, Hq, Hkv, D, 1, t_fresh, 2, C, 4)
    W = wl.stack_weights(23, 0, H, Hq, Hkv, D, F)
    g = np.random.default_rng(50 + D)
    n_out = (Hq + 2 * Hkv) * D
    bias = wl.round_bf16(0.5 * g.standard_normal(n_out).astype(np.float32)) if which in ("all", "bias") else None
    qg = wl.round_bf16(1 + 0.2 * g.standard_normal(D).astype(np.float32)) if which in ("all", "norm", "qnorm") else None
    kg = wl.round_bf16(1 + 0.2 * g.standard_normal(D).astype(np.float32)) if which in ("all", "norm") else None
    layer = dev_layers([W])[0]
    if bias is not None:
        layer["qkv_bias"] = bf16(bias)
    if qg is not None:
        layer["q_norm"] = bf16(qg)
    if kg is not None:
        layer["k_norm"] = bf16(kg)
    pc = Percache(n_layers=1, hidden=H, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=D, n_slots=4, slot_capacity=C,
                  max_pos=w.max_pos, device=DEV)
    for s_ in sorted(set(int(x) for x in w.slot_ids.reshape(-1))):
        k, v = w.slot_kv(s_)
        pc.percache_kv_put(0, s_, bf16(k), bf16(v))
    h_out = pc.percache_stack_reuse([layer], F, EPS, bf16(w.X), w.slot_ids, w.used_len)
    plain = pc.percache_stack_reuse(dev_layers([W]), F, EPS, bf16(w.X), w.slot_ids, w.used_len)
    torch.cuda.synchronize()
    sk, sv, ids = w.compact_store(0)
    ref, _, _ = oracle_block(w.X[0], W, Hq, Hkv, D, w.rope_theta, sk, sv, ids, w.used_len[0],
                             extras=dict(bias=bias, q_gain=qg, k_gain=kg, eps=EPS))
    check_hidden(host(h_out[0]), ref, f"variants {which} D={D} T={t_fresh}")
    assert np.abs(host(h_out[0]) - host(plain[0])).max() > 1e-2     # the variant is not the plain block
