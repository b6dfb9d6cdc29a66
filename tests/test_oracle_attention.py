"""Pins of the attention / projection / RoPE oracle (CPU only).

The paper prints no worked numeric example of these computations, so the oracle is pinned by
  * brute force: cache-reusing prefill == full recomputation of the contiguous prompt
    (Sec. 4.2.2, App. B.1), with planted mistakes that must break the equality;
  * an independent textbook formulation in numpy/scipy float64 (matmul + scipy softmax,
    complex-number RoPE);
  * invariants and closed-form special cases.
"""
import numpy as np
import pytest
from scipy.special import softmax as sp_softmax

import oracle
from paper_2601_11553_amd import workloads as wl


# ---------------------------------------------------------------- independent textbook reference
def rope_complex(u, pos, theta):
    """RoFormer rotation written with complex numbers: (u[m] + i u[m+D/2]) * exp(i pos theta^(-2m/D))."""
    u = np.asarray(u, np.float64)
    D = u.shape[-1]
    m = np.arange(D // 2)
    ang = pos * theta ** (-2.0 * m / D)
    z = (u[..., : D // 2] + 1j * u[..., D // 2:]) * np.exp(1j * ang)
    return np.concatenate([z.real, z.imag], axis=-1)


def textbook_causal_layer(X, W, Hq, Hkv, D, theta):
    """softmax(Q K^T / sqrt(D) + causal mask) V with numpy matmul; returns O[T,Hq*D], K, V [Hkv,T,D]."""
    X = np.asarray(X, np.float64)
    W = np.asarray(W, np.float64)
    T = X.shape[0]
    Y = X @ W.T
    q = Y[:, : Hq * D].reshape(T, Hq, D)
    k = Y[:, Hq * D:(Hq + Hkv) * D].reshape(T, Hkv, D)
    v = Y[:, (Hq + Hkv) * D:].reshape(T, Hkv, D)
    for t in range(T):
        q[t] = rope_complex(q[t], t, theta)
        k[t] = rope_complex(k[t], t, theta)
    G = Hq // Hkv
    O = np.zeros((T, Hq, D))
    mask = np.triu(np.full((T, T), -np.inf), k=1)
    for h in range(Hq):
        s = q[:, h] @ k[:, h // G].T / np.sqrt(D) + mask
        O[:, h] = sp_softmax(s, axis=-1) @ v[:, h // G]
    return O.reshape(T, Hq * D), k.transpose(1, 0, 2), v.transpose(1, 0, 2)


def slice_into_store(K, V, n_chunks, C):
    """The cache slicer (Sec. 4.1.1): rows [c*C, (c+1)*C) of the prompt's K/V become slot c."""
    Hkv, _, D = K.shape
    sk = np.stack([K[:, c * C:(c + 1) * C] for c in range(n_chunks)])
    sv = np.stack([V[:, c * C:(c + 1) * C] for c in range(n_chunks)])
    return sk.astype(np.float32), sv.astype(np.float32)


@pytest.fixture(scope="module")
def cfg0():
    w = wl.config0("f32", seed=0)
    full_O, full_K, full_V, full_Q = oracle.prefill_reuse(w.prompt, w.Wqkv, w.n_q_heads, w.n_kv_heads, w.head_dim, w.rope_theta)
    return w, full_O, full_K, full_V, full_Q


# ---------------------------------------------------------------- full prefill vs textbook
def test_full_prefill_matches_textbook_numpy(cfg0):
    w, full_O, full_K, full_V, _ = cfg0
    O, K, V = textbook_causal_layer(w.prompt, w.Wqkv, w.n_q_heads, w.n_kv_heads, w.head_dim, w.rope_theta)
    assert np.abs(full_O - O).max() < 2e-6
    assert np.abs(full_K - K).max() < 2e-6
    assert np.abs(full_V - V).max() < 2e-6


# ---------------------------------------------------------------- P1: reuse == full recompute
def _reuse(w, sk, sv, slot_ids, used_len, n_fresh_from):
    return oracle.prefill_reuse(w.prompt[n_fresh_from:], w.Wqkv, w.n_q_heads, w.n_kv_heads, w.head_dim,
                                w.rope_theta, sk, sv, slot_ids, used_len)


def test_reuse_equals_full_recompute(cfg0):
    w, full_O, full_K, full_V, _ = cfg0
    sk, sv = slice_into_store(full_K, full_V, w.n_chunks, w.chunk_tokens)
    O, Kf, Vf, _ = _reuse(w, sk, sv, [0, 1], [64, 64], w.l_pre)
    assert O.shape == (16, 4 * 64)
    assert np.abs(O - full_O[w.l_pre:]).max() < 1e-6
    assert np.abs(Kf - full_K[:, w.l_pre:]).max() < 1e-6
    assert np.abs(Vf - full_V[:, w.l_pre:]).max() < 1e-6


def test_reuse_against_textbook_directly(cfg0):
    w, _, full_K, full_V, _ = cfg0
    O_ref, _, _ = textbook_causal_layer(w.prompt, w.Wqkv, w.n_q_heads, w.n_kv_heads, w.head_dim, w.rope_theta)
    sk, sv = slice_into_store(full_K, full_V, w.n_chunks, w.chunk_tokens)
    O, _, _, _ = _reuse(w, sk, sv, [0, 1], [64, 64], w.l_pre)
    assert np.abs(O - O_ref[w.l_pre:]).max() < 2e-6


def test_slot_placement_is_invisible(cfg0):
    """The same chunks in other slots of a larger store, addressed by the permuted list: same output."""
    w, full_O, full_K, full_V, _ = cfg0
    sk, sv = slice_into_store(full_K, full_V, w.n_chunks, w.chunk_tokens)
    big_k = np.random.default_rng(5).standard_normal((5,) + sk.shape[1:]).astype(np.float32)
    big_v = np.random.default_rng(6).standard_normal((5,) + sv.shape[1:]).astype(np.float32)
    big_k[3], big_v[3] = sk[0], sv[0]
    big_k[1], big_v[1] = sk[1], sv[1]
    O, _, _, _ = _reuse(w, big_k, big_v, [3, 1], [64, 64], w.l_pre)
    assert np.abs(O - full_O[w.l_pre:]).max() < 1e-6


# ---------------------------------------------------------------- P2: planted mistakes must break P1
def test_negative_controls_break_equality(cfg0):
    w, full_O, full_K, full_V, _ = cfg0
    sk, sv = slice_into_store(full_K, full_V, w.n_chunks, w.chunk_tokens)
    ref = full_O[w.l_pre:]
    Hq, Hkv, D = w.n_q_heads, w.n_kv_heads, w.head_dim
    X = w.prompt[w.l_pre:]

    # (a) RoPE position counter not advanced by L_pre
    Q, Kf, Vf = oracle.qkv_rope(X, w.Wqkv, Hq, Hkv, D, 0, w.rope_theta)
    O = oracle.attention_reuse(Q, Kf, Vf, sk, sv, [0, 1], [64, 64])
    assert np.abs(O - ref).max() > 1e-3

    # (b) keys gathered from one chunk order, values from the other.  (Swapping BOTH is harmless:
    # loaded keys carry their positions inside them and softmax attention is invariant under a joint
    # permutation of keys and values -- checked as a positive property right after.)
    Q_ok = oracle.qkv_rope(X, w.Wqkv, Hq, Hkv, D, w.l_pre, w.rope_theta)[0]
    O = oracle.attention_reuse(Q_ok, full_K[:, w.l_pre:], full_V[:, w.l_pre:], sk, sv[::-1].copy(), [0, 1], [64, 64])
    assert np.abs(O - ref).max() > 1e-3
    O, _, _, _ = _reuse(w, sk, sv, [1, 0], [64, 64], w.l_pre)
    assert np.abs(O - ref).max() < 1e-6

    # (c) causal mask off by one (row i must see fresh key i): emulate by hiding the diagonal key
    Q, Kf, Vf = oracle.qkv_rope(X, w.Wqkv, Hq, Hkv, D, w.l_pre, w.rope_theta)
    Kshift = np.concatenate([Kf[:, :1] * 0 + 1e3, Kf[:, :-1]], axis=1)  # key t replaced by key t-1
    O = oracle.attention_reuse(Q, Kshift, Vf, sk, sv, [0, 1], [64, 64])
    assert np.abs(O - ref).max() > 1e-3

    # (d) wrong GQA mapping (h % Hkv instead of h // G): swap which kv head q heads 1,2 use
    Qswap = Q.copy()
    Qswap[[1, 2]] = Q[[2, 1]]
    O = oracle.attention_reuse(Qswap, Kf, Vf, sk, sv, [0, 1], [64, 64]).reshape(16, Hq, D)
    O[:, [1, 2]] = O[:, [2, 1]]
    assert np.abs(O.reshape(16, -1) - ref).max() > 1e-3

    # (e) transposed weight layout would not even have the right shape; a V/K swap must break it
    O = oracle.attention_reuse(Q, Vf, Kf, sk, sv, [0, 1], [64, 64])
    assert np.abs(O - ref).max() > 1e-3


# ---------------------------------------------------------------- P7: partial last chunk
def test_used_len_shortening_equals_recompute_on_shortened_prefix(cfg0):
    """App. B.2: the last few tokens of the final matched chunk are dropped and recomputed from text.

    Dropping 4 tokens of chunk 1 and feeding them as fresh rows must give the same final rows.
    """
    w, full_O, full_K, full_V, _ = cfg0
    sk, sv = slice_into_store(full_K, full_V, w.n_chunks, w.chunk_tokens)
    O, Kf, Vf, _ = _reuse(w, sk, sv, [0, 1], [64, 60], w.l_pre - 4)
    assert O.shape[0] == 20
    assert np.abs(O - full_O[w.l_pre - 4:]).max() < 1e-6
    assert np.abs(Kf - full_K[:, w.l_pre - 4:]).max() < 1e-6


def test_chunk_boundaries_are_invisible(cfg0):
    """2 slots x 64 tokens and 1 slot x 128 tokens describe the same key sequence."""
    w, full_O, full_K, full_V, _ = cfg0
    sk1, sv1 = slice_into_store(full_K, full_V, 1, 128)
    O, _, _, _ = _reuse(w, sk1, sv1, [0], [128], w.l_pre)
    assert np.abs(O - full_O[w.l_pre:]).max() < 1e-6


# ---------------------------------------------------------------- P3: softmax invariants
def test_softmax_rows_sum_to_one_and_output_in_convex_hull(cfg0):
    w, _, full_K, full_V, full_Q = cfg0
    sk, sv = slice_into_store(full_K, full_V, w.n_chunks, w.chunk_tokens)
    Q = full_Q[:, w.l_pre:]
    Kf, Vf = full_K[:, w.l_pre:], full_V[:, w.l_pre:]
    O, rs = oracle.attention_reuse(Q, Kf, Vf, sk, sv, [0, 1], [64, 64], want_row_sum=True)
    assert np.abs(rs - 1.0).max() < 1e-6
    G = w.n_q_heads // w.n_kv_heads
    O = O.reshape(w.t_fresh, w.n_q_heads, w.head_dim)
    for i in range(w.t_fresh):
        for h in range(w.n_q_heads):
            vis = full_V[h // G, : w.l_pre + i + 1]
            assert np.all(O[i, h] <= vis.max(0) + 1e-6) and np.all(O[i, h] >= vis.min(0) - 1e-6)


def test_sampled_rows_match_full_output(cfg0):
    w, full_O, full_K, full_V, _ = cfg0
    sk, sv = slice_into_store(full_K, full_V, w.n_chunks, w.chunk_tokens)
    rows, heads = [0, 7, 15, 3], [0, 3, 2, 1]
    Os, _, _, _ = oracle.prefill_reuse(w.prompt[w.l_pre:], w.Wqkv, w.n_q_heads, w.n_kv_heads, w.head_dim,
                                       w.rope_theta, sk, sv, [0, 1], [64, 64], samples=(rows, heads))
    ref = full_O[w.l_pre:].reshape(w.t_fresh, w.n_q_heads, w.head_dim)
    for s, (i, h) in enumerate(zip(rows, heads)):
        assert np.abs(Os[s] - ref[i, h]).max() < 1e-6


# ---------------------------------------------------------------- P4: RoPE closed forms
@pytest.mark.parametrize("D", [64, 128])
def test_rope_properties(D):
    g = np.random.default_rng(11)
    u = g.standard_normal(D).astype(np.float32)
    v = g.standard_normal(D).astype(np.float32)
    theta = 10000.0
    assert np.array_equal(oracle.rope(u, 0, theta), u)
    for pos in (1, 17, 143, 16639):
        r = oracle.rope(u, pos, theta)
        assert abs(np.linalg.norm(r) - np.linalg.norm(u)) < 1e-5
        assert np.abs(r - rope_complex(u, pos, theta)).max() < 1e-6
    # relative-position property
    a = float(np.dot(oracle.rope(u, 40, theta).astype(np.float64), oracle.rope(v, 33, theta)))
    b = float(np.dot(oracle.rope(u, 1040, theta).astype(np.float64), oracle.rope(v, 1033, theta)))
    assert abs(a - b) < 1e-4
    # the first pair rotates by exactly pos radians, the pairing is (m, m + D/2)
    e = np.zeros(D, np.float32)
    e[0] = 1.0
    r = oracle.rope(e, 1, theta)
    assert abs(r[0] - np.cos(1.0)) < 1e-7 and abs(r[D // 2] - np.sin(1.0)) < 1e-7
    assert np.abs(np.delete(r, [0, D // 2])).max() == 0.0


def test_projection_layout_and_positions():
    """W rows are [Q heads | K heads | V heads]; V is not rotated; row i sits at pos0 + i."""
    g = np.random.default_rng(3)
    H, Hq, Hkv, D, T = 32, 4, 2, 8, 5
    X = g.standard_normal((T, H)).astype(np.float32)
    W = g.standard_normal(((Hq + 2 * Hkv) * D, H)).astype(np.float32)
    Q, K, V = oracle.qkv_rope(X, W, Hq, Hkv, D, 100, 10000.0)
    Y = X.astype(np.float64) @ W.astype(np.float64).T
    for i in range(T):
        for h in range(Hq):
            assert np.abs(Q[h, i] - rope_complex(Y[i, h * D:(h + 1) * D], 100 + i, 10000.0)).max() < 1e-5
        for gk in range(Hkv):
            assert np.abs(K[gk, i] - rope_complex(Y[i, (Hq + gk) * D:(Hq + gk + 1) * D], 100 + i, 10000.0)).max() < 1e-5
            assert np.abs(V[gk, i] - Y[i, (Hq + Hkv + gk) * D:(Hq + Hkv + gk + 1) * D]).max() < 1e-5


# ---------------------------------------------------------------- P5: special cases
def test_single_query_single_chunk_is_textbook_attention():
    g = np.random.default_rng(21)
    D, C = 64, 37
    q = g.standard_normal((1, 1, D)).astype(np.float32)
    sk = g.standard_normal((1, 1, C, D)).astype(np.float32)
    sv = g.standard_normal((1, 1, C, D)).astype(np.float32)
    kf = g.standard_normal((1, 1, D)).astype(np.float32)
    vf = g.standard_normal((1, 1, D)).astype(np.float32)
    O = oracle.attention_reuse(q, kf, vf, sk, sv, [0], [C])
    Kall = np.concatenate([sk[0, 0], kf[0]], 0).astype(np.float64)
    Vall = np.concatenate([sv[0, 0], vf[0]], 0).astype(np.float64)
    p = sp_softmax(Kall @ q[0, 0].astype(np.float64) / np.sqrt(D))
    assert np.abs(O[0] - p @ Vall).max() < 1e-6


def test_uniform_keys_give_mean_of_values_and_peaked_key_selects_its_value():
    g = np.random.default_rng(22)
    D, C = 64, 50
    q = g.standard_normal((1, 1, D)).astype(np.float32)
    k_same = np.tile(g.standard_normal(D).astype(np.float32), (1, 1, C, 1))
    sv = g.standard_normal((1, 1, C, D)).astype(np.float32)
    O = oracle.attention_reuse(q, k_same[0, :, :1], sv[0, :, :1] * 0 + sv[0, 0, 0], k_same, sv, [0], [C])
    expect = (sv[0, 0].astype(np.float64).sum(0) + sv[0, 0, 0]) / (C + 1)
    assert np.abs(O[0] - expect).max() < 1e-6
    # one key aligned with q and scaled so its logit exceeds the rest by > 50
    sk = g.standard_normal((1, 1, C, D)).astype(np.float32) * 0.01
    sk[0, 0, 17] = q[0, 0] * (60.0 * np.sqrt(D) / float(np.dot(q[0, 0], q[0, 0])))
    kf = np.zeros((1, 1, D), np.float32)
    O = oracle.attention_reuse(q, kf, sv[0, :, :1], sk, sv, [0], [C])
    assert np.abs(O[0] - sv[0, 0, 17]).max() < 1e-6


# ---------------------------------------------------------------- P6: split invariance
def test_lse_merge_of_key_splits_equals_unsplit():
    g = np.random.default_rng(23)
    D, L = 64, 200
    q = g.standard_normal(D).astype(np.float32) * 2
    K = g.standard_normal((L, D)).astype(np.float32)
    V = g.standard_normal((L, D)).astype(np.float32)
    m, l, o = oracle.attend_stats(q, K, V)
    ref = sp_softmax(K.astype(np.float64) @ q / np.sqrt(D)) @ V
    assert np.abs(o - ref).max() < 1e-12
    cuts = [0, 13, 90, 91, 200]
    parts = [oracle.attend_stats(q, K[a:b], V[a:b]) for a, b in zip(cuts[:-1], cuts[1:])]
    merged = oracle.lse_merge([p[0] for p in parts], [p[1] for p in parts], np.stack([p[2] for p in parts]))
    assert np.abs(merged - ref).max() < 1e-12


def test_full_prefill_on_bf16_inputs_matches_textbook():
    """Same pin on inputs already rounded to the GPU storage dtype, head_dim 128, G = 3."""
    g = np.random.default_rng(31)
    H, Hq, Hkv, D, T = 96, 6, 2, 128, 40
    X = wl.round_bf16(g.standard_normal((T, H)).astype(np.float32))
    W = wl.round_bf16((g.standard_normal(((Hq + 2 * Hkv) * D, H)) * 0.1).astype(np.float32))
    O, K, V, _ = oracle.prefill_reuse(X, W, Hq, Hkv, D, 10000.0)
    Or, Kr, Vr = textbook_causal_layer(X, W, Hq, Hkv, D, 10000.0)
    assert np.abs(O - Or).max() < 2e-6 and np.abs(K - Kr).max() < 2e-6 and np.abs(V - Vr).max() < 2e-6


def test_projection_variants_bias_and_head_norm_match_numpy():
    """Bias on the projection and RMSNorm over the head dimension of q / k before RoPE (the Qwen-family variants):
    against a float64 numpy statement with complex-number RoPE; the plain call is the variant with everything off."""
    g = np.random.default_rng(3)
    T, H, Hq, Hkv, D = 5, 32, 4, 2, 16
    X = g.standard_normal((T, H)).astype(np.float32)
    W = (g.standard_normal(((Hq + 2 * Hkv) * D, H)) * 0.2).astype(np.float32)
    b = g.standard_normal((Hq + 2 * Hkv) * D).astype(np.float32)
    qg = (1 + 0.1 * g.standard_normal(D)).astype(np.float32)
    kg = (1 + 0.1 * g.standard_normal(D)).astype(np.float32)
    Q, K, V = oracle.qkv_rope(X, W, Hq, Hkv, D, 7, 10000.0, bias=b, q_gain=qg, k_gain=kg, eps=1e-6)
    Y = X.astype(np.float64) @ W.astype(np.float64).T + b

    def rope(u, pos):
        ang = pos * 10000.0 ** (-2 * np.arange(D // 2) / D)
        z = (u[:D // 2] + 1j * u[D // 2:]) * np.exp(1j * ang)
        return np.concatenate([z.real, z.imag])

    for i in range(T):
        for h in range(Hq + Hkv):
            u = Y[i, h * D:(h + 1) * D]
            u = u / np.sqrt((u * u).mean() + 1e-6) * (qg if h < Hq else kg)
            got = Q[h, i] if h < Hq else K[h - Hq, i]
            assert np.abs(rope(u, 7 + i) - got).max() < 1e-5
        for h in range(Hkv):
            assert np.abs(Y[i, (Hq + Hkv + h) * D:(Hq + Hkv + h + 1) * D] - V[h, i]).max() < 1e-5
    Q0, K0, V0 = oracle.qkv_rope(X, W, Hq, Hkv, D, 7, 10000.0)
    Q1, K1, V1 = oracle.qkv_rope(X, W, Hq, Hkv, D, 7, 10000.0, bias=np.zeros_like(b))
    assert np.array_equal(Q0, Q1) and np.array_equal(K0, K1) and np.array_equal(V0, V1)
    assert np.abs(Q0 - Q).max() > 0.1        # the variants do change the result
