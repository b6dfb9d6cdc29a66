"""Pins of the block-tail oracle (RMSNorm, linear, SwiGLU, residuals) and of multi-layer reuse.

App. B.1 says the operations after attention run as usual; these are the textbook definitions, so the
pins are numpy float64 re-statements, plus the multi-layer brute force: a stack run on the whole prompt
and a stack run on the fresh rows against per-layer stores sliced from the first run agree on the fresh
rows (causality makes fresh rows depend on cached tokens only through cached K and V).
"""
import numpy as np

import oracle
from paper_2601_11553_amd import workloads as wl


def test_rmsnorm_and_linear_match_numpy():
    g = np.random.default_rng(1)
    X = g.standard_normal((9, 40)).astype(np.float32) * 3
    gain = (1 + 0.1 * g.standard_normal(40)).astype(np.float32)
    W = g.standard_normal((13, 40)).astype(np.float32)
    Y = oracle.rmsnorm(X, gain, 1e-6)
    X64 = X.astype(np.float64)
    ref = X64 / np.sqrt((X64 ** 2).mean(-1, keepdims=True) + 1e-6) * gain
    assert np.abs(Y - ref).max() < 1e-6
    # unit-gain rows have mean square 1
    Y1 = oracle.rmsnorm(X, None, 0.0)
    assert np.abs((Y1.astype(np.float64) ** 2).mean(-1) - 1).max() < 1e-6
    assert np.abs(oracle.linear(X, W) - X64 @ W.astype(np.float64).T).max() < 1e-5


def test_block_tail_matches_numpy():
    g = np.random.default_rng(2)
    T, H, A, F = 6, 24, 32, 40
    h = g.standard_normal((T, H)).astype(np.float32)
    attn = g.standard_normal((T, A)).astype(np.float32)
    Wo = g.standard_normal((H, A)).astype(np.float32) * 0.2
    g2 = (1 + 0.1 * g.standard_normal(H)).astype(np.float32)
    Wg = g.standard_normal((F, H)).astype(np.float32) * 0.3
    Wu = g.standard_normal((F, H)).astype(np.float32) * 0.3
    Wd = g.standard_normal((H, F)).astype(np.float32) * 0.3
    out = oracle.block_tail(h, attn, Wo, g2, Wg, Wu, Wd, 1e-6)
    f = lambda a: a.astype(np.float64)
    mid = f(h) + f(attn) @ f(Wo).T
    mid = mid.astype(np.float32).astype(np.float64)
    n = mid / np.sqrt((mid ** 2).mean(-1, keepdims=True) + 1e-6) * f(g2)
    ga, up = n @ f(Wg).T, n @ f(Wu).T
    ref = mid + ((ga / (1 + np.exp(-ga))) * up) @ f(Wd).T
    assert np.abs(out - ref).max() < 1e-5
    # silu(0) = 0: zero gate weights leave only the attention residual
    out0 = oracle.block_tail(h, attn, Wo, g2, Wg * 0, Wu, Wd, 1e-6)
    assert np.abs(out0 - mid).max() < 1e-6


def test_two_layer_stack_reuse_equals_full():
    H, Hq, Hkv, D, F = 64, 4, 2, 16, 96
    C, n_c, Tf = 12, 2, 5
    total = C * n_c + Tf
    g = np.random.default_rng(4)
    h0 = g.standard_normal((total, H)).astype(np.float32)
    Ws = [wl.stack_weights(7, l, H, Hq, Hkv, D, F, dtype="f32") for l in range(2)]
    # full pass over the whole prompt, collecting K/V per layer
    h = h0
    stores = []
    for Wl in Ws:
        h, K, V = oracle.block(h, Wl.gain1, Wl.Wqkv * 5, Hq, Hkv, D, 10000.0, Wl.Wo * 5, Wl.gain2, Wl.Wgate * 5,
                               Wl.Wup * 5, Wl.Wdown * 5, 1e-6)
        stores.append((np.stack([K[:, c * C:(c + 1) * C] for c in range(n_c)]),
                       np.stack([V[:, c * C:(c + 1) * C] for c in range(n_c)])))
    full_last = h[C * n_c:]
    # reuse pass over fresh rows only
    hf = h0[C * n_c:]
    for Wl, (sk, sv) in zip(Ws, stores):
        hf, _, _ = oracle.block(hf, Wl.gain1, Wl.Wqkv * 5, Hq, Hkv, D, 10000.0, Wl.Wo * 5, Wl.gain2, Wl.Wgate * 5,
                                Wl.Wup * 5, Wl.Wdown * 5, 1e-6, sk, sv, [0, 1], [C, C])
    assert np.abs(hf - full_last).max() < 2e-5
    assert np.abs(hf - h0[C * n_c:]).max() > 1e-2   # the block did something
