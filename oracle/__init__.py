"""ctypes front-end of the CPU oracle (test infrastructure, not product code).

Only ``tests/``, the smoke check and the benchmark's CPU-baseline leg may
import this package.  It loads ``oracle/liboracle.so`` (plain C built with gcc
from ``percache_oracle.c``); it never imports, links or calls the HIP library.

Every function takes and returns numpy float32 arrays holding the exact values
the GPU side stores in bf16/fp16.  See the C file for the paper passages each
routine follows.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "percache_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP over independent rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-o", tmp, _SRC, "-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


_F = ctypes.POINTER(ctypes.c_float)
_D = ctypes.POINTER(ctypes.c_double)
_I = ctypes.POINTER(ctypes.c_int32)
_U8 = ctypes.POINTER(ctypes.c_uint8)


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _f(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _i(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _pf(a: Optional[np.ndarray]):
    return a.ctypes.data_as(_F) if a is not None else None


def _pi(a: Optional[np.ndarray]):
    return a.ctypes.data_as(_I) if a is not None else None


def lookup(E, probes, tau: float):
    """Sec. 4.2.1 query-level match.  Returns (idx, sim, hit, sim2)."""
    E = _f(E)
    probes = _f(probes)
    P, d = probes.shape
    N = E.shape[0]
    if N:
        assert E.shape[1] == d
    idx = np.empty(P, np.int32)
    sim = np.empty(P, np.float32)
    sim2 = np.empty(P, np.float32)
    hit = np.empty(P, np.uint8)
    _load().oracle_lookup(
        _pf(E), ctypes.c_int(N), ctypes.c_int(d), _pf(probes), ctypes.c_int(P),
        ctypes.c_float(tau), _pi(idx), _pf(sim), hit.ctypes.data_as(_U8), _pf(sim2))
    return idx, sim, hit, sim2


def similarities(E, probe) -> np.ndarray:
    E = _f(E)
    probe = _f(probe)
    out = np.empty(E.shape[0], np.float32)
    _load().oracle_similarities(_pf(E), ctypes.c_int(E.shape[0]), ctypes.c_int(E.shape[1]),
                                _pf(probe), _pf(out))
    return out


def lookup_topk(E, probes, k: int):
    """The k most similar bank rows of each probe, best first; equal similarities: lower row first (the ranking
    behind cache refresh, Sec. 4.1.3, and dense retrieval).  The definition written out: all N cosine
    similarities, then a stable sort.  Returns (idx [P, k] int32 with -1 past the bank size, sim [P, k] float32 with
    -inf there, next [P] float32 = similarity ranked k+1, for judging near-ties)."""
    E = _f(E)
    probes = _f(probes)
    P = probes.shape[0]
    N = E.shape[0]
    idx = np.full((P, k), -1, np.int32)
    sim = np.full((P, k), -np.inf, np.float32)
    nxt = np.full(P, -np.inf, np.float32)
    for p in range(P):
        if N == 0:
            continue
        s = similarities(E, probes[p])
        order = np.argsort(-s.astype(np.float64), kind="stable")
        m = min(k, N)
        idx[p, :m] = order[:m]
        sim[p, :m] = s[order[:m]]
        if N > k:
            nxt[p] = s[order[k]]
    return idx, sim, nxt


def refresh_scan(E, new, kth):
    """Cache refresh (Sec. 4.1.3) for bank rows E (stored query embeddings) against newly added chunk embeddings:
    per row the best cosine similarity over the new chunks, the lowest chunk attaining it, and whether it exceeds
    the row's current k-th best similarity ``kth`` (then a new chunk enters that query's top-k).  By definition,
    row by row.  Returns (best_sim [N] float32, best_new [N] int32, stale [N] uint8)."""
    E = _f(E)
    new = _f(new)
    kth = np.asarray(kth, np.float32)
    N = E.shape[0]
    best_sim = np.empty(N, np.float32)
    best_new = np.empty(N, np.int32)
    for j in range(N):
        s = similarities(new, E[j])
        c = int(np.argmax(s))          # first maximum = lowest index
        best_sim[j], best_new[j] = s[c], c
    return best_sim, best_new, (best_sim > kth).astype(np.uint8)


def rope(u, pos: int, theta: float) -> np.ndarray:
    """RoPE of one head vector at absolute position ``pos`` (App. B.1)."""
    u = _f(u).copy()
    _load().oracle_rope(_pf(u), ctypes.c_int(u.shape[-1]), ctypes.c_long(pos), ctypes.c_double(theta))
    return u


def qkv_rope(X, W, Hq: int, Hkv: int, D: int, pos0: int, theta: float, bias=None, q_gain=None, k_gain=None,
             eps: float = 1e-6):
    """Projection + RoPE of one query's retained rows.  Returns Q[Hq,T,D], K, V[Hkv,T,D].

    Model-family variants (the paper runs Llama and Qwen models, Sec. 5.1): ``bias`` [(Hq+2Hkv)*D] is added to the
    projection; ``q_gain`` / ``k_gain`` [D] switch on an RMSNorm over the head dimension of every q / k head before RoPE."""
    X = _f(X)
    W = _f(W)
    T, H = X.shape
    assert W.shape == ((Hq + 2 * Hkv) * D, H)
    Q = np.empty((Hq, T, D), np.float32)
    K = np.empty((Hkv, T, D), np.float32)
    V = np.empty((Hkv, T, D), np.float32)
    b = _f(bias) if bias is not None else None
    qg = _f(q_gain) if q_gain is not None else None
    kg = _f(k_gain) if k_gain is not None else None
    _load().oracle_qkv_rope_ex(_pf(X), _pf(W), _pf(b), _pf(qg), _pf(kg), ctypes.c_double(eps), ctypes.c_int(T),
                               ctypes.c_int(H), ctypes.c_int(Hq), ctypes.c_int(Hkv), ctypes.c_int(D),
                               ctypes.c_long(pos0), ctypes.c_double(theta), _pf(Q), _pf(K), _pf(V))
    return Q, K, V


def _store_args(store_k, store_v, Hkv, D):
    if store_k is None:
        return None, None, 1
    store_k = _f(store_k)
    store_v = _f(store_v)
    assert store_k.shape == store_v.shape and store_k.shape[1] == Hkv and store_k.shape[3] == D
    return store_k, store_v, store_k.shape[2]


def attention_reuse(Q, Kf, Vf, store_k, store_v, slot_ids: Sequence[int], used_len: Sequence[int],
                    samples: Optional[Tuple[Sequence[int], Sequence[int]]] = None,
                    want_row_sum: bool = False):
    """Attention of one query's fresh rows over [loaded chunks ; fresh] (Sec. 4.2.2).

    Returns O[T, Hq*D] (or [n_samples, D] when ``samples=(rows, heads)``), optionally
    with the per-row sum of softmax probabilities.
    """
    Q = _f(Q)
    Kf = _f(Kf)
    Vf = _f(Vf)
    Hq, T, D = Q.shape
    Hkv = Kf.shape[0]
    sk, sv, C = _store_args(store_k, store_v, Hkv, D)
    ids = _i(slot_ids)
    ul = _i(used_len)
    n_c = len(ids)
    if n_c:
        assert sk is not None and ids.max() < sk.shape[0] and ids.min() >= 0 and ul.max() <= C
    if samples is not None:
        si, sh = _i(samples[0]), _i(samples[1])
        ns = len(si)
        O = np.empty((ns, D), np.float32)
        rs = np.empty(ns, np.float32)
    else:
        si = sh = None
        ns = 0
        O = np.empty((T, Hq * D), np.float32)
        rs = np.empty((T, Hq), np.float32)
    _load().oracle_attention_reuse(
        _pf(Q), _pf(Kf), _pf(Vf), ctypes.c_int(T), ctypes.c_int(Hq), ctypes.c_int(Hkv),
        ctypes.c_int(D), _pf(sk), _pf(sv), ctypes.c_int(C), _pi(ids), _pi(ul), ctypes.c_int(n_c),
        ctypes.c_int(ns), _pi(si), _pi(sh), _pf(O), _pf(rs) if want_row_sum else None)
    return (O, rs) if want_row_sum else O


def prefill_reuse(X, W, Hq: int, Hkv: int, D: int, theta: float, store_k=None, store_v=None,
                  slot_ids: Sequence[int] = (), used_len: Sequence[int] = (),
                  samples: Optional[Tuple[Sequence[int], Sequence[int]]] = None, extras: Optional[dict] = None):
    """One query, one layer: project+RoPE the fresh rows at offset L_pre, then attend.

    ``slot_ids=()`` is the full recomputation (plain causal prefill of a contiguous
    prompt).  ``extras``: keyword arguments of qkv_rope for the bias / QK-norm variants.  Returns (O, Kf, Vf, Q).
    """
    X = _f(X)
    W = _f(W)
    T, H = X.shape
    if extras:
        l_pre = int(np.sum(_i(used_len))) if len(slot_ids) else 0
        Q, Kf, Vf = qkv_rope(X, W, Hq, Hkv, D, l_pre, theta, **extras)
        O = attention_reuse(Q, Kf, Vf, store_k, store_v, slot_ids, used_len, samples=samples)
        return O, Kf, Vf, Q
    sk, sv, C = _store_args(store_k, store_v, Hkv, D)
    ids = _i(slot_ids)
    ul = _i(used_len)
    n_c = len(ids)
    if samples is not None:
        si, sh = _i(samples[0]), _i(samples[1])
        ns = len(si)
        O = np.empty((ns, D), np.float32)
    else:
        si = sh = None
        ns = 0
        O = np.empty((T, Hq * D), np.float32)
    Kf = np.empty((Hkv, T, D), np.float32)
    Vf = np.empty((Hkv, T, D), np.float32)
    Q = np.empty((Hq, T, D), np.float32)
    _load().oracle_prefill_reuse(
        _pf(X), _pf(W), ctypes.c_int(T), ctypes.c_int(H), ctypes.c_int(Hq), ctypes.c_int(Hkv),
        ctypes.c_int(D), ctypes.c_double(theta), _pf(sk), _pf(sv), ctypes.c_int(C), _pi(ids),
        _pi(ul), ctypes.c_int(n_c), ctypes.c_int(ns), _pi(si), _pi(sh), _pf(O), _pf(Kf), _pf(Vf),
        _pf(Q))
    return O, Kf, Vf, Q


def attend_stats(q, K, V):
    """(max, sum-exp, normalised output) of one query vector over an explicit key list."""
    q = _f(q)
    K = _f(K)
    V = _f(V)
    L, D = K.shape
    m = ctypes.c_double()
    l = ctypes.c_double()
    o = np.empty(D, np.float64)
    _load().oracle_attend_stats(_pf(q), _pf(K), _pf(V), ctypes.c_int(L), ctypes.c_int(D),
                                ctypes.byref(m), ctypes.byref(l), o.ctypes.data_as(_D))
    return m.value, l.value, o


def lse_merge(m_s, l_s, o_s) -> np.ndarray:
    m_s = np.ascontiguousarray(m_s, np.float64)
    l_s = np.ascontiguousarray(l_s, np.float64)
    o_s = np.ascontiguousarray(o_s, np.float64)
    n, D = o_s.shape
    o = np.empty(D, np.float64)
    _load().oracle_lse_merge(m_s.ctypes.data_as(_D), l_s.ctypes.data_as(_D), o_s.ctypes.data_as(_D),
                             ctypes.c_int(n), ctypes.c_int(D), o.ctypes.data_as(_D))
    return o


def rmsnorm(X, gain, eps: float) -> np.ndarray:
    X = _f(X)
    T, H = X.shape
    g = _f(gain) if gain is not None else None
    Y = np.empty_like(X)
    _load().oracle_rmsnorm(_pf(X), _pf(g), ctypes.c_int(T), ctypes.c_int(H), ctypes.c_double(eps), _pf(Y))
    return Y


def linear(X, W) -> np.ndarray:
    X = _f(X)
    W = _f(W)
    T, n_in = X.shape
    n_out = W.shape[0]
    assert W.shape[1] == n_in
    Y = np.empty((T, n_out), np.float32)
    _load().oracle_linear(_pf(X), _pf(W), ctypes.c_int(T), ctypes.c_int(n_in), ctypes.c_int(n_out), _pf(Y))
    return Y


def block_tail(h_in, attn, Wo, gain2, Wgate, Wup, Wdown, eps: float) -> np.ndarray:
    """Residual + o_proj, RMSNorm, SwiGLU MLP, residual on the fresh rows (App. B.1: the
    operations after attention run as usual)."""
    h_in = _f(h_in)
    attn = _f(attn)
    Wo, Wgate, Wup, Wdown = _f(Wo), _f(Wgate), _f(Wup), _f(Wdown)
    g2 = _f(gain2) if gain2 is not None else None
    T, H = h_in.shape
    n_attn = attn.shape[1]
    F = Wgate.shape[0]
    assert Wo.shape == (H, n_attn) and Wup.shape == (F, H) and Wdown.shape == (H, F)
    out = np.empty((T, H), np.float32)
    _load().oracle_block_tail(_pf(h_in), _pf(attn), _pf(Wo), _pf(g2), _pf(Wgate), _pf(Wup), _pf(Wdown),
                              ctypes.c_int(T), ctypes.c_int(H), ctypes.c_int(n_attn), ctypes.c_int(F),
                              ctypes.c_double(eps), _pf(out))
    return out


def block(h, gain1, Wqkv, Hq, Hkv, D, theta, Wo, gain2, Wgate, Wup, Wdown, eps,
          store_k=None, store_v=None, slot_ids=(), used_len=(), extras: Optional[dict] = None):
    """One full pre-norm block on one query's fresh rows.  Returns (h_out, Kf, Vf)."""
    n1 = rmsnorm(h, gain1, eps)
    O, Kf, Vf, _ = prefill_reuse(n1, Wqkv, Hq, Hkv, D, theta, store_k, store_v, slot_ids, used_len, extras=extras)
    return block_tail(h, O, Wo, gain2, Wgate, Wup, Wdown, eps), Kf, Vf
