"""Pins of the query-level match oracle (Sec. 4.2.1): cosine top-1 over all stored queries, hit if it
exceeds tau.  Pinned by an exact-duplicate invariant, scale invariance, one-hot closed forms, a scipy
cosine-distance cross-check and brute force on tiny banks."""
import numpy as np
from scipy.spatial.distance import cdist

import oracle
from paper_2601_11553_amd import workloads as wl


def test_config0_exact_duplicate_hits_with_similarity_one():
    w = wl.lookup_config0("f32")
    idx, sim, hit, sim2 = oracle.lookup(w.bank, w.probes, w.tau)
    assert idx[0] == w.source[0] and hit[0] == 1 and abs(sim[0] - 1.0) <= 1e-6
    # random unit vectors in dim 128 are far from each other: no hit at 0.9
    assert not hit[1:].any() and np.all(np.abs(sim[1:]) < 0.5)
    assert np.all(sim2 <= sim)


def test_matches_scipy_cosine_and_numpy_argmax():
    g = np.random.default_rng(2)
    E = g.standard_normal((300, 48)).astype(np.float32) * g.uniform(0.1, 5.0, (300, 1)).astype(np.float32)
    P = g.standard_normal((17, 48)).astype(np.float32)
    idx, sim, hit, sim2 = oracle.lookup(E, P, 0.4)
    S = 1.0 - cdist(P.astype(np.float64), E.astype(np.float64), metric="cosine")
    assert np.array_equal(idx, S.argmax(1))
    assert np.abs(sim - S.max(1)).max() < 1e-6
    assert np.abs(sim2 - np.sort(S, axis=1)[:, -2]).max() < 1e-6
    assert np.array_equal(hit.astype(bool), S.max(1).astype(np.float32) > np.float32(0.4))
    for p in range(3):
        assert np.abs(oracle.similarities(E, P[p]) - S[p]).max() < 1e-6


def test_scale_invariance_and_one_hot_closed_form():
    E = np.eye(16, dtype=np.float32) * np.arange(1, 17, dtype=np.float32)[:, None]
    p = np.zeros((2, 16), np.float32)
    p[0, 5] = 3.0
    p[0, 9] = 4.0           # cos with e_5 = 0.6, with e_9 = 0.8
    p[1] = p[0] * 123.0
    idx, sim, hit, sim2 = oracle.lookup(E, p, 0.7)
    assert list(idx) == [9, 9]
    assert np.abs(sim - 0.8).max() < 1e-7 and np.abs(sim2 - 0.6).max() < 1e-7
    assert list(hit) == [1, 1]
    _, _, hit_strict, _ = oracle.lookup(E, p[:1] * 0 + E[3:4], 1.0)
    assert hit_strict[0] == 0  # similarity exactly 1 does not EXCEED a threshold of 1


def test_lowest_index_wins_ties_and_degenerate_inputs():
    E = np.zeros((6, 4), np.float32)
    E[1] = [1, 0, 0, 0]
    E[2] = [2, 0, 0, 0]      # same direction as row 1: equal similarity
    E[4] = [0, 1, 0, 0]
    p = np.array([[5, 0, 0, 0], [0, 0, 0, 0]], np.float32)
    idx, sim, hit, sim2 = oracle.lookup(E, p, 0.5)
    assert idx[0] == 1 and sim[0] == 1.0 and sim2[0] == 1.0 and hit[0] == 1
    # zero-norm probe: every similarity is 0 -> index 0, no hit
    assert idx[1] == 0 and sim[1] == 0.0 and hit[1] == 0
    # empty bank
    idx, sim, hit, _ = oracle.lookup(np.zeros((0, 4), np.float32), p, 0.5)
    assert list(idx) == [-1, -1] and np.all(np.isneginf(sim)) and not hit.any()


def test_brute_force_python_loops_tiny():
    g = np.random.default_rng(9)
    E = g.standard_normal((7, 5))
    P = g.standard_normal((3, 5))
    idx, sim, _, _ = oracle.lookup(E.astype(np.float32), P.astype(np.float32), 0.0)
    E32, P32 = E.astype(np.float32).astype(np.float64), P.astype(np.float32).astype(np.float64)
    for p in range(3):
        best, bj = -2.0, -1
        for j in range(7):
            dot = sum(P32[p, k] * E32[j, k] for k in range(5))
            s = dot / (sum(x * x for x in P32[p]) ** 0.5 * sum(x * x for x in E32[j]) ** 0.5)
            if s > best:
                best, bj = s, j
        assert idx[p] == bj and abs(sim[p] - best) < 1e-6


def test_clustered_recipe_statistics_small():
    """The cfg-3 recipe at reduced size: perturbed copies find their source, by a wide margin."""
    w = wl.lookup_clustered("small3", 3, n_clusters=40, per_cluster=25, dim=1024, n_probes=64,
                            sigma_cluster=0.05, sigma_probe=0.02, tau=0.92, n_exact=4, n_near=4)
    idx, sim, hit, sim2 = oracle.lookup(w.bank, w.probes, w.tau)
    copies = w.source[:64] >= 0
    assert np.array_equal(idx[:64][copies], w.source[:64][copies])
    assert np.all(sim[:64][copies] - sim2[:64][copies] > 0.3)
    assert not hit[:64].any()                      # literal per-coordinate noise: cos ~ 0.84 < 0.92
    assert hit[64:].all() and np.array_equal(idx[64:], w.source[64:])
    assert np.all(np.abs(sim[64:68] - 1.0) < 1e-3)  # exact copies of fp16 rows
    assert np.all(np.abs(sim - w.tau) > 1e-3)      # threshold comparison is never marginal


def test_topk_pins():
    """k = 1 is the query-level match; against a float64 numpy ranking; sorted, distinct, lower row first on ties."""
    g = np.random.default_rng(8)
    E = g.standard_normal((200, 24)).astype(np.float32)
    E[50] = E[17] * 3.0          # same direction: exact tie in cosine
    E[120] = 0.0
    P = np.concatenate([g.standard_normal((6, 24)).astype(np.float32), E[17:18]])
    i1, s1, _, _ = oracle.lookup(E, P, 0.5)
    ik, sk, nxt = oracle.lookup_topk(E, P, 5)
    assert np.array_equal(ik[:, 0], i1) and np.allclose(sk[:, 0], s1, atol=1e-7)
    En = E.astype(np.float64)
    nrm = np.linalg.norm(En, axis=1)
    for p in range(P.shape[0]):
        q = P[p].astype(np.float64)
        cos = np.where(nrm > 0, En @ q / np.where(nrm > 0, nrm, 1) / np.linalg.norm(q), 0.0)
        top = np.sort(cos)[::-1][:6]
        assert np.allclose(sk[p], top[:5], atol=1e-6) and abs(nxt[p] - top[5]) < 1e-6
        assert len(set(ik[p])) == 5 and np.all(np.diff(sk[p]) <= 0)
    assert list(ik[6, :2]) == [17, 50]                                   # tie: lower row first
    ik2, sk2, nxt2 = oracle.lookup_topk(E[:3], P[:2], 5)                 # k beyond the bank
    assert np.all(ik2[:, 3:] == -1) and np.all(np.isneginf(sk2[:, 3:])) and np.all(np.isneginf(nxt2))


def test_refresh_scan_marks_exactly_the_queries_whose_topk_changes():
    """Sec. 4.1.3 stated directly: re-rank every stored query against old + new chunks; a query is outdated iff a new
    chunk is among its k best.  The scan (threshold = old k-th similarity) must mark the same queries."""
    g = np.random.default_rng(21)
    d, k = 32, 3
    chunks = g.standard_normal((150, d)).astype(np.float32)
    queries = g.standard_normal((90, d)).astype(np.float32)
    new = np.concatenate([g.standard_normal((5, d)), queries[[4, 40]] + 0.05 * g.standard_normal((2, d))]).astype(np.float32)
    _, sk, _ = oracle.lookup_topk(chunks, queries, k)
    best_sim, best_new, stale = oracle.refresh_scan(queries, new, sk[:, k - 1])
    idx_all, _, _ = oracle.lookup_topk(np.concatenate([chunks, new]), queries, k)
    entered = (idx_all >= chunks.shape[0]).any(axis=1)
    assert np.array_equal(stale.astype(bool), entered) and stale[4] and stale[40] and 2 <= stale.sum() < 60
    # float64 numpy for the maxima
    cn = new / np.linalg.norm(new, axis=1, keepdims=True)
    qn = queries / np.linalg.norm(queries, axis=1, keepdims=True)
    cos = qn.astype(np.float64) @ cn.astype(np.float64).T
    assert np.array_equal(best_new, cos.argmax(axis=1)) and np.allclose(best_sim, cos.max(axis=1), atol=1e-6)
