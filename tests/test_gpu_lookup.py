"""GPU parity of the query-level match (Sec. 4.2.1) against the CPU oracle, through the C ABI.

Bar: index and hit flag bit-exact, except that where the oracle's two best similarities differ by less
than 1e-4 any index whose oracle similarity is within 1e-4 of the best is accepted; similarity within 2e-5.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2601_11553_amd import workloads as wl
from paper_2601_11553_amd.binding import Percache, PercacheError

from gpu_util import DEV, f16, host

pytestmark = pytest.mark.gpu


def _ctx(capacity, dim):
    return Percache(n_layers=1, hidden=256, n_q_heads=4, n_kv_heads=2, head_dim=64, n_slots=1, slot_capacity=64,
                    max_pos=64, bank_capacity=capacity, emb_dim=dim, device=DEV)


def _compare(bank, probes, tau, idx, sim, hit):
    o_idx, o_sim, o_hit, o_sim2 = oracle.lookup(bank, probes, tau)
    idx, sim, hit = idx.cpu().numpy(), sim.cpu().numpy(), hit.cpu().numpy()
    assert np.abs(sim - o_sim).max() < 2e-5, np.abs(sim - o_sim).max()
    clear = (o_sim - o_sim2) >= 1e-4
    assert np.array_equal(idx[clear], o_idx[clear]), np.nonzero(idx[clear] != o_idx[clear])
    for p in np.nonzero(~clear)[0]:
        s = oracle.similarities(bank, probes[p])
        assert o_sim[p] - s[idx[p]] < 1e-4
    assert np.array_equal(hit, o_hit)
    return int((~clear).sum())


def test_config0_lookup():
    w = wl.lookup_config0("f16")
    pc = _ctx(64, 128)
    pc.percache_bank_put(0, f16(w.bank))
    assert pc.percache_bank_size() == 64
    idx, sim, hit = pc.percache_lookup(f16(w.probes), w.tau)
    torch.cuda.synchronize()
    _compare(w.bank, w.probes, w.tau, idx, sim, hit)
    assert idx[0].item() == w.source[0] and hit[0].item() == 1 and abs(sim[0].item() - 1.0) < 1e-3
    assert hit[1:].sum().item() == 0


@pytest.mark.parametrize("n_clusters,per_cluster,n_probes", [(37, 27, 70), (50, 100, 16), (13, 5, 1), (64, 64, 130)])
def test_clustered_ragged_sizes(n_clusters, per_cluster, n_probes):
    """Bank sizes that are not multiples of the 16-row block, probe counts across the 32-probe pass."""
    w = wl.lookup_clustered("t", 11, n_clusters, per_cluster, 1024, n_probes, 0.05, 0.02, 0.92, n_exact=3, n_near=3)
    N = w.bank.shape[0]
    pc = _ctx(N + 5, 1024)
    # two puts: appends must continue where the first stopped
    cut = N // 3
    pc.percache_bank_put(0, f16(w.bank[:cut]))
    pc.percache_bank_put(cut, f16(w.bank[cut:]))
    idx, sim, hit = pc.percache_lookup(f16(w.probes), w.tau)
    torch.cuda.synchronize()
    _compare(w.bank, w.probes, w.tau, idx, sim, hit)
    assert hit[-6:].all()


@pytest.mark.parametrize("dim,n_probes", [(64, 5), (64, 20), (192, 7), (256, 31), (384, 9), (384, 25), (768, 3), (768, 33), (2048, 20),
                                          (512, 100), (512, 129), (768, 260), (1024, 128)])   # 512/100 and 1024/128: the 128-probe pass
def test_every_embedding_width(dim, n_probes):
    """Each row-chunk width of the streaming kernel (one chunk per row up to 256 elements, several beyond),
    with one and two probe blocks, on a bank long enough that every wavefront streams many row blocks."""
    w = wl.lookup_clustered("w", 100 + dim, 1031, 97, dim, n_probes, 0.05, 0.02, 0.92, n_exact=1, n_near=1)
    N = w.bank.shape[0]
    pc = _ctx(N, dim)
    pc.percache_bank_put(0, f16(w.bank))
    idx, sim, hit = pc.percache_lookup(f16(w.probes), w.tau)
    torch.cuda.synchronize()
    _compare(w.bank, w.probes, w.tau, idx, sim, hit)


@pytest.mark.parametrize("seed", list(range(16)))
def test_seeded_random_bank_shapes(seed):
    """Embedding width, bank size (ragged against every block size) and probe count drawn from a seed: every kernel
    of the lookup (one or two probe blocks per pass, the 128-probe pass, the matrix-product kernel) meets odd sizes."""
    g = np.random.default_rng(3000 + seed)
    dim = int(g.choice([64, 128, 192, 256, 384, 512, 768, 1024]))
    n_clusters = int(g.integers(1, 60))
    per_cluster = int(g.integers(1, 70))
    n_probes = int(g.choice([1, 5, 16, 17, 32, 33, 100, 128, 129, 200]))
    w = wl.lookup_clustered("r", 3100 + seed, n_clusters, per_cluster, dim, n_probes, 0.05, 0.02, 0.92, n_exact=1, n_near=1)
    pc = _ctx(w.bank.shape[0], dim)
    pc.percache_bank_put(0, f16(w.bank))
    idx, sim, hit = pc.percache_lookup(f16(w.probes), w.tau)
    torch.cuda.synchronize()
    _compare(w.bank, w.probes, w.tau, idx, sim, hit)


def test_ties_zero_vectors_and_empty_bank():
    d = 128
    g = np.random.default_rng(5)
    bank = wl.round_f16(g.standard_normal((40, d)).astype(np.float32))
    bank[7] = 0.0                    # zero-norm row: similarity 0
    bank[30] = bank[12] * 2.0        # same direction as row 12: exact tie, lowest index wins
    probes = np.stack([bank[12], np.zeros(d, np.float32), bank[30] * 0.5, -bank[3]]).astype(np.float32)
    pc = _ctx(64, d)
    idx, sim, hit = pc.percache_lookup(f16(probes), 0.5)
    torch.cuda.synchronize()
    assert idx.cpu().tolist() == [-1] * 4 and not hit.any().item() and torch.isneginf(sim).all().item()
    pc.percache_bank_put(0, f16(bank))
    idx, sim, hit = pc.percache_lookup(f16(probes), 0.5)
    torch.cuda.synchronize()
    o_idx, o_sim, o_hit, _ = oracle.lookup(bank, probes, 0.5)
    assert idx.cpu().tolist() == o_idx.tolist()
    assert idx[0].item() == 12 and idx[2].item() == 12 and idx[1].item() == 0
    assert np.array_equal(hit.cpu().numpy(), o_hit)
    assert np.abs(sim.cpu().numpy() - o_sim).max() < 2e-5


@pytest.mark.parametrize("n_probes,k", [(40, 1), (128, 1), (40, 8)])
def test_ties_and_zero_vectors_in_the_128_probe_pass(n_probes, k):
    """Exact ties (lowest row wins), a zero row, a zero probe and a ragged last 32-row block, at a width and probe
    counts the 128-probe pass takes."""
    d = 512
    g = np.random.default_rng(15)
    bank = wl.round_f16(g.standard_normal((75, d)).astype(np.float32))
    bank[7] = 0.0
    bank[40] = bank[12] * 2.0
    bank[70] = bank[12] * 0.5
    probes = wl.round_f16(g.standard_normal((n_probes, d)).astype(np.float32))
    probes[0] = bank[12]
    probes[1] = 0.0
    probes[n_probes - 1] = bank[70]
    pc = _ctx(128, d)
    pc.percache_bank_put(0, f16(bank))
    if k == 1:
        idx, sim, hit = pc.percache_lookup(f16(probes), 0.5)
        torch.cuda.synchronize()
        o_idx, o_sim, o_hit, _ = oracle.lookup(bank, probes, 0.5)
        assert idx.cpu().tolist() == o_idx.tolist()
        assert idx[0].item() == 12 and idx[n_probes - 1].item() == 12 and idx[1].item() == 0
        assert np.array_equal(hit.cpu().numpy(), o_hit)
        assert np.abs(sim.cpu().numpy() - o_sim).max() < 2e-5
    else:
        idx, sim = pc.percache_lookup_topk(f16(probes), k)
        torch.cuda.synchronize()
        assert idx[0, :3].cpu().tolist() == [12, 40, 70] and idx[1, :k].cpu().tolist() == list(range(k))
        _compare_topk(bank, probes, k, idx, sim)


@pytest.mark.parametrize("n_rows,d,n_probes", [(75, 512, 200), (300, 64, 256), (1031, 192, 600), (5000, 1024, 1000),
                                                (257, 128, 1152), (256, 256, 768), (3, 64, 250),
                                                (1031, 192, 150), (300, 64, 100), (5000, 1024, 170), (75, 128, 33), (600, 256, 300),
                                                (700, 128, 3000), (1, 64, 300), (2100, 2048, 384)])
def test_ties_zero_vectors_and_ragged_ends_in_the_256_row_tiles(n_rows, d, n_probes):
    """The matrix-product kernel on 256-row tiles (best match only; 256-probe tiles where the probes fill them to three
    quarters, 128-probe tiles with the deeper ring otherwise; more probe tiles than CUs / 8; a one-row bank): exact ties
    (lowest row wins) inside one lane's rows, across lanes, across wavefronts and across tiles; a zero row and a zero probe; banks that end inside a tile, inside a 32-row block, or hold fewer
    rows than one block; a single k-step (64 elements) and many."""
    g = np.random.default_rng(n_rows + d)
    bank = wl.round_f16(g.standard_normal((n_rows, d)).astype(np.float32))
    probes = wl.round_f16(g.standard_normal((n_probes, d)).astype(np.float32))
    probes[1] = 0.0
    if n_rows >= 75:
        bank[7] = 0.0
        bank[40] = bank[12] * 2.0     # same cosine as row 12: another 32-row block, another wavefront
        bank[13] = bank[12] * 0.5     # the next row: same lane or its neighbour
        bank[70] = bank[12] * 0.25
        probes[0] = bank[12]
        probes[n_probes - 1] = bank[70]
    if n_rows >= 300:
        bank[n_rows - 1] = bank[12] * 4.0   # the bank's last row, in a later tile: the earlier tile's row keeps the match
        bank[290] = bank[280]               # a tie that the later tile opens and wins by row order
        probes[5] = bank[290]
    pc = _ctx(n_rows + 3, d)
    pc.percache_bank_put(0, f16(bank))
    idx, sim, hit = pc.percache_lookup(f16(probes), 0.5)
    torch.cuda.synchronize()
    o_idx, o_sim, o_hit, o_sim2 = oracle.lookup(bank, probes, 0.5)
    if n_rows >= 75:
        assert idx[0].item() == 12 and idx[n_probes - 1].item() == 12
    if n_rows >= 300:
        assert idx[5].item() == 280
    assert idx[1].item() == 0
    _compare(bank, probes, 0.5, idx, sim, hit)
    # scaled copies have equal cosines only up to rounding of the norms: the planted rows are checked above, the rest by _compare


def test_overwrite_rows_and_error_paths():
    d = 128
    g = np.random.default_rng(6)
    bank = wl.round_f16(g.standard_normal((32, d)).astype(np.float32))
    pc = _ctx(64, d)
    pc.percache_bank_put(0, f16(bank))
    new = wl.round_f16(g.standard_normal((4, d)).astype(np.float32))
    pc.percache_bank_put(10, f16(new))
    bank[10:14] = new
    probes = np.concatenate([new[:2], bank[:2]])
    idx, sim, hit = pc.percache_lookup(f16(probes), 0.9)
    torch.cuda.synchronize()
    assert idx.cpu().tolist() == [10, 11, 0, 1] and hit.all().item()
    with pytest.raises(PercacheError) as e:
        pc.percache_bank_put(32, f16(np.concatenate([bank, bank[:8]])))   # 32 + 40 rows > capacity 64
    assert e.value.status == -5
    with pytest.raises(PercacheError) as e:
        pc.percache_bank_put(40, f16(bank[:1]))                           # would leave a hole
    assert e.value.status == -1
    assert pc.percache_bank_size() == 32
    nobank = Percache(n_layers=1, hidden=256, n_q_heads=4, n_kv_heads=2, head_dim=64, n_slots=1, slot_capacity=64,
                      max_pos=64, device=DEV)
    with pytest.raises(PercacheError) as e:
        nobank.percache_lookup(f16(probes), 0.9)
    assert e.value.status == -2


def test_config3_full_size_every_probe():
    """200k x 1024 fp16 bank, the 1024 probes of the recipe plus the hit-branch block; every one of the 1152 probes
    goes through the oracle's exhaustive scan."""
    w = wl.lookup_config3(n_exact=64, n_near=64)
    N, d = w.bank.shape
    P = w.probes.shape[0]
    pc = _ctx(N, d)
    pc.percache_bank_put(0, f16(w.bank))
    probes_dev = f16(w.probes)
    idx, sim, hit = pc.percache_lookup(probes_dev, w.tau)
    torch.cuda.synchronize()
    # one probe at a time (the paper's case) must give the same answers as the batched call
    for p in (0, 513, P - 1):
        i1, s1, h1 = pc.percache_lookup(probes_dev[p:p + 1], w.tau)
        torch.cuda.synchronize()
        assert i1.item() == idx[p].item() and h1.item() == hit[p].item() and abs(s1.item() - sim[p].item()) < 2e-6
    # 128 probes go through the 128-probe pass, the full call through the matrix-product kernel: same answers
    for lo in (0, 1000):
        i3, s3, h3 = pc.percache_lookup(probes_dev[lo:lo + 128], w.tau)
        torch.cuda.synchronize()
        assert torch.equal(i3, idx[lo:lo + 128]) and torch.equal(h3, hit[lo:lo + 128]) and (s3 - sim[lo:lo + 128]).abs().max().item() < 2e-6
    print("cfg3: oracle scan of all probes ...", flush=True)
    n_near_ties = _compare(w.bank, w.probes, w.tau, idx, sim, hit)
    print(f"cfg3: {P} probes through the oracle, {n_near_ties} with top-2 gap < 1e-4; hits in main block "
          f"{int(hit[:1024].sum())}/1024, in hit block {int(hit[1024:].sum())}/128", flush=True)
    idx_h, hit_h = idx.cpu().numpy(), hit.cpu().numpy()
    copies = w.source[:1024] >= 0
    assert np.array_equal(idx_h[:1024][copies], w.source[:1024][copies])   # perturbed copies find their source
    assert hit_h[1024:].all() and np.array_equal(idx_h[1024:], w.source[1024:])


def _compare_topk(bank, probes, k, idx, sim):
    o_idx, o_sim, o_next = oracle.lookup_topk(bank, probes, k)
    idx, sim = idx.cpu().numpy(), sim.cpu().numpy()
    fin = np.isfinite(o_sim)
    assert np.array_equal(np.isfinite(sim), fin) and np.array_equal(idx[~fin], o_idx[~fin])
    assert np.abs(sim[fin] - o_sim[fin]).max() < 2e-5
    n_loose = 0
    for p in range(probes.shape[0]):
        assert len(set(idx[p][fin[p]])) == int(fin[p].sum())                      # no row twice
        ranked = np.concatenate([o_sim[p], [o_next[p]]])
        s_all = None
        for j in range(k):
            if not fin[p, j]:
                continue
            clear = (j == 0 or ranked[j - 1] - ranked[j] >= 1e-4) and ranked[j] - ranked[j + 1] >= 1e-4
            if clear:
                assert idx[p, j] == o_idx[p, j], (p, j)
            else:                                                                   # near-tie: any row that close is right
                if s_all is None:
                    s_all = oracle.similarities(bank, probes[p])
                assert abs(s_all[idx[p, j]] - o_sim[p, j]) < 1e-4, (p, j)
                n_loose += 1
    return n_loose


@pytest.mark.parametrize("dim,n_probes,k", [(1024, 40, 8), (1024, 3, 3), (128, 17, 5), (384, 33, 2), (64, 5, 8), (1024, 150, 8), (192, 300, 4)])
def test_topk_vs_oracle(dim, n_probes, k):
    w = wl.lookup_clustered("k", 300 + dim, 523, 41, dim, n_probes, 0.05, 0.02, 0.92, n_exact=1, n_near=1)
    pc = _ctx(w.bank.shape[0], dim)
    pc.percache_bank_put(0, f16(w.bank))
    idx, sim = pc.percache_lookup_topk(f16(w.probes), k)
    i1, s1, _ = pc.percache_lookup(f16(w.probes), w.tau)
    torch.cuda.synchronize()
    loose = _compare_topk(w.bank, w.probes, k, idx, sim)
    assert torch.equal(idx[:, 0], i1) and torch.equal(sim[:, 0], s1)              # rank 1 is the query-level match
    print(f"top-{k}: {loose} near-tie entries judged by similarity", flush=True)


def test_topk_ties_small_bank_and_errors():
    d = 128
    g = np.random.default_rng(12)
    bank = wl.round_f16(g.standard_normal((5, d)).astype(np.float32))
    bank[3] = bank[1] * 2.0
    probes = np.stack([bank[1], bank[4]])
    pc = _ctx(16, d)
    idx, sim = pc.percache_lookup_topk(f16(probes), 4)
    torch.cuda.synchronize()
    assert (idx == -1).all().item() and torch.isneginf(sim).all().item()           # empty bank
    pc.percache_bank_put(0, f16(bank))
    idx, sim = pc.percache_lookup_topk(f16(probes), 8)
    torch.cuda.synchronize()
    assert idx[0, :2].tolist() == [1, 3] and (idx[:, 5:] == -1).all().item() and torch.isneginf(sim[:, 5:]).all().item()
    o_idx, o_sim, _ = oracle.lookup_topk(bank, probes, 8)
    assert np.array_equal(idx.cpu().numpy(), o_idx)
    with pytest.raises(PercacheError) as e:
        pc.percache_lookup_topk(f16(probes), 9)
    assert e.value.status == -2


@pytest.mark.parametrize("dim,n_new", [(1024, 5), (1024, 70), (128, 33)])
def test_refresh_scan_vs_oracle(dim, n_new):
    """Cache refresh (Sec. 4.1.3): stored queries in the bank, thresholds from the oracle's top-k over the chunk embeddings,
    new chunks scanned; against the oracle's row-by-row definition, and against a direct re-ranking."""
    k = 3
    wq = wl.lookup_clustered("q", 500 + dim, 97, 53, dim, 4, 0.05, 0.02, 0.92)       # bank rows = stored queries
    wc = wl.lookup_clustered("c", 600 + dim, 97, 31, dim, 4, 0.05, 0.02, 0.92)       # bank rows = knowledge chunks
    g = np.random.default_rng(dim + n_new)
    pick = g.integers(0, wq.bank.shape[0], size=n_new)
    new = wl.round_f16(wq.bank[pick] + 0.03 * g.standard_normal((n_new, dim)).astype(np.float32))
    _, o_sk, _ = oracle.lookup_topk(wc.bank, wq.bank, k)                              # each stored query's best chunks
    kth = torch.from_numpy(np.ascontiguousarray(o_sk[:, k - 1], np.float32)).to(DEV)
    qctx = _ctx(wq.bank.shape[0], dim)
    qctx.percache_bank_put(0, f16(wq.bank))
    best_sim, best_new, stale = qctx.percache_bank_refresh_scan(f16(new), kth)
    torch.cuda.synchronize()
    o_sim, o_new, o_stale = oracle.refresh_scan(wq.bank, new, kth.cpu().numpy())
    bs, bn, st = best_sim.cpu().numpy(), best_new.cpu().numpy(), stale.cpu().numpy()
    assert np.abs(bs - o_sim).max() < 2e-5
    loose = 0
    for j in np.nonzero(bn != o_new)[0]:                                              # only near-ties may differ
        s = oracle.similarities(new, wq.bank[j])
        assert o_sim[j] - s[bn[j]] < 1e-4
        loose += 1
    margin = np.abs(o_sim - kth.cpu().numpy()) > 2e-5           # the similarity tolerance: closer than that, either decision
    assert np.array_equal(st[margin], o_stale[margin])
    assert st[pick].all()                                                             # a near copy of a query enters its top-k
    print(f"refresh scan: {int(st.sum())}/{st.size} stored queries outdated, {loose} near-tie indices", flush=True)
