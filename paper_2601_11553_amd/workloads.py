"""Seeded synthetic inputs shaped like the paper's mobile-RAG prompts.

The paper's prompts are "system prompt + top-k retrieved knowledge chunks + a
short user query" (Sec. 2.1, Sec. 5.3); their text, datasets and trained
weights are not available, so every tensor here is drawn from a seeded
generator with that *structure*: k cached chunks of C tokens each followed by a
short fresh suffix, and a bank of clustered unit-norm query embeddings.

This module holds NO arithmetic of the method (no projection, RoPE, softmax or
similarity): only random draws, rounding to the storage dtype, and bookkeeping.
Both the HIP path and the CPU oracle are fed from it; neither is imported here.

All arrays are numpy float32 whose values are exactly representable in the
storage dtype ("bf16" / "f16"), so widening on one side and narrowing on the
other lose nothing.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Dict, Optional, Tuple

import numpy as np


# ----------------------------------------------------------------------------
# storage-dtype rounding (round to nearest even)
# ----------------------------------------------------------------------------
def round_bf16(a: np.ndarray) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = ((u + bias) & np.uint32(0xFFFF0000)).astype(np.uint32)
    return r.view(np.float32).reshape(a.shape)


def round_f16(a: np.ndarray) -> np.ndarray:
    return np.asarray(a, dtype=np.float32).astype(np.float16).astype(np.float32)


def round_to(a: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return round_bf16(a)
    if dtype == "f16":
        return round_f16(a)
    if dtype == "f32":
        return np.ascontiguousarray(a, dtype=np.float32)
    raise ValueError(dtype)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of an array already rounded with round_bf16."""
    return (np.ascontiguousarray(a, dtype=np.float32).view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def _rng(seed: int, tag: int, idx: int = 0) -> np.random.Generator:
    return np.random.default_rng([int(seed), int(tag), int(idx)])


_TAG_X, _TAG_W, _TAG_SLOT, _TAG_IDS, _TAG_BANK, _TAG_PROBE, _TAG_CENTER, _TAG_LAYER = range(1, 9)


# ----------------------------------------------------------------------------
# cache-reusing prefill workloads
# ----------------------------------------------------------------------------
@dataclass
class PrefillWorkload:
    name: str
    seed: int
    dtype: str          # storage dtype of X, W and the K/V store
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    batch: int
    t_fresh: int
    n_chunks: int
    chunk_tokens: int   # slot capacity C
    n_slots: int
    rope_theta: float = 10000.0
    n_layers: int = 1
    x_scale: float = 1.0
    X: np.ndarray = field(default=None, repr=False)          # [B, T_f, hidden]
    Wqkv: np.ndarray = field(default=None, repr=False)       # [(Hq+2Hkv)*D, hidden]
    slot_ids: np.ndarray = field(default=None, repr=False)   # [B, n_chunks] int32
    used_len: np.ndarray = field(default=None, repr=False)   # [B, n_chunks] int32

    @property
    def l_pre(self) -> np.ndarray:
        return self.used_len.sum(axis=1)

    @property
    def max_pos(self) -> int:
        return int(self.n_chunks * self.chunk_tokens + self.t_fresh)

    def slot_kv(self, slot: int, layer: int = 0) -> Tuple[np.ndarray, np.ndarray]:
        """K and V of one slot for one layer, each [Hkv, C, D] ~ N(0,1) in the storage dtype."""
        g = _rng(self.seed, _TAG_SLOT, layer * 1_000_003 + slot)
        shape = (self.n_kv_heads, self.chunk_tokens, self.head_dim)
        k = round_to(g.standard_normal(shape, dtype=np.float32), self.dtype)
        v = round_to(g.standard_normal(shape, dtype=np.float32), self.dtype)
        return k, v

    def slots_kv(self, slots, layer: int = 0, workers: int = 8) -> Dict[int, Tuple[np.ndarray, np.ndarray]]:
        slots = [int(s) for s in slots]
        with ThreadPoolExecutor(max_workers=workers) as ex:
            out = list(ex.map(lambda s: self.slot_kv(s, layer), slots))
        return dict(zip(slots, out))

    def compact_store(self, b: int, layer: int = 0):
        """The slots query ``b`` uses, packed as a small store plus remapped ids (oracle input)."""
        ids = [int(s) for s in self.slot_ids[b]]
        kv = self.slots_kv(ids, layer)
        sk = np.stack([kv[s][0] for s in ids]) if ids else np.zeros((0, self.n_kv_heads, self.chunk_tokens, self.head_dim), np.float32)
        sv = np.stack([kv[s][1] for s in ids]) if ids else sk.copy()
        return sk, sv, np.arange(len(ids), dtype=np.int32)


def make_prefill(name: str, seed: int, dtype: str, hidden: int, n_q_heads: int, n_kv_heads: int,
                 head_dim: int, batch: int, t_fresh: int, n_chunks: int, chunk_tokens: int, n_slots: int,
                 rope_theta: float = 10000.0, last_used_len: Optional[int] = None,
                 x_scale: float = 1.0, n_layers: int = 1) -> PrefillWorkload:
    """X ~ N(0, x_scale^2), Wqkv ~ N(0, 0.02^2); per query ``n_chunks`` distinct random slots."""
    w = PrefillWorkload(name, seed, dtype, hidden, n_q_heads, n_kv_heads, head_dim, batch, t_fresh,
                        n_chunks, chunk_tokens, n_slots, rope_theta, n_layers, x_scale)
    w.X = round_to(_rng(seed, _TAG_X).standard_normal((batch, t_fresh, hidden), dtype=np.float32) * np.float32(x_scale), dtype)
    n_out = (n_q_heads + 2 * n_kv_heads) * head_dim
    w.Wqkv = round_to(_rng(seed, _TAG_W).standard_normal((n_out, hidden), dtype=np.float32) * np.float32(0.02), dtype)
    g = _rng(seed, _TAG_IDS)
    w.slot_ids = np.stack([g.permutation(n_slots)[:n_chunks] for _ in range(batch)]).astype(np.int32).reshape(batch, n_chunks)
    w.used_len = np.full((batch, n_chunks), chunk_tokens, np.int32)
    if last_used_len is not None and n_chunks:
        w.used_len[:, -1] = last_used_len
    return w


def config1(**over) -> PrefillWorkload:
    """Qwen3-0.6B-shaped layer, batch 1, 4 cached chunks x 512 tokens, 64 fresh tokens."""
    kw = dict(name="cfg1", seed=1, dtype="bf16", hidden=1024, n_q_heads=16, n_kv_heads=8, head_dim=128,
              batch=1, t_fresh=64, n_chunks=4, chunk_tokens=512, n_slots=16)
    kw.update(over)
    return make_prefill(**kw)


def config2(**over) -> PrefillWorkload:
    """28-layer Qwen3-0.6B-shaped stack, 8 cached chunks x 512 from a 256-slot store, 128 fresh tokens."""
    kw = dict(name="cfg2", seed=2, dtype="bf16", hidden=1024, n_q_heads=16, n_kv_heads=8, head_dim=128,
              batch=1, t_fresh=128, n_chunks=8, chunk_tokens=512, n_slots=256, n_layers=28)
    kw.update(over)
    return make_prefill(**kw)


def config4(**over) -> PrefillWorkload:
    """3B-shaped GQA layer, batch 8, 16 cached chunks x 1024 tokens from a 1024-slot store, 256 fresh tokens."""
    kw = dict(name="cfg4", seed=4, dtype="bf16", hidden=3072, n_q_heads=24, n_kv_heads=8, head_dim=128,
              batch=8, t_fresh=256, n_chunks=16, chunk_tokens=1024, n_slots=1024)
    kw.update(over)
    return make_prefill(**kw)


@dataclass
class TinyLayerWorkload:
    """Config 0: one tiny layer whose cached K/V come from running the same layer on the chunk tokens."""
    seed: int
    dtype: str
    hidden: int = 256
    n_q_heads: int = 4
    n_kv_heads: int = 2
    head_dim: int = 64
    n_chunks: int = 2
    chunk_tokens: int = 64
    t_fresh: int = 16
    rope_theta: float = 10000.0
    prompt: np.ndarray = field(default=None, repr=False)   # [n_chunks*C + T_f, hidden]: chunk rows then fresh rows
    Wqkv: np.ndarray = field(default=None, repr=False)

    @property
    def l_pre(self) -> int:
        return self.n_chunks * self.chunk_tokens


def config0(dtype: str = "f32", seed: int = 0, **over) -> TinyLayerWorkload:
    w = TinyLayerWorkload(seed=seed, dtype=dtype, **over)
    total = w.n_chunks * w.chunk_tokens + w.t_fresh
    w.prompt = round_to(_rng(seed, _TAG_X).standard_normal((total, w.hidden), dtype=np.float32), dtype)
    n_out = (w.n_q_heads + 2 * w.n_kv_heads) * w.head_dim
    w.Wqkv = round_to(_rng(seed, _TAG_W).standard_normal((n_out, w.hidden), dtype=np.float32) * np.float32(0.02), dtype)
    return w


@dataclass
class StackWeights:
    """Weights of one pre-norm block: Wqkv, Wo, RMSNorm gains, SwiGLU MLP."""
    Wqkv: np.ndarray
    Wo: np.ndarray
    gain1: np.ndarray
    gain2: np.ndarray
    Wgate: np.ndarray
    Wup: np.ndarray
    Wdown: np.ndarray


def stack_weights(seed: int, layer: int, hidden: int, n_q_heads: int, n_kv_heads: int, head_dim: int,
                  ffn: int, dtype: str = "bf16") -> StackWeights:
    g = _rng(seed, _TAG_LAYER, layer)

    def n(shape, s=0.02):
        return round_to(g.standard_normal(shape, dtype=np.float32) * np.float32(s), dtype)

    n_out = (n_q_heads + 2 * n_kv_heads) * head_dim
    return StackWeights(
        Wqkv=n((n_out, hidden)), Wo=n((hidden, n_q_heads * head_dim)),
        gain1=round_to(1.0 + 0.1 * g.standard_normal(hidden, dtype=np.float32), dtype),
        gain2=round_to(1.0 + 0.1 * g.standard_normal(hidden, dtype=np.float32), dtype),
        Wgate=n((ffn, hidden)), Wup=n((ffn, hidden)), Wdown=n((hidden, ffn)))


# ----------------------------------------------------------------------------
# query-level match workloads
# ----------------------------------------------------------------------------
@dataclass
class LookupWorkload:
    name: str
    seed: int
    dtype: str
    tau: float
    bank: np.ndarray = field(default=None, repr=False)     # [N, d]
    probes: np.ndarray = field(default=None, repr=False)   # [P, d]
    source: np.ndarray = field(default=None, repr=False)   # [P] bank row a probe was derived from, else -1


def _normalize(a: np.ndarray) -> np.ndarray:
    return a / np.linalg.norm(a, axis=-1, keepdims=True)


def lookup_config0(dtype: str = "f32", seed: int = 0) -> LookupWorkload:
    """64 unit-norm Gaussian embeddings of dim 128; probes = 1 exact copy + 3 random; tau 0.9."""
    g = _rng(seed, _TAG_BANK)
    bank = round_to(_normalize(g.standard_normal((64, 128))).astype(np.float32), dtype)
    gp = _rng(seed, _TAG_PROBE)
    src = int(gp.integers(0, 64))
    rnd = round_to(_normalize(gp.standard_normal((3, 128))).astype(np.float32), dtype)
    probes = np.concatenate([bank[src:src + 1], rnd], axis=0)
    return LookupWorkload("lookup0", seed, dtype, 0.9, bank, probes, np.array([src, -1, -1, -1], np.int32))


def lookup_clustered(name: str, seed: int, n_clusters: int, per_cluster: int, dim: int, n_probes: int,
                     sigma_cluster: float, sigma_probe: float, tau: float, dtype: str = "f16",
                     n_exact: int = 0, n_near: int = 0, sigma_near: float = 0.005) -> LookupWorkload:
    """Bank = per_cluster draws normalize(c + sigma_cluster*g) around each of n_clusters unit centres.

    Probes: half perturbed copies normalize(e_j + sigma_probe*g) of random bank rows, half fresh draws
    from random clusters, shuffled; then optionally ``n_exact`` exact copies and ``n_near`` copies with
    the smaller noise ``sigma_near`` appended (these exercise the hit branch).  Noise sigmas are per
    coordinate.
    """
    gc = _rng(seed, _TAG_CENTER)
    centers = _normalize(gc.standard_normal((n_clusters, dim), dtype=np.float32))
    gb = _rng(seed, _TAG_BANK)
    N = n_clusters * per_cluster
    bank = np.empty((N, dim), np.float32)
    step = max(1, 4096 // per_cluster)
    for c0 in range(0, n_clusters, step):
        c1 = min(n_clusters, c0 + step)
        noise = gb.standard_normal(((c1 - c0) * per_cluster, dim), dtype=np.float32) * np.float32(sigma_cluster)
        rows = np.repeat(centers[c0:c1], per_cluster, axis=0) + noise
        bank[c0 * per_cluster:c1 * per_cluster] = _normalize(rows)
    # interleave clusters so that neighbours in memory are unrelated
    perm = gb.permutation(N)
    bank = round_to(bank[perm], dtype)
    gp = _rng(seed, _TAG_PROBE)
    n_copy = n_probes // 2
    n_new = n_probes - n_copy
    src = gp.integers(0, N, size=n_copy)
    copies = _normalize(bank[src] + gp.standard_normal((n_copy, dim), dtype=np.float32) * np.float32(sigma_probe))
    cl = gp.integers(0, n_clusters, size=n_new)
    fresh = _normalize(centers[cl] + gp.standard_normal((n_new, dim), dtype=np.float32) * np.float32(sigma_cluster))
    probes = np.concatenate([copies, fresh], axis=0)
    source = np.concatenate([src, -np.ones(n_new, np.int64)])
    order = gp.permutation(n_probes)
    probes, source = probes[order], source[order]
    if n_exact or n_near:
        se = gp.integers(0, N, size=n_exact)
        sn = gp.integers(0, N, size=n_near)
        near = _normalize(bank[sn] + gp.standard_normal((n_near, dim), dtype=np.float32) * np.float32(sigma_near))
        probes = np.concatenate([probes, bank[se], near], axis=0)
        source = np.concatenate([source, se, sn])
    return LookupWorkload(name, seed, dtype, tau, bank, round_to(probes.astype(np.float32), dtype),
                          source.astype(np.int32))


def lookup_config3(**over) -> LookupWorkload:
    """200k embeddings dim 1024 fp16 from 2000 clusters (sigma 0.05), 1024 probes (copy noise 0.02), tau 0.92."""
    kw = dict(name="cfg3", seed=3, n_clusters=2000, per_cluster=100, dim=1024, n_probes=1024,
              sigma_cluster=0.05, sigma_probe=0.02, tau=0.92, dtype="f16")
    kw.update(over)
    return lookup_clustered(**kw)
