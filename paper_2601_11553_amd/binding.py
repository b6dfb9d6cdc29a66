"""Thin ctypes binding over libpercache.so: argument marshalling only.

Every step of the hot path runs in the HIP kernels behind the C ABI declared in
``include/percache.h``; the functions here have the same names and only turn torch
tensors into device pointers (``.data_ptr()``), numpy/int lists into host arrays, and the
current torch stream into a ``hipStream_t``.  There is no CPU fallback: if the shared library
is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpercache.so")

PC_OK = 0
STATUS_NAMES = {0: "PC_OK", -1: "PC_EINVAL", -2: "PC_ESHAPE", -3: "PC_ESLOT", -4: "PC_ELEN", -5: "PC_ENOMEM", -6: "PC_EHIP"}

EXPORTS = [
    "percache_arena_bytes", "percache_create", "percache_destroy", "percache_last_error",
    "percache_bank_put", "percache_bank_size", "percache_lookup_workspace_bytes", "percache_lookup",
    "percache_lookup_noalloc", "percache_lookup_topk", "percache_bank_refresh_scan",
    "percache_kv_put", "percache_kv_put_batch", "percache_kv_get", "percache_kv_get_batch", "percache_kv_evict", "percache_kv_len",
    "percache_kv_slice", "percache_kv_append", "percache_stack_workspace_bytes", "percache_stack_reuse",
    "percache_stack_decode",
    "percache_tree_create", "percache_tree_destroy", "percache_tree_match", "percache_tree_insert",
    "percache_tree_nodes", "percache_tree_bytes",
    "percache_prefill_workspace_bytes", "percache_prefill_reuse", "percache_qkv_rope", "percache_attention_reuse",
    "percache_chunk_table_bytes", "percache_chunk_table_put", "percache_chunk_table_drop",
    "percache_prefill_reuse_table", "percache_stack_reuse_table",
    "percache_profile_enable", "percache_profile_read",
    "percache_peak_scratch_bytes", "percache_peak_mfma_bf16", "percache_peak_stream_read", "percache_peak_attention_tile_loop",
]
KERNEL_LOOKUP, KERNEL_QKV_ROPE, KERNEL_ATTENTION = 0, 1, 2


class PercacheError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {text}")
        self.status = status


class Config(ctypes.Structure):
    _fields_ = [
        ("n_layers", ctypes.c_int32), ("hidden", ctypes.c_int32), ("n_q_heads", ctypes.c_int32),
        ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32), ("n_slots", ctypes.c_int32),
        ("slot_capacity", ctypes.c_int32), ("max_pos", ctypes.c_int32), ("rope_theta", ctypes.c_float),
        ("bank_capacity", ctypes.c_int32), ("emb_dim", ctypes.c_int32), ("kv_fp8", ctypes.c_int32),
        ("n_slots_8bit", ctypes.c_int32),
    ]


class BlockWeights(ctypes.Structure):
    """percache_block_weights: device pointers of one block's weights."""
    _fields_ = [(n, ctypes.c_void_p) for n in ("gain1", "wqkv", "wo", "gain2", "w_gate", "w_up", "w_down",
                                               "qkv_bias", "q_norm", "k_norm")]


_lib = None
_vp, _i32, _sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
_pi32 = ctypes.POINTER(ctypes.c_int32)


def load_library() -> ctypes.CDLL:
    """Loads the built library; raises if it has not been built (no fallback path exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(f"{LIB_PATH} is missing: build it with `python -m paper_2601_11553_amd.build`")
    lib = ctypes.CDLL(LIB_PATH)
    cfgp = ctypes.POINTER(Config)
    sig = {
        "percache_arena_bytes": (_sz, [cfgp]),
        "percache_create": (_i32, [cfgp, _vp, _sz, ctypes.POINTER(_vp)]),
        "percache_destroy": (None, [_vp]),
        "percache_last_error": (ctypes.c_char_p, [_vp]),
        "percache_bank_put": (_i32, [_vp, _i32, _vp, _i32, _vp]),
        "percache_bank_size": (_i32, [_vp]),
        "percache_lookup_workspace_bytes": (_sz, [_vp, _i32]),
        "percache_lookup": (_i32, [_vp, _vp, _i32, ctypes.c_float, _vp, _vp, _vp, _vp, _sz, _vp]),
        "percache_lookup_noalloc": (_i32, [_vp, _vp, _i32, ctypes.c_float, _vp, _vp, _vp, _vp]),
        "percache_lookup_topk": (_i32, [_vp, _vp, _i32, _i32, _vp, _vp, _vp, _sz, _vp]),
        "percache_bank_refresh_scan": (_i32, [_vp, _vp, _i32, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
        "percache_kv_put": (_i32, [_vp, _i32, _i32, _vp, _vp, _i32, _vp]),
        "percache_kv_put_batch": (_i32, [_vp, _i32, _pi32, _i32, _vp, _vp, _i32, _vp]),
        "percache_kv_get": (_i32, [_vp, _i32, _i32, _vp, _vp, _pi32, _vp]),
        "percache_kv_get_batch": (_i32, [_vp, _i32, _pi32, _i32, _vp, _vp, _i32, _vp]),
        "percache_kv_evict": (_i32, [_vp, _i32, _i32]),
        "percache_kv_len": (_i32, [_vp, _i32, _i32]),
        "percache_prefill_workspace_bytes": (_sz, [_vp, _i32, _i32, _i32]),
        "percache_prefill_reuse": (_i32, [_vp, _i32, _vp, _vp, _i32, _i32, _pi32, _pi32, _pi32, _i32, _vp, _vp, _vp, _vp, _sz, _vp]),
        "percache_qkv_rope": (_i32, [_vp, _vp, _vp, _i32, _i32, _pi32, _pi32, _pi32, _i32, _i32, _vp, _vp, _vp, _vp, _sz, _vp]),
        "percache_attention_reuse": (_i32, [_vp, _i32, _vp, _vp, _vp, _i32, _i32, _pi32, _pi32, _pi32, _i32, _i32, _vp, _vp, _sz, _vp]),
        "percache_chunk_table_bytes": (_sz, [_vp, _i32, _i32]),
        "percache_chunk_table_put": (_i32, [_vp, _vp, _sz, _i32, _i32, _pi32, _pi32, _pi32, _i32, _vp]),
        "percache_chunk_table_drop": (_i32, [_vp, _vp]),
        "percache_prefill_reuse_table": (_i32, [_vp, _i32, _vp, _vp, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
        "percache_stack_reuse_table": (_i32, [_vp, ctypes.POINTER(BlockWeights), _i32, _i32, ctypes.c_float, _vp, _i32, _i32,
                                              _vp, _vp, _vp, _sz, _vp]),
        "percache_kv_slice": (_i32, [_vp, _i32, _vp, _vp, _i32, _pi32, _pi32, _i32, _vp]),
        "percache_kv_append": (_i32, [_vp, _i32, _i32, _vp, _vp, _i32, _vp]),
        "percache_stack_decode": (_i32, [_vp, ctypes.POINTER(BlockWeights), _i32, _i32, ctypes.c_float, _vp, _i32, _i32,
                                         _pi32, _pi32, _pi32, _i32, _pi32, _vp, _vp, _sz, _vp]),
        "percache_stack_workspace_bytes": (_sz, [_vp, _i32, _i32, _i32, _i32]),
        "percache_stack_reuse": (_i32, [_vp, ctypes.POINTER(BlockWeights), _i32, _i32, ctypes.c_float, _vp, _i32, _i32,
                                        _pi32, _pi32, _pi32, _i32, _pi32, _pi32, _i32, _vp, _vp, _sz, _vp]),
        "percache_tree_create": (_vp, [_i32, ctypes.c_int64, ctypes.c_int64, _i32]),
        "percache_tree_destroy": (None, [_vp]),
        "percache_tree_match": (_i32, [_vp, ctypes.POINTER(ctypes.c_char_p), _i32, _pi32, _pi32]),
        "percache_tree_insert": (_i32, [_vp, ctypes.POINTER(ctypes.c_char_p), _pi32, _i32, _pi32, ctypes.POINTER(ctypes.c_uint8),
                                        _pi32, _i32, _pi32]),
        "percache_tree_nodes": (_i32, [_vp]),
        "percache_tree_bytes": (ctypes.c_int64, [_vp]),
        "percache_profile_enable": (_i32, [_vp, _i32]),
        "percache_profile_read": (_i32, [_vp, _i32, ctypes.POINTER(ctypes.c_float), _pi32]),
        "percache_peak_scratch_bytes": (_sz, [_vp]),
        "percache_peak_mfma_bf16": (_i32, [_vp, _i32, _i32, _vp, _sz, ctypes.POINTER(ctypes.c_double), _vp]),
        "percache_peak_stream_read": (_i32, [_vp, _vp, _sz, _vp, _sz, _vp]),
        "percache_peak_attention_tile_loop": (_i32, [_vp, _vp, _sz, _i32, _vp, _sz, ctypes.POINTER(ctypes.c_double), _vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib


def _ptr(t) -> Optional[int]:
    return None if t is None else int(t.data_ptr())


def _stream() -> Optional[int]:
    import torch
    return int(torch.cuda.current_stream().cuda_stream) or None


def _host_i32(a, shape=None):
    if a is None:
        return None, None
    arr = np.ascontiguousarray(a, dtype=np.int32)
    if shape is not None:
        arr = arr.reshape(shape)
    return arr, arr.ctypes.data_as(_pi32)


class Percache:
    """One context = one arena (a torch uint8 CUDA tensor) + host bookkeeping.  Methods mirror the C calls."""

    def __init__(self, *, n_layers=1, hidden=1024, n_q_heads=16, n_kv_heads=8, head_dim=128, n_slots=16,
                 slot_capacity=512, max_pos=4096, rope_theta=10000.0, bank_capacity=0, emb_dim=0, kv_fp8=False,
                 n_slots_8bit=0, device="cuda:0"):
        import torch
        self.lib = load_library()
        self.cfg = Config(n_layers, hidden, n_q_heads, n_kv_heads, head_dim, n_slots, slot_capacity, max_pos,
                          rope_theta, bank_capacity, emb_dim, int(bool(kv_fp8)), int(n_slots_8bit))
        self.device = torch.device(device)
        need = self.lib.percache_arena_bytes(ctypes.byref(self.cfg))
        if need == 0:
            # let create produce the message
            out = _vp()
            st = self.lib.percache_create(ctypes.byref(self.cfg), None, 0, ctypes.byref(out))
            raise PercacheError(st, self.lib.percache_last_error(None).decode())
        self.arena = torch.empty(need + 256, dtype=torch.uint8, device=self.device)
        base = self.arena.data_ptr()
        self._arena_ptr = (base + 255) // 256 * 256
        out = _vp()
        with torch.cuda.device(self.device):
            st = self.lib.percache_create(ctypes.byref(self.cfg), self._arena_ptr, need, ctypes.byref(out))
        if st != PC_OK:
            raise PercacheError(st, self.lib.percache_last_error(None).decode())
        self.ctx = out
        self._ws = None
        self._lookup_ws = None

    # ------------------------------------------------------------------ helpers
    def _check(self, st: int):
        if st != PC_OK:
            raise PercacheError(st, self.lib.percache_last_error(self.ctx).decode())

    def close(self):
        if getattr(self, "ctx", None):
            self.lib.percache_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _workspace(self, nbytes: int):
        import torch
        if self._ws is None or self._ws.numel() < nbytes + 256:
            self._ws = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
        p = (self._ws.data_ptr() + 255) // 256 * 256
        return p

    def percache_profile_enable(self, on=True, kernels=None):
        """``kernels``: the kinds to bracket with events (default: all three)."""
        flag = 0 if not on else 1 if kernels is None else sum(1 << (k + 1) for k in set(kernels))
        self._check(self.lib.percache_profile_enable(self.ctx, flag))

    def percache_profile_read(self, kernel: int):
        """(summed milliseconds, launches) of one kernel kind since the last read; waits for the events."""
        ms, n = ctypes.c_float(0), ctypes.c_int32(0)
        self._check(self.lib.percache_profile_read(self.ctx, kernel, ctypes.byref(ms), ctypes.byref(n)))
        return ms.value, n.value

    # ------------------------------------------------------------------ achievable peaks (measurement aids)
    def _peak_scratch(self):
        import torch
        need = self.lib.percache_peak_scratch_bytes(self.ctx)
        if getattr(self, "_peak_ws", None) is None or self._peak_ws.numel() < need:
            self._peak_ws = torch.empty(need, dtype=torch.uint8, device=self.device)
        return self._peak_ws

    def percache_peak_mfma_bf16(self, iters: int, random_operands: bool) -> float:
        """Enqueues the register-resident bf16 MFMA loop; returns the flop count of the launch."""
        ws = self._peak_scratch()
        fl = ctypes.c_double(0.0)
        self._check(self.lib.percache_peak_mfma_bf16(self.ctx, iters, 1 if random_operands else 0, _ptr(ws), ws.numel(),
                                                     ctypes.byref(fl), _stream()))
        return fl.value

    def percache_peak_attention_tile_loop(self, kv, tiles: int) -> float:
        """Enqueues the model of the attention tile loop over ``kv`` (>= 8 MiB of bf16 values); returns the flop count."""
        ws = self._peak_scratch()
        fl = ctypes.c_double(0.0)
        self._check(self.lib.percache_peak_attention_tile_loop(self.ctx, _ptr(kv), kv.numel() * kv.element_size(), tiles, _ptr(ws),
                                                               ws.numel(), ctypes.byref(fl), _stream()))
        return fl.value

    def percache_peak_stream_read(self, buf) -> int:
        """Enqueues one streaming read of ``buf``; returns the bytes read."""
        ws = self._peak_scratch()
        nbytes = buf.numel() * buf.element_size()
        self._check(self.lib.percache_peak_stream_read(self.ctx, _ptr(buf), nbytes, _ptr(ws), ws.numel(), _stream()))
        return nbytes // 16 * 16

    # ------------------------------------------------------------------ front tier
    def percache_bank_put(self, index: int, emb):
        self._check(self.lib.percache_bank_put(self.ctx, index, _ptr(emb), emb.shape[0], _stream()))

    def percache_bank_size(self) -> int:
        return self.lib.percache_bank_size(self.ctx)

    def percache_lookup(self, probes, tau: float, idx_out=None, sim_out=None, hit_out=None):
        import torch
        n = probes.shape[0]
        if idx_out is None:
            idx_out = torch.empty(n, dtype=torch.int32, device=self.device)
            sim_out = torch.empty(n, dtype=torch.float32, device=self.device)
            hit_out = torch.empty(n, dtype=torch.uint8, device=self.device)
        need = self.lib.percache_lookup_workspace_bytes(self.ctx, n)
        if self._lookup_ws is None or self._lookup_ws.numel() < need + 256:
            self._lookup_ws = torch.empty(need + 256, dtype=torch.uint8, device=self.device)
        ws = (self._lookup_ws.data_ptr() + 255) // 256 * 256
        self._check(self.lib.percache_lookup(self.ctx, _ptr(probes), n, tau, _ptr(idx_out), _ptr(sim_out),
                                             _ptr(hit_out), ws, need, _stream()))
        return idx_out, sim_out, hit_out

    def percache_lookup_noalloc(self, probes, tau: float, idx_out, sim_out, hit_out):
        """percache_lookup into caller-provided outputs, partial results in the library's static scratch (no workspace)."""
        self._check(self.lib.percache_lookup_noalloc(self.ctx, _ptr(probes), probes.shape[0], tau, _ptr(idx_out),
                                                     _ptr(sim_out), _ptr(hit_out), _stream()))
        return idx_out, sim_out, hit_out

    def percache_lookup_topk(self, probes, k: int):
        """(idx [P, k] int32, sim [P, k] float32): the k best bank rows per probe, best first."""
        import torch
        n = probes.shape[0]
        idx_out = torch.empty((n, k), dtype=torch.int32, device=self.device)
        sim_out = torch.empty((n, k), dtype=torch.float32, device=self.device)
        need = self.lib.percache_lookup_workspace_bytes(self.ctx, n)
        if self._lookup_ws is None or self._lookup_ws.numel() < need + 256:
            self._lookup_ws = torch.empty(need + 256, dtype=torch.uint8, device=self.device)
        ws = (self._lookup_ws.data_ptr() + 255) // 256 * 256
        self._check(self.lib.percache_lookup_topk(self.ctx, _ptr(probes), n, k, _ptr(idx_out), _ptr(sim_out), ws, need, _stream()))
        return idx_out, sim_out

    def percache_bank_refresh_scan(self, new_emb, kth_sim):
        """(best_sim [N] float32, best_new [N] int32, stale [N] uint8) for the N bank rows against the new rows."""
        import torch
        n_new, N = new_emb.shape[0], self.percache_bank_size()
        best_sim = torch.empty(N, dtype=torch.float32, device=self.device)
        best_new = torch.empty(N, dtype=torch.int32, device=self.device)
        stale = torch.empty(N, dtype=torch.uint8, device=self.device)
        need = self.lib.percache_lookup_workspace_bytes(self.ctx, n_new)
        if self._lookup_ws is None or self._lookup_ws.numel() < need + 256:
            self._lookup_ws = torch.empty(need + 256, dtype=torch.uint8, device=self.device)
        ws = (self._lookup_ws.data_ptr() + 255) // 256 * 256
        self._check(self.lib.percache_bank_refresh_scan(self.ctx, _ptr(new_emb), n_new, _ptr(kth_sim), _ptr(best_sim),
                                                        _ptr(best_new), _ptr(stale), ws, need, _stream()))
        return best_sim, best_new, stale

    # ------------------------------------------------------------------ K/V store
    def percache_kv_put(self, layer: int, slot: int, k, v, n_tokens: Optional[int] = None):
        n = k.shape[1] if n_tokens is None else n_tokens
        self._check(self.lib.percache_kv_put(self.ctx, layer, slot, _ptr(k), _ptr(v), n, _stream()))

    def percache_kv_put_batch(self, layer: int, slots, k, v, n_tokens: Optional[int] = None):
        """k, v: [n, Hkv, n_tokens, D]; chunk i is written to slot slots[i] (one launch)."""
        arr, p = _host_i32(slots)
        n = k.shape[2] if n_tokens is None else n_tokens
        self._check(self.lib.percache_kv_put_batch(self.ctx, layer, p, len(arr), _ptr(k), _ptr(v), n, _stream()))

    def percache_kv_get(self, layer: int, slot: int):
        import torch
        n = self.lib.percache_kv_len(self.ctx, layer, slot)
        if n <= 0:
            self._check(n if n < 0 else -3)
        shape = (self.cfg.n_kv_heads, n, self.cfg.head_dim)
        k = torch.empty(shape, dtype=torch.bfloat16, device=self.device)
        v = torch.empty(shape, dtype=torch.bfloat16, device=self.device)
        cnt = ctypes.c_int32(0)
        self._check(self.lib.percache_kv_get(self.ctx, layer, slot, _ptr(k), _ptr(v), ctypes.byref(cnt), _stream()))
        assert cnt.value == n
        return k, v

    def percache_kv_get_batch(self, layer: int, slots, n_tokens: int, k_out=None, v_out=None):
        """The first n_tokens tokens of every slot named, as [n, Hkv, n_tokens, D] tensors (one launch)."""
        import torch
        arr, p = _host_i32(slots)
        shape = (len(arr), self.cfg.n_kv_heads, n_tokens, self.cfg.head_dim)
        if k_out is None:
            k_out = torch.empty(shape, dtype=torch.bfloat16, device=self.device)
            v_out = torch.empty(shape, dtype=torch.bfloat16, device=self.device)
        self._check(self.lib.percache_kv_get_batch(self.ctx, layer, p, len(arr), _ptr(k_out), _ptr(v_out), n_tokens, _stream()))
        return k_out, v_out

    def percache_kv_slice(self, layer: int, k, v, bounds, slots):
        """k, v: [Hkv, seq_len, D]; piece j = tokens [bounds[j], bounds[j+1]) goes to slot slots[j] (< 0: skipped)."""
        b, bp = _host_i32(bounds)
        sl, sp = _host_i32(slots)
        assert len(b) == len(sl) + 1
        self._check(self.lib.percache_kv_slice(self.ctx, layer, _ptr(k), _ptr(v), k.shape[1], bp, sp, len(sl), _stream()))

    def percache_kv_append(self, layer: int, slot: int, k, v):
        self._check(self.lib.percache_kv_append(self.ctx, layer, slot, _ptr(k), _ptr(v), k.shape[1], _stream()))

    def percache_kv_evict(self, layer: int, slot: int):
        self._check(self.lib.percache_kv_evict(self.ctx, layer, slot))

    def percache_kv_len(self, layer: int, slot: int) -> int:
        return self.lib.percache_kv_len(self.ctx, layer, slot)

    # ------------------------------------------------------------------ prefill
    def _chunk_args(self, batch, slot_ids, used_len, n_chunks):
        slot_ids = np.zeros((batch, 0), np.int32) if slot_ids is None else np.asarray(slot_ids, np.int32).reshape(batch, -1)
        max_chunks = slot_ids.shape[1]
        if n_chunks is None:
            n_chunks = np.full(batch, max_chunks, np.int32)
        ids, ids_p = _host_i32(slot_ids)
        ul, ul_p = _host_i32(used_len, (batch, max_chunks)) if used_len is not None else (None, None)
        nc, nc_p = _host_i32(n_chunks, (batch,))
        return (ids, ul, nc), ids_p, ul_p, nc_p, max_chunks

    def percache_prefill_workspace_bytes(self, batch, t_fresh, max_chunks) -> int:
        return self.lib.percache_prefill_workspace_bytes(self.ctx, batch, t_fresh, max_chunks)

    def percache_prefill_reuse(self, layer, x_fresh, wqkv, slot_ids=None, used_len=None, n_chunks=None,
                               attn_out=None, k_fresh_out=None, v_fresh_out=None):
        import torch
        batch, t_fresh, _ = x_fresh.shape
        keep, ids_p, ul_p, nc_p, max_chunks = self._chunk_args(batch, slot_ids, used_len, n_chunks)
        c = self.cfg
        if attn_out is None:
            attn_out = torch.empty((batch, t_fresh, c.n_q_heads * c.head_dim), dtype=torch.bfloat16, device=self.device)
        need = self.percache_prefill_workspace_bytes(batch, t_fresh, max_chunks)
        ws = self._workspace(need)
        self._check(self.lib.percache_prefill_reuse(self.ctx, layer, _ptr(x_fresh), _ptr(wqkv), batch, t_fresh, ids_p,
                                                    ul_p, nc_p, max_chunks, _ptr(attn_out), _ptr(k_fresh_out),
                                                    _ptr(v_fresh_out), ws, need, _stream()))
        return attn_out

    # device-resident chunk lists: a table tensor written once, then calls that enqueue kernels only
    def percache_chunk_table_put(self, slot_ids, used_len=None, n_chunks=None, layer: int = 0, table=None):
        """Writes the chunk list into ``table`` (a uint8 CUDA tensor, created if None) and returns it with its max_chunks."""
        import torch
        batch = len(slot_ids)
        keep, ids_p, ul_p, nc_p, max_chunks = self._chunk_args(batch, slot_ids, used_len, n_chunks)
        need = self.lib.percache_chunk_table_bytes(self.ctx, batch, max_chunks)
        if table is None:
            table = torch.empty(need, dtype=torch.uint8, device=self.device)
        self._check(self.lib.percache_chunk_table_put(self.ctx, _ptr(table), table.numel(), layer, batch, ids_p, ul_p, nc_p,
                                                      max_chunks, _stream()))
        table.max_chunks = max_chunks
        return table

    def percache_chunk_table_drop(self, table):
        self._check(self.lib.percache_chunk_table_drop(self.ctx, _ptr(table)))

    def prefill_workspace(self, batch, t_fresh, max_chunks):
        """(pointer, bytes) of the binding's workspace tensor, grown if needed: for callers that must not allocate later."""
        need = self.percache_prefill_workspace_bytes(batch, t_fresh, max_chunks)
        return self._workspace(need), need

    def percache_prefill_reuse_table(self, layer, x_fresh, wqkv, table, attn_out, k_fresh_out=None, v_fresh_out=None):
        batch, t_fresh, _ = x_fresh.shape
        need = self.percache_prefill_workspace_bytes(batch, t_fresh, table.max_chunks)
        ws = self._workspace(need)
        self._check(self.lib.percache_prefill_reuse_table(self.ctx, layer, _ptr(x_fresh), _ptr(wqkv), batch, t_fresh, _ptr(table),
                                                          _ptr(attn_out), _ptr(k_fresh_out), _ptr(v_fresh_out), ws, need, _stream()))
        return attn_out

    def percache_stack_reuse_table(self, layers, ffn: int, eps: float, h_in, table, h_out, weights=None):
        """``weights``: the marshalled layer array of an earlier call (returned), to keep host work out of a hot loop."""
        batch, t_fresh, _ = h_in.shape
        arr = weights if weights is not None else self._weights(layers)
        need = self.percache_stack_workspace_bytes(batch, t_fresh, table.max_chunks, ffn)
        ws = self._workspace(need)
        self._check(self.lib.percache_stack_reuse_table(self.ctx, arr, len(layers), ffn, eps, _ptr(h_in), batch, t_fresh,
                                                        _ptr(table), _ptr(h_out), ws, need, _stream()))
        return arr

    def percache_qkv_rope(self, layer, x_fresh, wqkv, slot_ids=None, used_len=None, n_chunks=None,
                          q_out=None, k_out=None, v_out=None):
        import torch
        batch, t_fresh, _ = x_fresh.shape
        keep, ids_p, ul_p, nc_p, max_chunks = self._chunk_args(batch, slot_ids, used_len, n_chunks)
        c = self.cfg
        if q_out is None:
            q_out = torch.empty((batch, c.n_q_heads, t_fresh, c.head_dim), dtype=torch.bfloat16, device=self.device)
            k_out = torch.empty((batch, c.n_kv_heads, t_fresh, c.head_dim), dtype=torch.bfloat16, device=self.device)
            v_out = torch.empty_like(k_out)
        need = self.percache_prefill_workspace_bytes(batch, t_fresh, max_chunks)
        ws = self._workspace(need)
        self._check(self.lib.percache_qkv_rope(self.ctx, _ptr(x_fresh), _ptr(wqkv), batch, t_fresh, ids_p, ul_p, nc_p,
                                               max_chunks, layer, _ptr(q_out), _ptr(k_out), _ptr(v_out), ws, need,
                                               _stream()))
        return q_out, k_out, v_out

    def percache_attention_reuse(self, layer, q, k_fresh, v_fresh, slot_ids=None, used_len=None, n_chunks=None,
                                 n_splits: int = 0, attn_out=None):
        import torch
        batch, _, t_fresh, _ = q.shape
        keep, ids_p, ul_p, nc_p, max_chunks = self._chunk_args(batch, slot_ids, used_len, n_chunks)
        c = self.cfg
        if attn_out is None:
            attn_out = torch.empty((batch, t_fresh, c.n_q_heads * c.head_dim), dtype=torch.bfloat16, device=self.device)
        need = self.percache_prefill_workspace_bytes(batch, t_fresh, max_chunks)
        ws = self._workspace(need)
        self._check(self.lib.percache_attention_reuse(self.ctx, layer, _ptr(q), _ptr(k_fresh), _ptr(v_fresh), batch,
                                                      t_fresh, ids_p, ul_p, nc_p, max_chunks, n_splits, _ptr(attn_out),
                                                      ws, need, _stream()))
        return attn_out

    # ------------------------------------------------------------------ stack of layers on the retained rows
    def percache_stack_workspace_bytes(self, batch, t_fresh, max_chunks, ffn) -> int:
        return self.lib.percache_stack_workspace_bytes(self.ctx, batch, t_fresh, max_chunks, ffn)

    @staticmethod
    def _weights(layers):
        arr = (BlockWeights * len(layers))()
        for i, lw in enumerate(layers):
            for name, _t in BlockWeights._fields_:
                setattr(arr[i], name, _ptr(lw.get(name)))   # the three variant fields may be missing (absent)
        return arr

    def percache_stack_reuse(self, layers, ffn: int, eps: float, h_in, slot_ids=None, used_len=None, n_chunks=None,
                             save_bounds=None, save_slots=None, h_out=None):
        """layers: one dict per layer with the tensors gain1, wqkv, wo, gain2, w_gate, w_up, w_down (bf16, on device)."""
        import torch
        batch, t_fresh, _ = h_in.shape
        keep, ids_p, ul_p, nc_p, max_chunks = self._chunk_args(batch, slot_ids, used_len, n_chunks)
        arr = self._weights(layers)
        sb, sb_p = _host_i32(save_bounds)
        n_save = 0 if sb is None else len(sb) - 1
        ss, ss_p = _host_i32(save_slots, (batch, n_save)) if n_save else (None, None)
        if h_out is None:
            h_out = torch.empty_like(h_in)
        need = self.percache_stack_workspace_bytes(batch, t_fresh, max_chunks, ffn)
        ws = self._workspace(need)
        self._check(self.lib.percache_stack_reuse(self.ctx, arr, len(layers), ffn, eps, _ptr(h_in), batch, t_fresh, ids_p,
                                                  ul_p, nc_p, max_chunks, sb_p, ss_p, n_save, _ptr(h_out), ws, need,
                                                  _stream()))
        return h_out

    def percache_stack_decode(self, layers, ffn: int, eps: float, h_in, slot_ids, append_slots, used_len=None, n_chunks=None,
                              h_out=None):
        """One decoding step for [batch, n_new, hidden] new rows; their K/V are appended to append_slots[b]."""
        import torch
        batch, n_new, _ = h_in.shape
        keep, ids_p, ul_p, nc_p, max_chunks = self._chunk_args(batch, slot_ids, used_len, n_chunks)
        arr = self._weights(layers)
        ap, ap_p = _host_i32(append_slots, (batch,))
        if h_out is None:
            h_out = torch.empty_like(h_in)
        need = self.percache_stack_workspace_bytes(batch, n_new, max_chunks, ffn)
        ws = self._workspace(need)
        self._check(self.lib.percache_stack_decode(self.ctx, arr, len(layers), ffn, eps, _ptr(h_in), batch, n_new, ids_p, ul_p,
                                                   nc_p, max_chunks, ap_p, _ptr(h_out), ws, need, _stream()))
        return h_out


class CacheTree:
    """Host-side chunk prefix tree with LFU eviction (percache_tree_*): marshalling only."""

    def __init__(self, n_slots: int, byte_limit: int, bytes_per_token: int, tail_discard_tokens: int = 0):
        self.lib = load_library()
        self.n_slots = n_slots
        self.t = self.lib.percache_tree_create(n_slots, byte_limit, bytes_per_token, tail_discard_tokens)
        if not self.t:
            raise PercacheError(-1, "percache_tree_create: bad argument")

    def close(self):
        if getattr(self, "t", None):
            self.lib.percache_tree_destroy(self.t)
            self.t = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @staticmethod
    def _texts(chunks):
        arr = (ctypes.c_char_p * len(chunks))(*[c.encode() if isinstance(c, str) else bytes(c) for c in chunks])
        return arr

    def percache_tree_match(self, chunks):
        """Returns (slots, used_len) of the longest stored chain that is a prefix of ``chunks``."""
        n = len(chunks)
        slots = (ctypes.c_int32 * max(n, 1))()
        used = (ctypes.c_int32 * max(n, 1))()
        m = self.lib.percache_tree_match(self.t, self._texts(chunks), n, slots, used)
        if m < 0:
            raise PercacheError(m, "percache_tree_match")
        return list(slots[:m]), list(used[:m])

    def percache_tree_insert(self, chunks, tokens):
        """Returns (n_shared, slots, is_new, evicted_slots)."""
        n = len(chunks)
        slots = (ctypes.c_int32 * n)()
        new = (ctypes.c_uint8 * n)()
        ev = (ctypes.c_int32 * self.n_slots)()
        n_ev = ctypes.c_int32(0)
        tok = (ctypes.c_int32 * n)(*[int(x) for x in tokens])
        s = self.lib.percache_tree_insert(self.t, self._texts(chunks), tok, n, slots, new, ev, self.n_slots, ctypes.byref(n_ev))
        evicted = list(ev[:n_ev.value])
        if s < 0:
            err = PercacheError(s, "percache_tree_insert")
            err.evicted = evicted
            raise err
        return s, list(slots), [bool(x) for x in new], evicted

    def percache_tree_nodes(self) -> int:
        return self.lib.percache_tree_nodes(self.t)

    def percache_tree_bytes(self) -> int:
        return self.lib.percache_tree_bytes(self.t)
