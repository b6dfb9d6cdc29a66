"""Helpers shared by the GPU parity tests: host<->device conversion and the tolerance check."""
import numpy as np
import torch

DEV = "cuda:0"
# Tolerance for bf16 attention / projection outputs against the unrounded oracle.
MAX_ABS, MEAN_ABS = 2e-2, 2e-3
# Additional bound used here because outputs of flat softmaxes are O(0.03): relative Frobenius error.
REL_FRO = 1e-2


def bf16(a):
    return torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(DEV, torch.bfloat16)


def f16(a):
    return torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(DEV, torch.float16)


def host(t):
    return t.float().cpu().numpy()


def check_close(got, ref, what="", max_abs=MAX_ABS, mean_abs=MEAN_ABS, rel_fro=REL_FRO):
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    err = np.abs(got - ref)
    fro = np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-30)
    msg = f"{what}: max-abs {err.max():.3e} mean-abs {err.mean():.3e} rel-fro {fro:.3e} (|ref| max {np.abs(ref).max():.3e})"
    print(msg, flush=True)
    assert err.max() < max_abs and err.mean() < mean_abs and fro < rel_fro, msg


def make_ctx(w, n_layers=1, bank_capacity=0, emb_dim=0, max_pos=None, **over):
    from paper_2601_11553_amd.binding import Percache
    kw = dict(n_layers=n_layers, hidden=w.hidden, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim,
              n_slots=w.n_slots, slot_capacity=w.chunk_tokens, max_pos=max_pos or w.max_pos,
              rope_theta=w.rope_theta, bank_capacity=bank_capacity, emb_dim=emb_dim, device=DEV)
    kw.update(over)
    return Percache(**kw)


def fill_slots(pc, w, slots, layer=0):
    kv = w.slots_kv(sorted(set(int(s) for s in slots)), layer)
    for s, (k, v) in kv.items():
        pc.percache_kv_put(layer, s, bf16(k), bf16(v))
    return kv
