"""The lookup entry point that allocates nothing (percache_lookup_noalloc: partial results in the library's file-scope
device array instead of a caller workspace) against percache_lookup, through the C ABI: same kernels, so index, hit
flag and similarity must agree bit for bit.  Two calls in a row share the array, the second with a smaller input."""
import numpy as np
import pytest
import torch

from paper_2601_11553_amd import workloads as wl
from paper_2601_11553_amd.binding import Percache, PercacheError

from gpu_util import DEV, f16

pytestmark = pytest.mark.gpu


def test_lookup_noalloc_matches_lookup_on_two_calls_in_a_row():
    w = wl.lookup_clustered("na", 77, 61, 53, 1024, 32, 0.05, 0.02, 0.92, n_exact=4, n_near=4)
    N, d = w.bank.shape
    pc = Percache(n_layers=1, hidden=256, n_q_heads=4, n_kv_heads=2, head_dim=64, n_slots=1, slot_capacity=64,
                  max_pos=64, bank_capacity=N + 7, emb_dim=d, device=DEV)
    pc.percache_bank_put(0, f16(w.bank))
    probes = f16(w.probes)
    for n in (32, 5):                                   # the second call is smaller and meets the first one's leftovers
        p = probes[40 - n:40].contiguous()              # the last probes: the exact and near copies are among them
        ref = pc.percache_lookup(p, w.tau)
        out = (torch.full((n,), -7, dtype=torch.int32, device=DEV), torch.full((n,), -7.0, dtype=torch.float32, device=DEV),
               torch.full((n,), 9, dtype=torch.uint8, device=DEV))
        mem_before = torch.cuda.memory_allocated()
        pc.percache_lookup_noalloc(p, w.tau, *out)
        assert torch.cuda.memory_allocated() == mem_before
        torch.cuda.synchronize()
        for a, b in zip(out, ref):
            assert torch.equal(a, b), (n, a, b)
        assert out[2].sum().item() >= min(n, 8) - 4     # hits of the copy block are in the window
    # limits: more probes than one pass takes are refused with a message, outputs untouched
    big = probes[:33].contiguous()
    o = (torch.zeros(33, dtype=torch.int32, device=DEV), torch.zeros(33, dtype=torch.float32, device=DEV),
         torch.zeros(33, dtype=torch.uint8, device=DEV))
    with pytest.raises(PercacheError) as e:
        pc.percache_lookup_noalloc(big, w.tau, *o)
    assert e.value.status == -2 and "at most 32" in str(e.value)
    pc.close()
