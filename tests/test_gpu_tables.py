"""Device-resident chunk lists (percache_chunk_table_put + the *_table calls) through the C ABI: the same kernels as the
host-list calls, so results must agree bit for bit; a table-taking stack call captured into a HIP graph must replay to
the eager result every time, also after another list has been written into the same table."""
import numpy as np
import pytest
import torch

from paper_2601_11553_amd import workloads as wl
from paper_2601_11553_amd.binding import Percache, PercacheError

from gpu_util import DEV, bf16, fill_slots, make_ctx
from test_gpu_stack import EPS, dev_layers

pytestmark = pytest.mark.gpu


def test_prefill_from_a_device_table_equals_the_host_list_call():
    w = wl.make_prefill("tbl", 41, "bf16", 512, 6, 2, 128, 3, 70, 3, 192, 12)
    w.used_len[0] = [192, 100, 1]
    w.used_len[1] = [65, 0, 190]
    pc = make_ctx(w)
    fill_slots(pc, w, w.slot_ids.reshape(-1))
    x, wq = bf16(w.X), bf16(w.Wqkv)
    ref = pc.percache_prefill_reuse(0, x, wq, w.slot_ids, w.used_len).clone()
    table = pc.percache_chunk_table_put(w.slot_ids, w.used_len)
    out = torch.empty_like(ref)
    pc.percache_prefill_reuse_table(0, x, wq, table, out)
    torch.cuda.synchronize()
    assert torch.equal(out, ref)
    # errors, all found on the host: a table the context does not know, another batch size, a slot changed since the put
    other = torch.empty_like(table)
    other.max_chunks = table.max_chunks
    with pytest.raises(PercacheError) as e:
        pc.percache_prefill_reuse_table(0, x, wq, other, out)
    assert e.value.status == -1
    with pytest.raises(PercacheError) as e:
        pc.percache_prefill_reuse_table(0, x[:2].contiguous(), wq, table, out[:2])
    assert e.value.status == -1
    s0 = int(w.slot_ids[0, 0])
    k, v = w.slot_kv(s0)
    pc.percache_kv_put(0, s0, bf16(k[:, :150]), bf16(v[:, :150]))          # shorter than the 192 tokens the table uses
    with pytest.raises(PercacheError) as e:
        pc.percache_prefill_reuse_table(0, x, wq, table, out)
    assert e.value.status == -4
    pc.percache_kv_evict(0, s0)
    with pytest.raises(PercacheError) as e:
        pc.percache_prefill_reuse_table(0, x, wq, table, out)
    assert e.value.status == -3
    pc.percache_kv_put(0, s0, bf16(k), bf16(v))
    pc.percache_prefill_reuse_table(0, x, wq, table, out)                  # valid again
    torch.cuda.synchronize()
    assert torch.equal(out, ref)
    pc.percache_chunk_table_drop(table)
    with pytest.raises(PercacheError):
        pc.percache_prefill_reuse_table(0, x, wq, table, out)
    pc.close()


def test_stack_from_a_device_table_captured_into_a_graph():
    """Three layers over four chunks, 40 fresh rows.  The call is captured once; every replay is compared with an eager
    host-list call made in between (with synchronisations of its own), first for the captured list (bit for bit), then
    for two other lists written into the same table (the replay keeps the captured launch shapes, so only up to the
    rounding of another key-axis partition)."""
    H, Hq, Hkv, D, F, C, L, T, n_c = 256, 4, 2, 128, 384, 128, 3, 40, 4
    w = wl.make_prefill("graph", 43, "bf16", H, Hq, Hkv, D, 2, T, n_c, C, 12)
    Ws = [wl.stack_weights(43, l, H, Hq, Hkv, D, F) for l in range(L)]
    layers = dev_layers(Ws)
    pc = Percache(n_layers=L, hidden=H, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=D, n_slots=12, slot_capacity=C,
                  max_pos=n_c * C + T, device=DEV)
    for l in range(L):
        for s_, (k, v) in w.slots_kv(range(12), l).items():
            pc.percache_kv_put(l, s_, bf16(k), bf16(v))
    x = bf16(w.X)
    lists = [(w.slot_ids, w.used_len)]
    g = np.random.default_rng(7)
    for _ in range(2):
        ids = np.stack([g.permutation(12)[:n_c] for _ in range(2)]).astype(np.int32)
        used = g.integers(1, C + 1, size=(2, n_c)).astype(np.int32)
        lists.append((ids, used))
    table = pc.percache_chunk_table_put(*lists[0])
    out = torch.empty_like(x)
    arr = pc.percache_stack_reuse_table(layers, F, EPS, x, table, out)      # warm-up outside the capture
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        graph.capture_begin()
        pc.percache_stack_reuse_table(layers, F, EPS, x, table, out, weights=arr)
        graph.capture_end()
    torch.cuda.synchronize()
    for n_list, (ids, used) in enumerate(lists):
        pc.percache_chunk_table_put(ids, used, table=table)                 # ordered on the stream, outside the graph
        for rep in range(3):
            eager = pc.percache_stack_reuse(layers, F, EPS, x, ids, used)   # the program's own eager work in between
            torch.cuda.synchronize()
            out.zero_()
            graph.replay()
            torch.cuda.synchronize()
            if n_list == 0:
                assert torch.equal(out, eager), rep
            else:   # the replay keeps the key-axis partition of the captured list, the eager call picks its own: fp32 rounding apart
                diff = (out.float() - eager.float()).abs().max().item()
                assert diff <= 2.0 ** -7 * eager.float().abs().max().item(), (n_list, rep, diff)
    pc.close()
