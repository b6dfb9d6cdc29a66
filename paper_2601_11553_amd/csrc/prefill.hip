// Host entry points of the cache-reusing prefill (Sec. 4.2.2, App. B.1): argument validation against the
// host mirror of the slot table, chunk-table staging, and the launches of the projection and attention kernels.
#include "percache_internal.hpp"

namespace {

struct Prepared {
  pc::PrefillWs ws;
  int tbl_stride;
  int min_tiles;
};

// Everything that can fail is checked here, before any enqueue.
pc_status prepare(percache_ctx *ctx, int32_t layer, int32_t batch, int32_t t_fresh, const int32_t *slot_ids,
                  const int32_t *used_len, const int32_t *n_chunks, int32_t max_chunks, void *workspace,
                  size_t workspace_bytes, std::vector<int32_t> &rows, Prepared &p, const pc_table_shadow *shadow = nullptr) {
  if (!ctx) return PC_EINVAL;
  pc_status st = pc::build_chunk_table(ctx, layer, batch, t_fresh, slot_ids, used_len, n_chunks, max_chunks, rows);
  if (st != PC_OK) return st;
  if (shadow && rows != shadow->rows)
    return pc::fail(ctx, PC_ELEN, "the slots' formats or lengths no longer match the device chunk table: put it again");
  {  // sizes the kernels index with 32 bits (checked again where they are launched; here: before anything is enqueued)
    const percache_config &c = ctx->cfg;
    const long F = (long)(c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim, M = (long)batch * t_fresh;
    if (F * c.hidden >= (1L << 31) || M * c.hidden >= (1L << 31) || M * F >= (1L << 31))
      return pc::fail(ctx, PC_ESHAPE, "operand larger than 2^31 elements");
  }
  size_t need = percache_prefill_workspace_bytes(ctx, batch, t_fresh, max_chunks);
  if (!workspace || workspace_bytes < need)
    return pc::fail(ctx, PC_ENOMEM, "prefill workspace has %zu bytes, need %zu", workspace_bytes, need);
  if ((uintptr_t)workspace % pc::kAlign) return pc::fail(ctx, PC_EINVAL, "workspace must be 256-byte aligned");
  p.ws = pc::carve_prefill_ws(ctx->cfg, ctx->n_cu, workspace, batch, t_fresh, max_chunks);
  p.tbl_stride = pc::tbl_stride(max_chunks);
  p.min_tiles = INT32_MAX;
  for (int b = 0; b < batch; ++b) {
    int tiles = rows[(size_t)b * p.tbl_stride + 2] + (t_fresh + pc::kKvTile - 1) / pc::kKvTile;
    if (tiles < p.min_tiles) p.min_tiles = tiles;
  }
  return PC_OK;
}

bool aligned16(const void *p) { return ((uintptr_t)p % 16) == 0; }

}  // namespace

extern "C" {

size_t percache_prefill_workspace_bytes(const percache_ctx *ctx, int32_t batch, int32_t t_fresh, int32_t max_chunks) {
  if (!ctx || batch < 1 || t_fresh < 1 || max_chunks < 0) return 0;
  return pc::carve_prefill_ws(ctx->cfg, ctx->n_cu, nullptr, batch, t_fresh, max_chunks).total;
}

pc_status percache_qkv_rope(percache_ctx *ctx, const void *x_fresh_dev, const void *wqkv_dev, int32_t batch,
                            int32_t t_fresh, const int32_t *slot_ids_host, const int32_t *used_len_host,
                            const int32_t *n_chunks_host, int32_t max_chunks, int32_t layer, void *q_out_dev,
                            void *k_fresh_out_dev, void *v_fresh_out_dev, void *workspace_dev, size_t workspace_bytes,
                            void *stream) {
  if (!ctx) return PC_EINVAL;
  if (!x_fresh_dev || !wqkv_dev || !q_out_dev || !k_fresh_out_dev || !v_fresh_out_dev)
    return pc::fail(ctx, PC_EINVAL, "NULL tensor pointer");
  if (!aligned16(x_fresh_dev) || !aligned16(wqkv_dev) || !aligned16(q_out_dev) || !aligned16(k_fresh_out_dev) ||
      !aligned16(v_fresh_out_dev))
    return pc::fail(ctx, PC_EINVAL, "tensor pointers must be 16-byte aligned");
  std::vector<int32_t> rows;
  Prepared p;
  pc_status st = prepare(ctx, layer, batch, t_fresh, slot_ids_host, used_len_host, n_chunks_host, max_chunks,
                         workspace_dev, workspace_bytes, rows, p);
  if (st != PC_OK) return st;
  hipStream_t s = (hipStream_t)stream;
  st = pc::upload_table(ctx, rows, p.ws.table, s);
  if (st != PC_OK) return st;
  return pc::launch_qkv_rope(ctx, (const __bf16 *)x_fresh_dev, (const __bf16 *)wqkv_dev, batch, t_fresh, p.ws.table,
                             p.tbl_stride, (__bf16 *)q_out_dev, (__bf16 *)k_fresh_out_dev, (__bf16 *)v_fresh_out_dev, s, p.ws.gemm_part);
}

pc_status percache_attention_reuse(percache_ctx *ctx, int32_t layer, const void *q_dev, const void *k_fresh_dev,
                                   const void *v_fresh_dev, int32_t batch, int32_t t_fresh,
                                   const int32_t *slot_ids_host, const int32_t *used_len_host,
                                   const int32_t *n_chunks_host, int32_t max_chunks, int32_t n_splits,
                                   void *attn_out_dev, void *workspace_dev, size_t workspace_bytes, void *stream) {
  if (!ctx) return PC_EINVAL;
  if (!q_dev || !k_fresh_dev || !v_fresh_dev || !attn_out_dev) return pc::fail(ctx, PC_EINVAL, "NULL tensor pointer");
  if (!aligned16(q_dev) || !aligned16(k_fresh_dev) || !aligned16(v_fresh_dev) || !aligned16(attn_out_dev))
    return pc::fail(ctx, PC_EINVAL, "tensor pointers must be 16-byte aligned");
  if (batch >= 1 && t_fresh >= 1) {
    int cap = pc::max_splits_for(ctx->cfg, ctx->n_cu, batch, t_fresh);
    if (n_splits < 0 || n_splits > cap) return pc::fail(ctx, PC_EINVAL, "n_splits %d outside [0,%d] for this shape", n_splits, cap);
  }
  std::vector<int32_t> rows;
  Prepared p;
  pc_status st = prepare(ctx, layer, batch, t_fresh, slot_ids_host, used_len_host, n_chunks_host, max_chunks,
                         workspace_dev, workspace_bytes, rows, p);
  if (st != PC_OK) return st;
  hipStream_t s = (hipStream_t)stream;
  st = pc::upload_table(ctx, rows, p.ws.table, s);
  if (st != PC_OK) return st;
  st = pc::launch_v_repack(ctx, (const __bf16 *)v_fresh_dev, p.ws.v_blk, batch, t_fresh, s);
  if (st != PC_OK) return st;
  return pc::launch_attention(ctx, layer, (const __bf16 *)q_dev, (const __bf16 *)k_fresh_dev, p.ws.v_blk,
                              batch, t_fresh, p.ws.table, p.tbl_stride, p.min_tiles, n_splits, (__bf16 *)attn_out_dev,
                              p.ws.part_o, p.ws.part_ml, s, pc::table_formats(rows, p.tbl_stride, batch));
}

static pc_status run_prefill(percache_ctx *ctx, int32_t layer, const void *x_fresh_dev, const void *wqkv_dev,
                             int32_t batch, int32_t t_fresh, const int32_t *slot_ids_host,
                             const int32_t *used_len_host, const int32_t *n_chunks_host, int32_t max_chunks,
                             void *attn_out_dev, void *k_fresh_out_dev, void *v_fresh_out_dev, void *workspace_dev,
                             size_t workspace_bytes, void *stream, const int32_t *table_dev, const pc_table_shadow *shadow) {
  if (!ctx) return PC_EINVAL;
  if (!x_fresh_dev || !wqkv_dev || !attn_out_dev) return pc::fail(ctx, PC_EINVAL, "NULL tensor pointer");
  if (!aligned16(x_fresh_dev) || !aligned16(wqkv_dev) || !aligned16(attn_out_dev) || !aligned16(k_fresh_out_dev) ||
      !aligned16(v_fresh_out_dev))
    return pc::fail(ctx, PC_EINVAL, "tensor pointers must be 16-byte aligned");
  std::vector<int32_t> rows;
  Prepared p;
  pc_status st = prepare(ctx, layer, batch, t_fresh, slot_ids_host, used_len_host, n_chunks_host, max_chunks,
                         workspace_dev, workspace_bytes, rows, p, shadow);
  if (st != PC_OK) return st;
  hipStream_t s = (hipStream_t)stream;
  if (table_dev) {
    p.ws.table = const_cast<int32_t *>(table_dev);  // the list is on the device already: nothing to copy
  } else {
    st = pc::upload_table(ctx, rows, p.ws.table, s);
    if (st != PC_OK) return st;
  }
  __bf16 *kf = k_fresh_out_dev ? (__bf16 *)k_fresh_out_dev : p.ws.k;
  __bf16 *vf = v_fresh_out_dev ? (__bf16 *)v_fresh_out_dev : p.ws.v;
  bool v_blocked = false;
  st = pc::launch_qkv_rope(ctx, (const __bf16 *)x_fresh_dev, (const __bf16 *)wqkv_dev, batch, t_fresh, p.ws.table,
                           p.tbl_stride, p.ws.q, kf, vf, s, p.ws.gemm_part, pc::QkvExtras(), p.ws.v_blk, &v_blocked);
  if (st != PC_OK) return st;
  if (!v_blocked) st = pc::launch_v_repack(ctx, vf, p.ws.v_blk, batch, t_fresh, s);
  if (st != PC_OK) return st;
  return pc::launch_attention(ctx, layer, p.ws.q, kf, p.ws.v_blk, batch, t_fresh, p.ws.table, p.tbl_stride, p.min_tiles, 0,
                              (__bf16 *)attn_out_dev, p.ws.part_o, p.ws.part_ml, s, pc::table_formats(rows, p.tbl_stride, batch));
}

pc_status percache_prefill_reuse(percache_ctx *ctx, int32_t layer, const void *x_fresh_dev, const void *wqkv_dev,
                                 int32_t batch, int32_t t_fresh, const int32_t *slot_ids_host,
                                 const int32_t *used_len_host, const int32_t *n_chunks_host, int32_t max_chunks,
                                 void *attn_out_dev, void *k_fresh_out_dev, void *v_fresh_out_dev, void *workspace_dev,
                                 size_t workspace_bytes, void *stream) {
  return run_prefill(ctx, layer, x_fresh_dev, wqkv_dev, batch, t_fresh, slot_ids_host, used_len_host, n_chunks_host, max_chunks,
                     attn_out_dev, k_fresh_out_dev, v_fresh_out_dev, workspace_dev, workspace_bytes, stream, nullptr, nullptr);
}

pc_status percache_prefill_reuse_table(percache_ctx *ctx, int32_t layer, const void *x_fresh_dev, const void *wqkv_dev,
                                       int32_t batch, int32_t t_fresh, const void *table_dev, void *attn_out_dev,
                                       void *k_fresh_out_dev, void *v_fresh_out_dev, void *workspace_dev,
                                       size_t workspace_bytes, void *stream) {
  if (!ctx) return PC_EINVAL;
  const pc_table_shadow *sh = pc::find_table(ctx, table_dev, batch);
  if (!sh) return PC_EINVAL;
  return run_prefill(ctx, layer, x_fresh_dev, wqkv_dev, batch, t_fresh, sh->ids.data(), sh->used.data(), sh->n_chunks.data(),
                     sh->max_chunks, attn_out_dev, k_fresh_out_dev, v_fresh_out_dev, workspace_dev, workspace_bytes, stream,
                     (const int32_t *)table_dev, sh);
}

}  // extern "C"
