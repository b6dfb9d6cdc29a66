// Context life cycle, arena layout, RoPE table, chunk-table validation and staging.
#include <cmath>
#include <cstring>

#include "percache_internal.hpp"

namespace {
thread_local std::string g_create_err;

// Scratch of the entry points that allocate nothing (partial results of the lookup pass).  Every GPU holds its own
// copy of this array at its own address; in host code the array's name is only a stand-in for hipGetSymbolAddress,
// never a pointer to hand to a kernel.  Address per device, resolved at percache_create with that device current.
__device__ __align__(256) unsigned char scratch[pc::kStaticScratchBytes];
constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices] = {};

bool config_ok(const percache_config *c, std::string &why) {
  char buf[256];
  auto bad = [&](const char *m) { why = m; return false; };
  if (!c) return bad("config is NULL");
  if (c->n_layers < 1 || c->hidden < 64 || c->n_q_heads < 1 || c->n_kv_heads < 1 || c->n_slots < 1 ||
      c->slot_capacity < 1 || c->max_pos < 1 || c->bank_capacity < 0)
    return bad("non-positive dimension in config");
  if (c->head_dim != 64 && c->head_dim != 128) return bad("head_dim must be 64 or 128");
  if (c->hidden % 64) return bad("hidden must be a multiple of 64");
  if (c->n_q_heads % c->n_kv_heads) return bad("n_q_heads must be a multiple of n_kv_heads");
  if (c->slot_capacity % 64) return bad("slot_capacity must be a multiple of 64");
  if (c->bank_capacity > 0 && (c->emb_dim < 64 || c->emb_dim % 64 || c->emb_dim > 2048))
    return bad("emb_dim must be a multiple of 64 in [64, 2048]");
  if (!(c->rope_theta > 1.0f)) return bad("rope_theta must exceed 1");
  if (c->kv_fp8 != 0 && c->kv_fp8 != 1) return bad("kv_fp8 must be 0 or 1");
  if (c->n_slots_8bit < 0 || c->n_slots_8bit > c->n_slots) return bad("n_slots_8bit must lie in [0, n_slots]");
  if (c->kv_fp8 && c->n_slots_8bit) return bad("n_slots_8bit must be 0 when every slot is 8-bit (kv_fp8 = 1)");
  if (((c->n_q_heads + 2 * c->n_kv_heads) * c->head_dim) % 128) return bad("(n_q_heads + 2 n_kv_heads) * head_dim must be a multiple of 128");
  (void)buf;
  return true;
}

struct Layout {
  size_t rope, bank, bank_inv, k_store, v_store, k8_store, v8_store, k_scale, v_scale, total;
};
Layout layout_of(const percache_config &c) {
  Layout l;
  size_t off = 0;
  l.rope = off;
  off += pc::align_up((size_t)c.max_pos * (c.head_dim / 2) * 2 * sizeof(float));
  l.bank = off;
  off += pc::align_up((size_t)c.bank_capacity * (size_t)(c.bank_capacity ? c.emb_dim : 0) * 2);
  l.bank_inv = off;
  off += pc::align_up((size_t)c.bank_capacity * sizeof(float));
  const size_t n8 = c.kv_fp8 ? c.n_slots : c.n_slots_8bit, n16 = c.n_slots - n8;
  const size_t per_slot = (size_t)c.n_layers * c.n_kv_heads * c.slot_capacity * c.head_dim;
  l.k_store = off;
  off += pc::align_up(n16 * per_slot * 2);
  l.v_store = off;
  off += pc::align_up(n16 * per_slot * 2);
  l.k8_store = off;
  off += pc::align_up(n8 * per_slot);
  l.v8_store = off;
  off += pc::align_up(n8 * per_slot);
  size_t scales = (size_t)c.n_layers * n8 * c.n_kv_heads * (c.slot_capacity / pc::kKvTile) * sizeof(float);
  l.k_scale = off;
  off += pc::align_up(scales);
  l.v_scale = off;
  off += pc::align_up(scales);
  l.total = off;
  return l;
}
}  // namespace

namespace pc {
pc_status fail(percache_ctx *ctx, pc_status st, const char *fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (ctx) ctx->err = buf; else g_create_err = buf;
  return st;
}

pc_status build_chunk_table(percache_ctx *ctx, int32_t layer, int32_t batch, int32_t t_fresh,
                            const int32_t *slot_ids, const int32_t *used_len, const int32_t *n_chunks,
                            int32_t max_chunks, std::vector<int32_t> &rows) {
  const percache_config &c = ctx->cfg;
  if (batch < 1 || t_fresh < 1) return fail(ctx, PC_EINVAL, "batch and t_fresh must be positive");
  if (max_chunks < 0) return fail(ctx, PC_EINVAL, "max_chunks is negative");
  if (layer < 0 || layer >= c.n_layers) return fail(ctx, PC_ESLOT, "layer %d out of range [0,%d)", layer, c.n_layers);
  if (!n_chunks) return fail(ctx, PC_EINVAL, "n_chunks_host is NULL");
  if (max_chunks > 0 && !slot_ids) return fail(ctx, PC_EINVAL, "slot_ids_host is NULL");
  const int stride = tbl_stride(max_chunks);
  rows.assign((size_t)batch * stride, 0);
  for (int b = 0; b < batch; ++b) {
    int nc = n_chunks[b];
    if (nc < 0 || nc > max_chunks) return fail(ctx, PC_EINVAL, "n_chunks[%d]=%d outside [0,%d]", b, nc, max_chunks);
    int32_t *row = rows.data() + (size_t)b * stride;
    long l_pre = 0, tiles = 0;
    for (int ci = 0; ci < nc; ++ci) {
      int slot = slot_ids[(size_t)b * max_chunks + ci];
      if (slot < 0 || slot >= c.n_slots) return fail(ctx, PC_ESLOT, "query %d chunk %d: slot %d out of range [0,%d)", b, ci, slot, c.n_slots);
      int stored = ctx->slot_len[(size_t)layer * c.n_slots + slot];
      if (stored <= 0) return fail(ctx, PC_ESLOT, "query %d chunk %d: slot %d of layer %d is empty", b, ci, slot, layer);
      int used = used_len ? used_len[(size_t)b * max_chunks + ci] : stored;
      if (used < 0 || used > stored) return fail(ctx, PC_ELEN, "query %d chunk %d: used length %d outside [0,%d]", b, ci, used, stored);
      row[kTblHeader + 2 * ci] = slot;
      row[kTblHeader + 2 * ci + 1] = used;
      if (used > 0) row[3] |= ctx->is8(slot) ? 1 : 2;
      l_pre += used;
      tiles += (used + kKvTile - 1) / kKvTile;
    }
    if (l_pre + t_fresh > c.max_pos) return fail(ctx, PC_ELEN, "query %d: L_pre %ld + t_fresh %d exceeds max_pos %d", b, l_pre, t_fresh, c.max_pos);
    row[0] = nc;
    row[1] = (int32_t)l_pre;
    row[2] = (int32_t)tiles;
  }
  return PC_OK;
}

pc_status upload_table(percache_ctx *ctx, const std::vector<int32_t> &rows, int32_t *dst_dev, hipStream_t stream) {
  if (rows.size() > ctx->stage_ints) {
    // grow every ring entry (host allocation only); wait for copies still reading the old ones
    for (int i = 0; i < kStageRing; ++i) {
      if (ctx->stage_used[i]) PC_HIP(ctx, hipEventSynchronize(ctx->stage_ev[i]));
      ctx->stage_used[i] = false;
      if (ctx->stage[i]) PC_HIP(ctx, hipHostFree(ctx->stage[i]));
      ctx->stage[i] = nullptr;
    }
    size_t want = rows.size() * 2;
    for (int i = 0; i < kStageRing; ++i) PC_HIP(ctx, hipHostMalloc((void **)&ctx->stage[i], want * sizeof(int32_t), hipHostMallocDefault));
    ctx->stage_ints = want;
  }
  int i = ctx->stage_next;
  ctx->stage_next = (i + 1) % kStageRing;
  if (ctx->stage_used[i]) PC_HIP(ctx, hipEventSynchronize(ctx->stage_ev[i]));
  memcpy(ctx->stage[i], rows.data(), rows.size() * sizeof(int32_t));
  PC_HIP(ctx, hipMemcpyAsync(dst_dev, ctx->stage[i], rows.size() * sizeof(int32_t), hipMemcpyHostToDevice, stream));
  PC_HIP(ctx, hipEventRecord(ctx->stage_ev[i], stream));
  ctx->stage_used[i] = true;
  return PC_OK;
}

const pc_table_shadow *find_table(percache_ctx *ctx, const void *table_dev, int32_t batch) {
  auto it = ctx->tables.find(table_dev);
  if (!table_dev || it == ctx->tables.end()) {
    fail(ctx, PC_EINVAL, "table_dev %p was not written by percache_chunk_table_put on this context", table_dev);
    return nullptr;
  }
  if (it->second.batch != batch) {
    fail(ctx, PC_EINVAL, "the chunk table holds %d queries, the call has %d", it->second.batch, batch);
    return nullptr;
  }
  return &it->second;
}

int max_splits_for(const percache_config &c, int n_cu, int32_t batch, int32_t t_fresh) {
  long rows = (long)(c.n_q_heads / c.n_kv_heads) * t_fresh;
  long base = (long)batch * c.n_kv_heads * ((rows + 127) / 128);
  long s = (2L * n_cu + base - 1) / base;
  if (s < 4) s = 4;
  if (s > kMaxSplits) s = kMaxSplits;
  return (int)s;
}

void prof_begin(percache_ctx *ctx, int kind, hipStream_t stream) {
  if (!(ctx->prof_mask >> kind & 1) || ctx->prof_n[kind] >= kProfMax) return;
  (void)hipEventRecord(ctx->prof_beg[kind][ctx->prof_n[kind]], stream);
}
void prof_end(percache_ctx *ctx, int kind, hipStream_t stream) {
  if (!(ctx->prof_mask >> kind & 1) || ctx->prof_n[kind] >= kProfMax) return;
  (void)hipEventRecord(ctx->prof_end[kind][ctx->prof_n[kind]], stream);
  ++ctx->prof_n[kind];
}

PrefillWs carve_prefill_ws(const percache_config &c, int n_cu, void *base, int32_t batch, int32_t t_fresh, int32_t max_chunks) {
  PrefillWs w;
  char *p = (char *)base;
  size_t off = 0;
  auto take = [&](size_t bytes) { char *r = p ? p + off : nullptr; off += align_up(bytes); return r; };
  w.table = (int32_t *)take((size_t)batch * tbl_stride(max_chunks) * sizeof(int32_t));
  size_t qn = (size_t)batch * c.n_q_heads * t_fresh * c.head_dim;
  size_t kn = (size_t)batch * c.n_kv_heads * t_fresh * c.head_dim;
  w.q = (__bf16 *)take(qn * 2);
  w.k = (__bf16 *)take(kn * 2);
  w.v = (__bf16 *)take(kn * 2);
  w.v_blk = (__bf16 *)take((size_t)batch * c.n_kv_heads * ((t_fresh + kKvTile - 1) / kKvTile) * kKvTile * c.head_dim * 2);
  const size_t M = (size_t)batch * t_fresh;
  w.gemm_part = (float *)take(splitk_applies((long)M) ? (size_t)kMaxSplitK * M * (c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim * sizeof(float) : 0);
  size_t rows = (size_t)batch * c.n_q_heads * t_fresh;
  w.max_splits = max_splits_for(c, n_cu, batch, t_fresh);
  w.part_o = (__bf16 *)take(rows * w.max_splits * c.head_dim * 2);
  w.part_ml = (float *)take(rows * w.max_splits * 2 * sizeof(float));
  w.total = off;
  return w;
}
}  // namespace pc

extern "C" {

size_t percache_arena_bytes(const percache_config *cfg) {
  std::string why;
  if (!config_ok(cfg, why)) return 0;
  return layout_of(*cfg).total;
}

pc_status percache_create(const percache_config *cfg, void *arena_dev, size_t arena_bytes, percache_ctx **out) {
  std::string why;
  if (!out) return pc::fail(nullptr, PC_EINVAL, "out is NULL");
  *out = nullptr;
  if (!config_ok(cfg, why)) return pc::fail(nullptr, PC_ESHAPE, "%s", why.c_str());
  if (!arena_dev) return pc::fail(nullptr, PC_EINVAL, "arena is NULL");
  if ((uintptr_t)arena_dev % pc::kAlign) return pc::fail(nullptr, PC_EINVAL, "arena must be 256-byte aligned");
  Layout l = layout_of(*cfg);
  if (arena_bytes < l.total) return pc::fail(nullptr, PC_ENOMEM, "arena has %zu bytes, need %zu", arena_bytes, l.total);

  percache_ctx *ctx = new percache_ctx;
  ctx->cfg = *cfg;
  ctx->arena = (char *)arena_dev;
  ctx->arena_bytes = arena_bytes;
  ctx->rope = (float *)(ctx->arena + l.rope);
  ctx->bank = (_Float16 *)(ctx->arena + l.bank);
  ctx->bank_inv = (float *)(ctx->arena + l.bank_inv);
  ctx->n_slots8 = cfg->kv_fp8 ? cfg->n_slots : cfg->n_slots_8bit;
  ctx->n_slots16 = cfg->n_slots - ctx->n_slots8;
  ctx->k_store = (__bf16 *)(ctx->arena + l.k_store);
  ctx->v_store = (__bf16 *)(ctx->arena + l.v_store);
  ctx->k8_store = (uint8_t *)(ctx->arena + l.k8_store);
  ctx->v8_store = (uint8_t *)(ctx->arena + l.v8_store);
  ctx->k_scale = (float *)(ctx->arena + l.k_scale);
  ctx->v_scale = (float *)(ctx->arena + l.v_scale);
  ctx->slot_stride = (size_t)cfg->n_kv_heads * cfg->slot_capacity * cfg->head_dim;
  ctx->layer_stride = ctx->slot_stride * ctx->n_slots16;
  ctx->layer_stride8 = ctx->slot_stride * ctx->n_slots8;
  ctx->slot_len.assign((size_t)cfg->n_layers * cfg->n_slots, 0);

  auto bail = [&](hipError_t e, const char *what) {
    pc::fail(nullptr, PC_EHIP, "%s: %s", what, hipGetErrorString(e));
    percache_destroy(ctx);
    return PC_EHIP;
  };
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return bail(e, "hipGetDevice");
  hipDeviceProp_t prop;
  e = hipGetDeviceProperties(&prop, dev);
  if (e != hipSuccess) return bail(e, "hipGetDeviceProperties");
  ctx->n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
  if (dev < 0 || dev >= kMaxDevices) return bail(hipErrorInvalidDevice, "device ordinal beyond the library's table");
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return bail(e, "hipGetSymbolAddress(scratch)");
    g_scratch_ptr[dev] = p;
  }
  ctx->static_scratch = g_scratch_ptr[dev];
  for (int i = 0; i < pc::kStageRing; ++i) {
    e = hipEventCreateWithFlags(&ctx->stage_ev[i], hipEventDisableTiming);
    if (e != hipSuccess) return bail(e, "hipEventCreate");
  }

  // RoPE table (App. B.1: sine/cosine lookup indexed by absolute position), built in double.
  const int half = cfg->head_dim / 2;
  std::vector<float> tab((size_t)cfg->max_pos * half * 2);
  std::vector<double> inv_freq(half);
  for (int m = 0; m < half; ++m) inv_freq[m] = std::pow((double)cfg->rope_theta, -2.0 * m / cfg->head_dim);
  for (int p = 0; p < cfg->max_pos; ++p)
    for (int m = 0; m < half; ++m) {
      double a = (double)p * inv_freq[m];
      tab[((size_t)p * half + m) * 2] = (float)std::cos(a);
      tab[((size_t)p * half + m) * 2 + 1] = (float)std::sin(a);
    }
  e = hipMemcpy(ctx->rope, tab.data(), tab.size() * sizeof(float), hipMemcpyHostToDevice);
  if (e != hipSuccess) return bail(e, "hipMemcpy(rope table)");
  e = hipDeviceSynchronize();
  if (e != hipSuccess) return bail(e, "hipDeviceSynchronize");
  *out = ctx;
  return PC_OK;
}

void percache_destroy(percache_ctx *ctx) {
  if (!ctx) return;
  for (int i = 0; i < pc::kStageRing; ++i) {
    if (ctx->stage_used[i]) (void)hipEventSynchronize(ctx->stage_ev[i]);
    if (ctx->stage[i]) (void)hipHostFree(ctx->stage[i]);
    if (ctx->stage_ev[i]) (void)hipEventDestroy(ctx->stage_ev[i]);
  }
  for (int k = 0; k < 3; ++k) {
    for (hipEvent_t e : ctx->prof_beg[k]) (void)hipEventDestroy(e);
    for (hipEvent_t e : ctx->prof_end[k]) (void)hipEventDestroy(e);
  }
  delete ctx;
}

size_t percache_chunk_table_bytes(const percache_ctx *ctx, int32_t batch, int32_t max_chunks) {
  if (!ctx || batch < 1 || max_chunks < 0) return 0;
  return pc::align_up((size_t)batch * pc::tbl_stride(max_chunks) * sizeof(int32_t));
}

pc_status percache_chunk_table_put(percache_ctx *ctx, void *table_dev, size_t table_bytes, int32_t layer, int32_t batch,
                                   const int32_t *slot_ids_host, const int32_t *used_len_host,
                                   const int32_t *n_chunks_host, int32_t max_chunks, void *stream) {
  if (!ctx) return PC_EINVAL;
  if (!table_dev || (uintptr_t)table_dev % 16) return pc::fail(ctx, PC_EINVAL, "table_dev is NULL or not 16-byte aligned");
  pc_table_shadow sh;
  // (a list is valid for every call whose fresh length still fits max_pos: checked against one fresh token here, against
  // the real count by the call that uses the table)
  pc_status st = pc::build_chunk_table(ctx, layer, batch, 1, slot_ids_host, used_len_host, n_chunks_host, max_chunks, sh.rows);
  if (st != PC_OK) return st;
  const size_t need = percache_chunk_table_bytes(ctx, batch, max_chunks);
  if (table_bytes < need) return pc::fail(ctx, PC_ENOMEM, "chunk table has %zu bytes, need %zu", table_bytes, need);
  const int stride = pc::tbl_stride(max_chunks);
  sh.batch = batch;
  sh.max_chunks = max_chunks;
  sh.ids.assign((size_t)batch * max_chunks, 0);
  sh.used.assign((size_t)batch * max_chunks, 0);
  sh.n_chunks.assign(n_chunks_host, n_chunks_host + batch);
  for (int b = 0; b < batch; ++b)
    for (int ci = 0; ci < n_chunks_host[b]; ++ci) {
      sh.ids[(size_t)b * max_chunks + ci] = sh.rows[(size_t)b * stride + pc::kTblHeader + 2 * ci];
      sh.used[(size_t)b * max_chunks + ci] = sh.rows[(size_t)b * stride + pc::kTblHeader + 2 * ci + 1];
    }
  st = pc::upload_table(ctx, sh.rows, (int32_t *)table_dev, (hipStream_t)stream);
  if (st != PC_OK) return st;
  ctx->tables[table_dev] = std::move(sh);
  return PC_OK;
}

pc_status percache_chunk_table_drop(percache_ctx *ctx, const void *table_dev) {
  if (!ctx) return PC_EINVAL;
  if (!ctx->tables.erase(table_dev)) return pc::fail(ctx, PC_EINVAL, "table_dev %p is not known to this context", table_dev);
  return PC_OK;
}

pc_status percache_profile_enable(percache_ctx *ctx, int32_t on) {
  if (!ctx) return PC_EINVAL;
  if (on < 0 || on > 15) return pc::fail(ctx, PC_EINVAL, "profile switch %d: 0, 1 or a mask of bits 1..3", on);
  if (on && ctx->prof_beg[0].empty()) {
    for (int k = 0; k < 3; ++k) {
      ctx->prof_beg[k].resize(pc::kProfMax);
      ctx->prof_end[k].resize(pc::kProfMax);
      for (int i = 0; i < pc::kProfMax; ++i) {
        PC_HIP(ctx, hipEventCreate(&ctx->prof_beg[k][i]));
        PC_HIP(ctx, hipEventCreate(&ctx->prof_end[k][i]));
      }
    }
  }
  ctx->prof_mask = on == 1 ? 7u : ((unsigned)on >> 1) & 7u;
  for (int k = 0; k < 3; ++k) ctx->prof_n[k] = 0;
  return PC_OK;
}

pc_status percache_profile_read(percache_ctx *ctx, int32_t kernel, float *sum_ms_host, int32_t *count_host) {
  if (!ctx) return PC_EINVAL;
  if (kernel < 0 || kernel > 2 || !sum_ms_host || !count_host) return pc::fail(ctx, PC_EINVAL, "bad kernel id or NULL output");
  float sum = 0.f;
  int n = ctx->prof_n[kernel];
  for (int i = 0; i < n; ++i) {
    PC_HIP(ctx, hipEventSynchronize(ctx->prof_end[kernel][i]));
    float ms = 0.f;
    PC_HIP(ctx, hipEventElapsedTime(&ms, ctx->prof_beg[kernel][i], ctx->prof_end[kernel][i]));
    sum += ms;
  }
  *sum_ms_host = sum;
  *count_host = n;
  ctx->prof_n[kernel] = 0;
  return PC_OK;
}

const char *percache_last_error(const percache_ctx *ctx) { return ctx ? ctx->err.c_str() : g_create_err.c_str(); }

int32_t percache_bank_size(const percache_ctx *ctx) { return ctx ? ctx->bank_size : PC_EINVAL; }

}  // extern "C"
