// Slot-indexed per-layer K/V store: the device-resident form of the per-chunk tensor files of
// Sec. 4.1.1 (cache slicer output).  Store layout per layer: [slot][kv head][token][head_dim] bf16,
// so one (slot, head) tile is a single contiguous run that the attention kernel streams.
#include "percache_internal.hpp"

namespace {

// Copies Hkv runs of n_tok*D elements between the caller's dense [Hkv, n_tok, D] tensor and the
// slot's [Hkv, C, D] region, 16 bytes per lane.  blockIdx.y selects K (0) or V (1).
template <bool kToStore>
__global__ __launch_bounds__(256) void kv_copy_kernel(uint4 *__restrict__ slot_k, uint4 *__restrict__ slot_v,
                                                      uint4 *__restrict__ dense_k, uint4 *__restrict__ dense_v,
                                                      int n_heads, int run_vec, int slot_head_vec) {
  uint4 *slot = blockIdx.y ? slot_v : slot_k;
  uint4 *dense = blockIdx.y ? dense_v : dense_k;
  const long total = (long)n_heads * run_vec;
  for (long e = (long)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (long)gridDim.x * blockDim.x) {
    int g = (int)(e / run_vec);
    int r = (int)(e - (long)g * run_vec);
    long s = (long)g * slot_head_vec + r;
    if (kToStore) slot[s] = dense[e]; else dense[e] = slot[s];
  }
}

pc_status check_slot(percache_ctx *ctx, int32_t layer, int32_t slot) {
  if (!ctx) return PC_EINVAL;
  if (layer < 0 || layer >= ctx->cfg.n_layers) return pc::fail(ctx, PC_ESLOT, "layer %d out of range [0,%d)", layer, ctx->cfg.n_layers);
  if (slot < 0 || slot >= ctx->cfg.n_slots) return pc::fail(ctx, PC_ESLOT, "slot %d out of range [0,%d)", slot, ctx->cfg.n_slots);
  return PC_OK;
}

}  // namespace

extern "C" {

pc_status percache_kv_put(percache_ctx *ctx, int32_t layer, int32_t slot, const void *k_dev, const void *v_dev,
                          int32_t n_tokens, void *stream) {
  pc_status st = check_slot(ctx, layer, slot);
  if (st != PC_OK) return st;
  if (!k_dev || !v_dev) return pc::fail(ctx, PC_EINVAL, "k_dev / v_dev is NULL");
  if (((uintptr_t)k_dev | (uintptr_t)v_dev) % 16) return pc::fail(ctx, PC_EINVAL, "k_dev / v_dev must be 16-byte aligned");
  const percache_config &c = ctx->cfg;
  if (n_tokens < 1 || n_tokens > c.slot_capacity) return pc::fail(ctx, PC_ELEN, "n_tokens %d outside [1,%d]", n_tokens, c.slot_capacity);
  size_t off = (size_t)layer * ctx->layer_stride + (size_t)slot * ctx->slot_stride;
  int run_vec = n_tokens * c.head_dim / 8;
  int slot_head_vec = c.slot_capacity * c.head_dim / 8;
  long total = (long)c.n_kv_heads * run_vec;
  int blocks = (int)((total + 255) / 256);
  if (blocks > 2048) blocks = 2048;
  hipLaunchKernelGGL(kv_copy_kernel<true>, dim3(blocks, 2), dim3(256), 0, (hipStream_t)stream,
                     (uint4 *)(ctx->k_store + off), (uint4 *)(ctx->v_store + off), (uint4 *)k_dev, (uint4 *)v_dev,
                     c.n_kv_heads, run_vec, slot_head_vec);
  PC_HIP(ctx, hipGetLastError());
  ctx->slot_len[(size_t)layer * c.n_slots + slot] = n_tokens;
  return PC_OK;
}

pc_status percache_kv_get(percache_ctx *ctx, int32_t layer, int32_t slot, void *k_out_dev, void *v_out_dev,
                          int32_t *n_tokens_out_host, void *stream) {
  pc_status st = check_slot(ctx, layer, slot);
  if (st != PC_OK) return st;
  if (!k_out_dev || !v_out_dev) return pc::fail(ctx, PC_EINVAL, "k_out_dev / v_out_dev is NULL");
  if (((uintptr_t)k_out_dev | (uintptr_t)v_out_dev) % 16) return pc::fail(ctx, PC_EINVAL, "outputs must be 16-byte aligned");
  const percache_config &c = ctx->cfg;
  int n_tokens = ctx->slot_len[(size_t)layer * c.n_slots + slot];
  if (n_tokens <= 0) return pc::fail(ctx, PC_ESLOT, "slot %d of layer %d is empty", slot, layer);
  size_t off = (size_t)layer * ctx->layer_stride + (size_t)slot * ctx->slot_stride;
  int run_vec = n_tokens * c.head_dim / 8;
  int slot_head_vec = c.slot_capacity * c.head_dim / 8;
  long total = (long)c.n_kv_heads * run_vec;
  int blocks = (int)((total + 255) / 256);
  if (blocks > 2048) blocks = 2048;
  hipLaunchKernelGGL(kv_copy_kernel<false>, dim3(blocks, 2), dim3(256), 0, (hipStream_t)stream,
                     (uint4 *)(ctx->k_store + off), (uint4 *)(ctx->v_store + off), (uint4 *)k_out_dev,
                     (uint4 *)v_out_dev, c.n_kv_heads, run_vec, slot_head_vec);
  PC_HIP(ctx, hipGetLastError());
  if (n_tokens_out_host) *n_tokens_out_host = n_tokens;
  return PC_OK;
}

pc_status percache_kv_evict(percache_ctx *ctx, int32_t layer, int32_t slot) {
  pc_status st = check_slot(ctx, layer, slot);
  if (st != PC_OK) return st;
  ctx->slot_len[(size_t)layer * ctx->cfg.n_slots + slot] = 0;
  return PC_OK;
}

int32_t percache_kv_len(const percache_ctx *ctx, int32_t layer, int32_t slot) {
  if (!ctx) return PC_EINVAL;
  if (layer < 0 || layer >= ctx->cfg.n_layers || slot < 0 || slot >= ctx->cfg.n_slots) return PC_ESLOT;
  return ctx->slot_len[(size_t)layer * ctx->cfg.n_slots + slot];
}

}  // extern "C"
