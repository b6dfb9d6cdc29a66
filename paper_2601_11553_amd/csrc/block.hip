// The rest of a pre-norm transformer block around the cache-reusing attention module, on the retained (fresh)
// rows only, so that a stack of layers can be chained (App. B.1: after the attention module the computation
// goes on as in an ordinary block; the cached rows' activations are never needed again because the next layer
// crops them once more):
//   h' = h + (attention(RMSNorm(h) ...)) Wo^T,   h'' = h' + (silu(n Wgate^T) * (n Wup^T)) Wdown^T,  n = RMSNorm(h').
// Kernels: a row-wise RMSNorm, and the shared projection main loop with two epilogues (residual add; SwiGLU on a
// gate/up feature pair held by the same lane).  percache_stack_reuse chains the layers; percache_kv_slice is the
// cache slicer of Sec. 4.1.1 (cuts the K/V of a prefilled sequence at chunk boundaries into slots).
#include <cstring>

#include "gemm_tile.hpp"

namespace {
using pc::f32x16;
using pc::u32x4;
using pc::gemm::BF;
using pc::gemm::pack4;
using pc::gemm::unpack4;

// ---------------------------------------------------------------------------------------------------
// y = x / sqrt(mean(x^2) + eps) * gain; one wavefront per row, fp32 arithmetic, bf16 in and out.
// ---------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void rmsnorm_kernel(const __bf16 *__restrict__ X, const __bf16 *__restrict__ gain,
                                                      __bf16 *__restrict__ Y, int M, int H, float eps) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= M) return;
  const u32x4 *x = (const u32x4 *)(X + (size_t)row * H);
  const u32x4 *gv = (const u32x4 *)gain;
  u32x4 *y = (u32x4 *)(Y + (size_t)row * H);
  const int nv = H / 8;
  float ss = 0.f;
  for (int v = lane; v < nv; v += 64) {
    pc::bf16x8 h = __builtin_bit_cast(pc::bf16x8, x[v]);
#pragma unroll
    for (int e = 0; e < 8; ++e) ss += (float)h[e] * (float)h[e];
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
  const float r = 1.0f / sqrtf(ss / (float)H + eps);
  for (int v = lane; v < nv; v += 64) {
    pc::bf16x8 h = __builtin_bit_cast(pc::bf16x8, x[v]);
    pc::bf16x8 gq = __builtin_bit_cast(pc::bf16x8, gv[v]);
    pc::bf16x8 o;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = (__bf16)((float)h[e] * r * (float)gq[e]);
    y[v] = __builtin_bit_cast(u32x4, o);
  }
}

// ---------------------------------------------------------------------------------------------------
// Y[M, N] = A[M, K] W[N, K]^T + R[M, N]   (o_proj and down projection with the residual add fused)
// ---------------------------------------------------------------------------------------------------
template <int NTB>
__global__ __launch_bounds__(256, 2) void linear_residual_kernel(const __bf16 *__restrict__ A, const __bf16 *__restrict__ W,
                                                                 const __bf16 *__restrict__ R, __bf16 *__restrict__ Y, int M,
                                                                 int N, int K) {
  constexpr int BT = 64 * NTB;
  __shared__ __align__(16) char lds[pc::gemm::Shape<NTB>::LDS_BYTES];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wf = wave & 1, wt = wave >> 1;
  const int l32 = lane & 31, g = lane >> 5;
  const int f0 = blockIdx.x * BF, m0 = blockIdx.y * BT;
  f32x16 acc[2][NTB];
  pc::gemm::mainloop<NTB>(lds, [&](int row) __attribute__((always_inline)) { return W + (size_t)(f0 + row) * K; }, A, m0, M,
                          K, 2 * wf, 2 * wf + 1, acc);
#pragma unroll
  for (int t = 0; t < NTB; ++t) {
    const int m_raw = m0 + (wt * NTB + t) * 32 + l32;
    const bool ok = m_raw < M;
    const int m = ok ? m_raw : M - 1;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const size_t at = (size_t)m * N + f0 + (2 * wf + a) * 32 + q4 * 8 + g * 4;
        float res[4];
        unpack4(*(const uint2 *)(R + at), res);
        if (ok)
          *(uint2 *)(Y + at) = pack4(acc[a][t][q4 * 4 + 0] + res[0], acc[a][t][q4 * 4 + 1] + res[1],
                                   acc[a][t][q4 * 4 + 2] + res[2], acc[a][t][q4 * 4 + 3] + res[3]);
      }
  }
}

// ---------------------------------------------------------------------------------------------------
// Y[M, F] = silu(A Wgate^T) * (A Wup^T).  A workgroup takes 64 gate rows and the 64 up rows of the same
// features; wavefront wf owns gate block wf and up block wf + 2, so both halves of a product sit in one lane.
// ---------------------------------------------------------------------------------------------------
template <int NTB>
__global__ __launch_bounds__(256, 2) void linear_swiglu_kernel(const __bf16 *__restrict__ A, const __bf16 *__restrict__ Wg,
                                                               const __bf16 *__restrict__ Wu, __bf16 *__restrict__ Y, int M,
                                                               int F, int K) {
  constexpr int BT = 64 * NTB;
  __shared__ __align__(16) char lds[pc::gemm::Shape<NTB>::LDS_BYTES];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wf = wave & 1, wt = wave >> 1;
  const int l32 = lane & 31, g = lane >> 5;
  const int f0 = blockIdx.x * (BF / 2), m0 = blockIdx.y * BT;
  f32x16 acc[2][NTB];
  pc::gemm::mainloop<NTB>(
      lds, [&](int row) __attribute__((always_inline)) { return (row < 64 ? Wg : Wu) + (size_t)(f0 + (row & 63)) * K; }, A, m0, M, K,
      wf, wf + 2, acc);
#pragma unroll
  for (int t = 0; t < NTB; ++t) {
    const int m_raw = m0 + (wt * NTB + t) * 32 + l32;
    const bool ok = m_raw < M;
    const int m = ok ? m_raw : M - 1;
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      float o[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float gate = acc[0][t][q4 * 4 + e], up = acc[1][t][q4 * 4 + e];
        o[e] = gate / (1.0f + __expf(-gate)) * up;
      }
      if (ok) *(uint2 *)(Y + (size_t)m * F + f0 + wf * 32 + q4 * 8 + g * 4) = pack4(o[0], o[1], o[2], o[3]);
    }
  }
}

bool aligned16(const void *p) { return ((uintptr_t)p % 16) == 0; }

pc_status launch_rmsnorm(percache_ctx *ctx, const __bf16 *x, const __bf16 *gain, __bf16 *y, int M, int H, float eps,
                         hipStream_t s) {
  hipLaunchKernelGGL(rmsnorm_kernel, dim3((M + 3) / 4), dim3(256), 0, s, x, gain, y, M, H, eps);
  PC_HIP(ctx, hipGetLastError());
  return PC_OK;
}
pc_status launch_linear_residual(percache_ctx *ctx, const __bf16 *a, const __bf16 *w, const __bf16 *res, __bf16 *y, int M,
                                 int N, int K, hipStream_t s) {
  const bool big = M > 64 * 3;
  dim3 grid(N / BF, big ? (M + 127) / 128 : (M + 63) / 64);
  if (big) hipLaunchKernelGGL(linear_residual_kernel<2>, grid, dim3(256), 0, s, a, w, res, y, M, N, K);
  else hipLaunchKernelGGL(linear_residual_kernel<1>, grid, dim3(256), 0, s, a, w, res, y, M, N, K);
  PC_HIP(ctx, hipGetLastError());
  return PC_OK;
}
pc_status launch_linear_swiglu(percache_ctx *ctx, const __bf16 *a, const __bf16 *wg, const __bf16 *wu, __bf16 *y, int M, int F,
                               int K, hipStream_t s) {
  const bool big = M > 64 * 3;
  dim3 grid(F / (BF / 2), big ? (M + 127) / 128 : (M + 63) / 64);
  if (big) hipLaunchKernelGGL(linear_swiglu_kernel<2>, grid, dim3(256), 0, s, a, wg, wu, y, M, F, K);
  else hipLaunchKernelGGL(linear_swiglu_kernel<1>, grid, dim3(256), 0, s, a, wg, wu, y, M, F, K);
  PC_HIP(ctx, hipGetLastError());
  return PC_OK;
}

// Workspace of the stack call: the prefill workspace followed by the block's own activations.
struct StackWs {
  pc::PrefillWs pf;
  __bf16 *normed;  // [M, H]
  __bf16 *attn;    // [M, Hq*D]
  __bf16 *mid;     // [M, H]
  __bf16 *act;     // [M, F]
  size_t total;
};
StackWs carve_stack_ws(const percache_ctx *ctx, void *base, int batch, int t_fresh, int max_chunks, int ffn) {
  const percache_config &c = ctx->cfg;
  StackWs w;
  w.pf = pc::carve_prefill_ws(c, ctx->n_cu, base, batch, t_fresh, max_chunks);
  size_t off = w.pf.total;
  char *p = (char *)base;
  auto take = [&](size_t bytes) { char *r = p ? p + off : nullptr; off += pc::align_up(bytes); return (__bf16 *)r; };
  const size_t M = (size_t)batch * t_fresh;
  w.normed = take(M * c.hidden * 2);
  w.attn = take(M * c.n_q_heads * c.head_dim * 2);
  w.mid = take(M * c.hidden * 2);
  w.act = take(M * ffn * 2);
  w.total = off;
  return w;
}

}  // namespace

extern "C" {

pc_status percache_kv_slice(percache_ctx *ctx, int32_t layer, const void *k_dev, const void *v_dev, int32_t seq_len,
                            const int32_t *bounds_host, const int32_t *slots_host, int32_t n, void *stream) {
  if (!ctx) return PC_EINVAL;
  const percache_config &c = ctx->cfg;
  if (!k_dev || !v_dev || !bounds_host || !slots_host) return pc::fail(ctx, PC_EINVAL, "NULL pointer");
  if (!aligned16(k_dev) || !aligned16(v_dev)) return pc::fail(ctx, PC_EINVAL, "k_dev / v_dev must be 16-byte aligned");
  if (n < 1 || seq_len < 1) return pc::fail(ctx, PC_EINVAL, "n and seq_len must be positive");
  if (layer < 0 || layer >= c.n_layers) return pc::fail(ctx, PC_ESLOT, "layer %d out of range [0,%d)", layer, c.n_layers);
  for (int j = 0; j < n; ++j) {
    const int lo = bounds_host[j], hi = bounds_host[j + 1];
    if (lo < 0 || hi > seq_len || hi <= lo) return pc::fail(ctx, PC_ELEN, "chunk %d: bounds [%d,%d) not inside [0,%d)", j, lo, hi, seq_len);
    if (slots_host[j] < 0) continue;
    if (hi - lo > c.slot_capacity) return pc::fail(ctx, PC_ELEN, "chunk %d: %d tokens exceed the slot capacity %d", j, hi - lo, c.slot_capacity);
    if (slots_host[j] >= c.n_slots) return pc::fail(ctx, PC_ESLOT, "chunk %d: slot %d out of range [0,%d)", j, slots_host[j], c.n_slots);
    for (int i = 0; i < j; ++i)
      if (slots_host[i] == slots_host[j]) return pc::fail(ctx, PC_EINVAL, "slot %d appears twice", slots_host[j]);
  }
  for (int j = 0; j < n; ++j) {
    if (slots_host[j] < 0) continue;
    const int lo = bounds_host[j], cnt = bounds_host[j + 1] - lo;
    pc_status st = pc::launch_kv_store(ctx, layer, slots_host[j], (const __bf16 *)k_dev + (size_t)lo * c.head_dim,
                                       (const __bf16 *)v_dev + (size_t)lo * c.head_dim, cnt, (long)seq_len * c.head_dim,
                                       (hipStream_t)stream);
    if (st != PC_OK) return st;
    ctx->slot_len[(size_t)layer * c.n_slots + slots_host[j]] = cnt;
  }
  return PC_OK;
}

size_t percache_stack_workspace_bytes(const percache_ctx *ctx, int32_t batch, int32_t t_fresh, int32_t max_chunks, int32_t ffn) {
  if (!ctx || batch < 1 || t_fresh < 1 || max_chunks < 0 || ffn < 1) return 0;
  return carve_stack_ws(ctx, nullptr, batch, t_fresh, max_chunks, ffn).total;
}

pc_status percache_stack_reuse(percache_ctx *ctx, const percache_block_weights *layers_host, int32_t n_layers, int32_t ffn,
                               float eps, const void *h_in_dev, int32_t batch, int32_t t_fresh,
                               const int32_t *slot_ids_host, const int32_t *used_len_host, const int32_t *n_chunks_host,
                               int32_t max_chunks, const int32_t *save_bounds_host, const int32_t *save_slots_host,
                               int32_t n_save, void *h_out_dev, void *workspace_dev, size_t workspace_bytes, void *stream) {
  if (!ctx) return PC_EINVAL;
  const percache_config &c = ctx->cfg;
  if (!layers_host || !h_in_dev || !h_out_dev) return pc::fail(ctx, PC_EINVAL, "NULL pointer");
  if (n_layers < 1 || n_layers > c.n_layers) return pc::fail(ctx, PC_ESHAPE, "n_layers %d outside [1,%d]", n_layers, c.n_layers);
  if (ffn < 64 || ffn % 64) return pc::fail(ctx, PC_ESHAPE, "ffn %d must be a positive multiple of 64", ffn);
  if (c.hidden % BF) return pc::fail(ctx, PC_ESHAPE, "hidden %d must be a multiple of %d for the block projections", c.hidden, BF);
  if (!(eps > 0.f)) return pc::fail(ctx, PC_EINVAL, "eps must be positive");
  if (!aligned16(h_in_dev) || !aligned16(h_out_dev)) return pc::fail(ctx, PC_EINVAL, "tensor pointers must be 16-byte aligned");
  if (n_save < 0 || (n_save > 0 && (!save_bounds_host || !save_slots_host))) return pc::fail(ctx, PC_EINVAL, "bad save arguments");
  for (int l = 0; l < n_layers; ++l) {
    const percache_block_weights &w = layers_host[l];
    const void *ptrs[7] = {w.gain1, w.wqkv, w.wo, w.gain2, w.w_gate, w.w_up, w.w_down};
    for (const void *p : ptrs)
      if (!p || !aligned16(p)) return pc::fail(ctx, PC_EINVAL, "layer %d: NULL or misaligned weight pointer", l);
  }
  // chunk tables of every layer (the slot table is per layer): all must agree, so that one upload serves the stack
  std::vector<int32_t> rows, rows_l;
  pc_status st = pc::build_chunk_table(ctx, 0, batch, t_fresh, slot_ids_host, used_len_host, n_chunks_host, max_chunks, rows);
  if (st != PC_OK) return st;
  for (int l = 1; l < n_layers; ++l) {
    st = pc::build_chunk_table(ctx, l, batch, t_fresh, slot_ids_host, used_len_host, n_chunks_host, max_chunks, rows_l);
    if (st != PC_OK) return st;
    if (rows_l != rows) return pc::fail(ctx, PC_ELEN, "the chunks' stored lengths differ between layer 0 and layer %d", l);
  }
  const long M = (long)batch * t_fresh;
  if (M * (long)(ffn > c.hidden ? ffn : c.hidden) >= (1L << 31)) return pc::fail(ctx, PC_ESHAPE, "activation larger than 2^31 elements");
  for (int b = 0; b < batch && n_save > 0; ++b) {
    for (int j = 0; j < n_save; ++j) {
      const int lo = save_bounds_host[j], hi = save_bounds_host[j + 1], slot = save_slots_host[(size_t)b * n_save + j];
      if (lo < 0 || hi > t_fresh || hi <= lo) return pc::fail(ctx, PC_ELEN, "save chunk %d: bounds [%d,%d) not inside [0,%d)", j, lo, hi, t_fresh);
      if (slot < 0) continue;
      if (hi - lo > c.slot_capacity) return pc::fail(ctx, PC_ELEN, "save chunk %d: %d tokens exceed the slot capacity %d", j, hi - lo, c.slot_capacity);
      if (slot >= c.n_slots) return pc::fail(ctx, PC_ESLOT, "save chunk %d: slot %d out of range [0,%d)", j, slot, c.n_slots);
      // a slot being read by this very call must not be overwritten by it
      for (int bb = 0; bb < batch; ++bb)
        for (int ci = 0; ci < n_chunks_host[bb]; ++ci)
          if (slot_ids_host[(size_t)bb * max_chunks + ci] == slot) return pc::fail(ctx, PC_EINVAL, "save slot %d is also read by this call", slot);
      for (int k = 0; k < b * n_save + j; ++k)
        if (save_slots_host[k] == slot) return pc::fail(ctx, PC_EINVAL, "save slot %d appears twice", slot);
    }
  }
  const size_t need = percache_stack_workspace_bytes(ctx, batch, t_fresh, max_chunks, ffn);
  if (!workspace_dev || workspace_bytes < need) return pc::fail(ctx, PC_ENOMEM, "stack workspace has %zu bytes, need %zu", workspace_bytes, need);
  if ((uintptr_t)workspace_dev % pc::kAlign) return pc::fail(ctx, PC_EINVAL, "workspace must be 256-byte aligned");

  StackWs ws = carve_stack_ws(ctx, workspace_dev, batch, t_fresh, max_chunks, ffn);
  const int stride = pc::tbl_stride(max_chunks);
  int min_tiles = INT32_MAX;
  for (int b = 0; b < batch; ++b) {
    int tiles = rows[(size_t)b * stride + 2] + (t_fresh + pc::kKvTile - 1) / pc::kKvTile;
    if (tiles < min_tiles) min_tiles = tiles;
  }
  hipStream_t s = (hipStream_t)stream;
  st = pc::upload_table(ctx, rows, ws.pf.table, s);
  if (st != PC_OK) return st;
  const int H = c.hidden, A = c.n_q_heads * c.head_dim;
  const __bf16 *h_cur = (const __bf16 *)h_in_dev;
  __bf16 *h_out = (__bf16 *)h_out_dev;
  for (int l = 0; l < n_layers; ++l) {
    const percache_block_weights &w = layers_host[l];
#define PC_TRY(call) do { st = (call); if (st != PC_OK) return st; } while (0)
    PC_TRY(launch_rmsnorm(ctx, h_cur, (const __bf16 *)w.gain1, ws.normed, (int)M, H, eps, s));
    PC_TRY(pc::launch_qkv_rope(ctx, ws.normed, (const __bf16 *)w.wqkv, batch, t_fresh, ws.pf.table, stride, ws.pf.q, ws.pf.k, ws.pf.v, s));
    PC_TRY(pc::launch_v_repack(ctx, ws.pf.v, ws.pf.v_blk, batch, t_fresh, s));
    PC_TRY(pc::launch_attention(ctx, l, ws.pf.q, ws.pf.k, ws.pf.v_blk, batch, t_fresh, ws.pf.table, stride, min_tiles, 0, ws.attn,
                                ws.pf.part_o, ws.pf.part_ml, s));
    for (int b = 0; b < batch && n_save > 0; ++b)
      for (int j = 0; j < n_save; ++j) {
        const int slot = save_slots_host[(size_t)b * n_save + j];
        if (slot < 0) continue;
        const int lo = save_bounds_host[j], cnt = save_bounds_host[j + 1] - lo;
        const size_t at = ((size_t)b * c.n_kv_heads * t_fresh + lo) * c.head_dim;
        PC_TRY(pc::launch_kv_store(ctx, l, slot, ws.pf.k + at, ws.pf.v + at, cnt, (long)t_fresh * c.head_dim, s));
        ctx->slot_len[(size_t)l * c.n_slots + slot] = cnt;
      }
    PC_TRY(launch_linear_residual(ctx, ws.attn, (const __bf16 *)w.wo, h_cur, ws.mid, (int)M, H, A, s));
    PC_TRY(launch_rmsnorm(ctx, ws.mid, (const __bf16 *)w.gain2, ws.normed, (int)M, H, eps, s));
    PC_TRY(launch_linear_swiglu(ctx, ws.normed, (const __bf16 *)w.w_gate, (const __bf16 *)w.w_up, ws.act, (int)M, ffn, H, s));
    PC_TRY(launch_linear_residual(ctx, ws.act, (const __bf16 *)w.w_down, ws.mid, h_out, (int)M, H, ffn, s));
#undef PC_TRY
    h_cur = h_out;
  }
  return PC_OK;
}

}  // extern "C"
