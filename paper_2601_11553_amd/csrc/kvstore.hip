// Slot-indexed per-layer K/V store: the device-resident form of the per-chunk tensor files of
// Sec. 4.1.1 (cache slicer output).
//
// Layout per layer and (slot, kv head), chosen for the attention kernel's streams:
//   K: [token][head_dim] bf16                       -- one 64-key tile is a contiguous 16 KB run (D = 128)
//   V: [token / 64][head_dim][64 keys] bf16 blocks  -- the transposed tile the PV product consumes, also one
//      contiguous run; inside each group of 16 keys the order is pc::blocked_key (see percache_internal.hpp);
//      keys past the stored count are zero in the last block.
// percache_kv_put / percache_kv_get convert from / to the caller's dense [kv head][token][head_dim] tensors.
#include "percache_internal.hpp"

namespace {
using pc::kKvTile;

// blockIdx.y == 0: K, Hkv runs of n_tok*D elements copied 16 bytes per lane.
// blockIdx.y == 1: V, one output 16-byte vector (8 key positions of one head-dim index) per thread and step.
struct SlotList {
  int32_t slot[64];
};

template <bool kToStore>
__global__ __launch_bounds__(256) void kv_copy_kernel(pc::u32x4 *__restrict__ slot_k, __bf16 *__restrict__ slot_v,
                                                      pc::u32x4 *__restrict__ dense_k, __bf16 *__restrict__ dense_v,
                                                      int n_heads, int n_tok, int D, int C, SlotList slots,
                                                      long slot_stride_elems, long dense_head_stride) {
  // blockIdx.z selects the chunk: its slot and its dense tensor.  dense_head_stride: elements between the heads of
  // a dense tensor (n_tok * D when the chunk is a tensor of its own, more when it is a token range of a longer one)
  if (slots.slot[blockIdx.z] < 0) return;  // (an entry of the other slot format: the other launch copies it)
  {
    const long so = (long)slots.slot[blockIdx.z] * slot_stride_elems;
    const long dn = (long)blockIdx.z * n_heads * dense_head_stride;
    slot_k += so / 8;
    slot_v += so;
    dense_k += dn / 8;
    dense_v += dn;
  }
  const long stride = (long)gridDim.x * blockDim.x;
  const long tid0 = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (blockIdx.y == 0) {
    const int run_vec = n_tok * D / 8, slot_head_vec = C * D / 8;
    const long total = (long)n_heads * run_vec;
    for (long e = tid0; e < total; e += stride) {
      int g = (int)(e / run_vec);
      int r = (int)(e - (long)g * run_vec);
      long s = (long)g * slot_head_vec + r;
      long dd = (long)g * (dense_head_stride / 8) + r;
      if (kToStore) slot_k[s] = dense_k[dd]; else dense_k[dd] = slot_k[s];
    }
    return;
  }
  const int n_tiles = (n_tok + kKvTile - 1) / kKvTile;
  if (kToStore) {
    // vector id -> (head, tile, chunk of 8 positions, head-dim index); d fastest so dense reads coalesce
    const long total = (long)n_heads * n_tiles * 8 * D;
    for (long e = tid0; e < total; e += stride) {
      int d = (int)(e % D);
      long r = e / D;
      int chunk = (int)(r & 7);
      r >>= 3;
      int tile = (int)(r % n_tiles);
      int g = (int)(r / n_tiles);
      pc::bf16x8 o;
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        int pos = chunk * 8 + k;
        int t = tile * kKvTile + (pos & ~15) + pc::blocked_key(pos & 15);
        o[k] = t < n_tok ? dense_v[(size_t)g * dense_head_stride + (size_t)t * D + d] : (__bf16)0.f;
      }
      *(pc::bf16x8 *)(slot_v + (((size_t)g * C + (size_t)tile * kKvTile) * D) + (size_t)d * kKvTile + chunk * 8) = o;
    }
  } else {
    // vector id -> (head, token, 8 head-dim indices)
    const int dv = D / 8;
    const long total = (long)n_heads * n_tok * dv;
    for (long e = tid0; e < total; e += stride) {
      int dc = (int)(e % dv);
      long r = e / dv;
      int t = (int)(r % n_tok);
      int g = (int)(r / n_tok);
      int tile = t / kKvTile, tin = t - tile * kKvTile;
      int pos = (tin & ~15) + pc::blocked_key(tin & 15);
      const __bf16 *src = slot_v + (((size_t)g * C + (size_t)tile * kKvTile) * D) + pos;
      pc::bf16x8 o;
#pragma unroll
      for (int k = 0; k < 8; ++k) o[k] = src[(size_t)(dc * 8 + k) * kKvTile];
      *(pc::bf16x8 *)(dense_v + (size_t)g * dense_head_stride + (size_t)t * D + dc * 8) = o;
    }
  }
}

// Appends n_new tokens behind the `off` tokens a slot already holds.  K: rows copied to their place.  V: every
// position of the 64-key blocks that receive a token is rewritten from `off` on -- the new tokens, then zeros, so
// that the padding of the last block stays finite (masked probabilities multiply it).
__global__ __launch_bounds__(256) void kv_append_kernel(__bf16 *__restrict__ slot_k, __bf16 *__restrict__ slot_v,
                                                        const __bf16 *__restrict__ k_new, const __bf16 *__restrict__ v_new,
                                                        int n_heads, int off, int n_new, int D, int C, long new_head_stride) {
  const int tile0 = off / kKvTile, n_tiles = (off + n_new + kKvTile - 1) / kKvTile - tile0;
  const long stride = (long)gridDim.x * blockDim.x;
  const long tid0 = (long)blockIdx.x * blockDim.x + threadIdx.x;
  const long total_k = (long)n_heads * n_new * D;
  for (long e = tid0; e < total_k; e += stride) {
    const int dd = (int)(e % D);
    const long r = e / D;
    const int t = (int)(r % n_new), g = (int)(r / n_new);
    slot_k[((size_t)g * C + off + t) * D + dd] = k_new[(size_t)g * new_head_stride + (size_t)t * D + dd];
  }
  const long total_v = (long)n_heads * n_tiles * D * kKvTile;
  for (long e = tid0; e < total_v; e += stride) {
    const int p = (int)(e % kKvTile);  // physical position inside the block
    long r = e / kKvTile;
    const int dd = (int)(r % D);
    r /= D;
    const int tile = tile0 + (int)(r % n_tiles), g = (int)(r / n_tiles);
    const int t_abs = tile * kKvTile + (p & ~15) + pc::blocked_key(p & 15);
    if (t_abs < off) continue;  // older tokens stay
    const int t = t_abs - off;
    const __bf16 val = t < n_new ? v_new[(size_t)g * new_head_stride + (size_t)t * D + dd] : (__bf16)0.f;
    slot_v[((size_t)g * C + (size_t)tile * kKvTile) * D + (size_t)dd * kKvTile + p] = val;
  }
}

// ---------------------------------------------------------------------------------------------------
// 8-bit slots.  Layout per (slot, kv head):  K [token][head_dim] bytes;  V [token / 64][head_dim][64] bytes with
// key order pc::blocked_key8 inside a block, zero codes past the stored count;  one scale 2^e per 64-token block
// for K and one for V.  One workgroup per (chunk, kv head, 64-token block).
// ---------------------------------------------------------------------------------------------------
// 2^e with e the smallest integer such that amax <= 448 * 2^e, e kept in [-110, 127] (0 for amax == 0).
// 448 = 1.75 * 2^8: with amax = 1.f * 2^k the answer is k - 8 when 1.f <= 1.75, else k - 7.
__device__ __forceinline__ int block_exponent(float amax) {
  if (amax == 0.f) return 0;
  const unsigned bits = __float_as_uint(amax);
  const int field = (int)((bits >> 23) & 0xff);
  if (field == 0) return -110;  // below 2^-126
  const int k = field - 127;
  const int e = (bits & 0x7fffffu) <= 0x600000u ? k - 8 : k - 7;
  return e < -110 ? -110 : (e > 127 ? 127 : e);
}
__device__ __forceinline__ float pow2f(int e) { return __uint_as_float((unsigned)(e + 127) << 23); }  // e in [-126, 127]

// four E4M3 codes of four floats already divided by the scale (round to nearest even in hardware; |y| <= 448)
__device__ __forceinline__ unsigned encode4(float a, float b, float c, float d) {
  int w = __builtin_amdgcn_cvt_pk_fp8_f32(__builtin_amdgcn_fmed3f(a, -448.f, 448.f), __builtin_amdgcn_fmed3f(b, -448.f, 448.f), 0, false);
  w = __builtin_amdgcn_cvt_pk_fp8_f32(__builtin_amdgcn_fmed3f(c, -448.f, 448.f), __builtin_amdgcn_fmed3f(d, -448.f, 448.f), w, true);
  return (unsigned)w;
}

// off > 0: the slot already holds `off` tokens and the dense tensors are the tokens that follow them (append).  The
// block that was partly filled is then quantised afresh from the values its old tokens read back as plus the new
// tokens (its exponent is recomputed over all of them; old codes are re-rounded only if the exponent moves); the
// launch covers the blocks from off / 64 on, and n_tok counts old and new tokens together.
template <int D>
__global__ __launch_bounds__(256) void kv_quant_kernel(uint8_t *__restrict__ slot_k, uint8_t *__restrict__ slot_v,
                                                       float *__restrict__ scale_k, float *__restrict__ scale_v,
                                                       const __bf16 *__restrict__ dense_k, const __bf16 *__restrict__ dense_v,
                                                       int n_heads, int n_tok, int C, SlotList slots, long slot_stride_elems,
                                                       long scale_slot_stride, long dense_head_stride, int off) {
  constexpr int DV = D / 8, NV = kKvTile * DV / 256;  // 8-element vectors per row; vectors per thread
  __shared__ float red[2][4];
  __shared__ __align__(16) uint8_t vt[kKvTile][D + 16];  // V codes [key][d] (padded rows), read back transposed
  const int blk = blockIdx.x + off / kKvTile, g = blockIdx.y, tid = threadIdx.x;
  const int slot = slots.slot[blockIdx.z];
  if (slot < 0) return;  // (a bf16 slot: the other launch copies it; the whole workgroup leaves)
  const size_t dense_at = ((size_t)blockIdx.z * n_heads + g) * dense_head_stride;
  const size_t slot_at = (size_t)slot * slot_stride_elems + (size_t)g * C * D;
  const size_t sc = (size_t)slot * scale_slot_stride + (size_t)g * (C / kKvTile) + blk;
  const bool has_old = blk * kKvTile < off;  // (only the first block of an append)
  const float old_sk = has_old ? scale_k[sc] : 1.f, old_sv = has_old ? scale_v[sc] : 1.f;
  pc::bf16x8 kv[NV], vv[NV];
  float ak = 0.f, av = 0.f;
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    const int v = tid + 256 * j, r = v / DV, dc = v - r * DV;
    const int t = blk * kKvTile + r;
    if (t < off) {
      // what the stored codes read back as (exact in bf16)
      typedef float f32x2 __attribute__((ext_vector_type(2)));
      const uint2 ck = *(const uint2 *)(slot_k + slot_at + (size_t)t * D + dc * 8);
      const uint8_t *vcol = slot_v + slot_at + (size_t)blk * kKvTile * D + pc::blocked_pos8(r);
      unsigned wk[2] = {ck.x, ck.y}, wv[2] = {0, 0};
#pragma unroll
      for (int e = 0; e < 8; ++e) wv[e >> 2] |= (unsigned)vcol[(size_t)(dc * 8 + e) * kKvTile] << (8 * (e & 3));
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const f32x2 k0 = __builtin_amdgcn_cvt_pk_f32_fp8((int)wk[h], false), k1 = __builtin_amdgcn_cvt_pk_f32_fp8((int)wk[h], true);
        const f32x2 v0 = __builtin_amdgcn_cvt_pk_f32_fp8((int)wv[h], false), v1 = __builtin_amdgcn_cvt_pk_f32_fp8((int)wv[h], true);
        kv[j][4 * h + 0] = (__bf16)(k0[0] * old_sk); kv[j][4 * h + 1] = (__bf16)(k0[1] * old_sk);
        kv[j][4 * h + 2] = (__bf16)(k1[0] * old_sk); kv[j][4 * h + 3] = (__bf16)(k1[1] * old_sk);
        vv[j][4 * h + 0] = (__bf16)(v0[0] * old_sv); vv[j][4 * h + 1] = (__bf16)(v0[1] * old_sv);
        vv[j][4 * h + 2] = (__bf16)(v1[0] * old_sv); vv[j][4 * h + 3] = (__bf16)(v1[1] * old_sv);
      }
    } else if (t < n_tok) {
      kv[j] = *(const pc::bf16x8 *)(dense_k + dense_at + (size_t)(t - off) * D + dc * 8);
      vv[j] = *(const pc::bf16x8 *)(dense_v + dense_at + (size_t)(t - off) * D + dc * 8);
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) { kv[j][e] = (__bf16)0.f; vv[j][e] = (__bf16)0.f; }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      ak = fmaxf(ak, fabsf((float)kv[j][e]));
      av = fmaxf(av, fabsf((float)vv[j][e]));
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    ak = fmaxf(ak, __shfl_xor(ak, o, 64));
    av = fmaxf(av, __shfl_xor(av, o, 64));
  }
  if ((tid & 63) == 0) { red[0][tid >> 6] = ak; red[1][tid >> 6] = av; }
  __syncthreads();
  ak = fmaxf(fmaxf(red[0][0], red[0][1]), fmaxf(red[0][2], red[0][3]));
  av = fmaxf(fmaxf(red[1][0], red[1][1]), fmaxf(red[1][2], red[1][3]));
  const int ek = block_exponent(ak), ev = block_exponent(av);
  const float ik = pow2f(-ek), iv = pow2f(-ev);
  if (tid == 0) {
    scale_k[sc] = pow2f(ek);
    scale_v[sc] = pow2f(ev);
  }
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    const int v = tid + 256 * j, r = v / DV, dc = v - r * DV;
    const int t = blk * kKvTile + r;
    uint2 ck, cv;
    ck.x = encode4((float)kv[j][0] * ik, (float)kv[j][1] * ik, (float)kv[j][2] * ik, (float)kv[j][3] * ik);
    ck.y = encode4((float)kv[j][4] * ik, (float)kv[j][5] * ik, (float)kv[j][6] * ik, (float)kv[j][7] * ik);
    cv.x = encode4((float)vv[j][0] * iv, (float)vv[j][1] * iv, (float)vv[j][2] * iv, (float)vv[j][3] * iv);
    cv.y = encode4((float)vv[j][4] * iv, (float)vv[j][5] * iv, (float)vv[j][6] * iv, (float)vv[j][7] * iv);
    if (t < n_tok) *(uint2 *)(slot_k + slot_at + (size_t)t * D + dc * 8) = ck;
    *(uint2 *)(&vt[r][dc * 8]) = cv;  // rows past the stored count hold zero codes
  }
  __syncthreads();
  // transposed write: one 16-byte run of a head-dim row per thread and step
  uint8_t *vblk = slot_v + slot_at + (size_t)blk * kKvTile * D;
  for (int o = tid; o < D * (kKvTile / 16); o += 256) {
    const int d = o / (kKvTile / 16), c16 = o - d * (kKvTile / 16);
    unsigned w[4] = {0, 0, 0, 0};
#pragma unroll
    for (int p = 0; p < 16; ++p) w[p >> 2] |= (unsigned)vt[pc::blocked_key8(c16 * 16 + p)][d] << (8 * (p & 3));
    *(uint4 *)(vblk + (size_t)d * kKvTile + c16 * 16) = make_uint4(w[0], w[1], w[2], w[3]);
  }
}

// The values an 8-bit slot holds, as dense bf16 [kv head][token][head_dim]: code * 2^e (exact).
template <int D>
__global__ __launch_bounds__(256) void kv_dequant_kernel(const uint8_t *__restrict__ slot_k, const uint8_t *__restrict__ slot_v,
                                                         const float *__restrict__ scale_k, const float *__restrict__ scale_v,
                                                         __bf16 *__restrict__ dense_k, __bf16 *__restrict__ dense_v, int n_heads,
                                                         int n_tok, int C, SlotList slots, long slot_stride_elems,
                                                         long scale_slot_stride, long dense_head_stride, int /*unused*/) {
  constexpr int DV = D / 8, NV = kKvTile * DV / 256;
  const int blk = blockIdx.x, g = blockIdx.y, tid = threadIdx.x;
  const int slot = slots.slot[blockIdx.z];
  if (slot < 0) return;
  const size_t dense_at = ((size_t)blockIdx.z * n_heads + g) * dense_head_stride;
  const size_t slot_at = (size_t)slot * slot_stride_elems + (size_t)g * C * D;
  const size_t sc = (size_t)slot * scale_slot_stride + (size_t)g * (C / kKvTile) + blk;
  const float sk = scale_k[sc], sv = scale_v[sc];
  const uint8_t *vblk = slot_v + slot_at + (size_t)blk * kKvTile * D;
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    const int v = tid + 256 * j, r = v / DV, dc = v - r * DV;
    const int t = blk * kKvTile + r;
    if (t >= n_tok) continue;
    const uint2 ck = *(const uint2 *)(slot_k + slot_at + (size_t)t * D + dc * 8);
    const int pos = pc::blocked_pos8(r);
    unsigned cvx = 0, cvy = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      cvx |= (unsigned)vblk[(size_t)(dc * 8 + e) * kKvTile + pos] << (8 * e);
      cvy |= (unsigned)vblk[(size_t)(dc * 8 + 4 + e) * kKvTile + pos] << (8 * e);
    }
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    pc::bf16x8 ok, ov;
    const unsigned wk[2] = {ck.x, ck.y}, wv[2] = {cvx, cvy};
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const f32x2 k0 = __builtin_amdgcn_cvt_pk_f32_fp8((int)wk[h], false), k1 = __builtin_amdgcn_cvt_pk_f32_fp8((int)wk[h], true);
      const f32x2 v0 = __builtin_amdgcn_cvt_pk_f32_fp8((int)wv[h], false), v1 = __builtin_amdgcn_cvt_pk_f32_fp8((int)wv[h], true);
      ok[4 * h + 0] = (__bf16)(k0[0] * sk); ok[4 * h + 1] = (__bf16)(k0[1] * sk);
      ok[4 * h + 2] = (__bf16)(k1[0] * sk); ok[4 * h + 3] = (__bf16)(k1[1] * sk);
      ov[4 * h + 0] = (__bf16)(v0[0] * sv); ov[4 * h + 1] = (__bf16)(v0[1] * sv);
      ov[4 * h + 2] = (__bf16)(v1[0] * sv); ov[4 * h + 3] = (__bf16)(v1[1] * sv);
    }
    *(pc::bf16x8 *)(dense_k + dense_at + (size_t)t * D + dc * 8) = ok;
    *(pc::bf16x8 *)(dense_v + dense_at + (size_t)t * D + dc * 8) = ov;
  }
}

pc_status check_slot(percache_ctx *ctx, int32_t layer, int32_t slot) {
  if (!ctx) return PC_EINVAL;
  if (layer < 0 || layer >= ctx->cfg.n_layers) return pc::fail(ctx, PC_ESLOT, "layer %d out of range [0,%d)", layer, ctx->cfg.n_layers);
  if (slot < 0 || slot >= ctx->cfg.n_slots) return pc::fail(ctx, PC_ESLOT, "slot %d out of range [0,%d)", slot, ctx->cfg.n_slots);
  return PC_OK;
}

// Copies between dense tensors and the slots of a list (at most 64 entries; entry i <-> dense block i).  A list may
// name slots of both formats: each format gets its own launch, in which the entries of the other format are marked -1.
template <bool kToStore>
pc_status launch_copy(percache_ctx *ctx, int layer, const int32_t *slot_list, int n, void *k_dev, void *v_dev, int n_tokens,
                      hipStream_t stream, long dense_head_stride = 0) {
  const percache_config &c = ctx->cfg;
  SlotList sl16, sl8;
  int n16 = 0, n8 = 0;
  for (int i = 0; i < 64; ++i) {
    sl16.slot[i] = sl8.slot[i] = -1;
    if (i >= n) continue;
    if (ctx->is8(slot_list[i])) { sl8.slot[i] = slot_list[i] - ctx->n_slots16; ++n8; }
    else { sl16.slot[i] = slot_list[i]; ++n16; }
  }
  const long dhs = dense_head_stride ? dense_head_stride : (long)n_tokens * c.head_dim;
  if (n8) {
    const size_t off = (size_t)layer * ctx->layer_stride8;
    const long sc_slot = (long)c.n_kv_heads * (c.slot_capacity / kKvTile);
    const size_t sc_off = (size_t)layer * ctx->n_slots8 * sc_slot;
    dim3 grid((n_tokens + kKvTile - 1) / kKvTile, c.n_kv_heads, n);
#define PC_KV8(KERNEL, DD)                                                                                                    \
  hipLaunchKernelGGL((KERNEL<DD>), grid, dim3(256), 0, stream, ctx->k8_store + off, ctx->v8_store + off, ctx->k_scale + sc_off, \
                     ctx->v_scale + sc_off, (__bf16 *)k_dev, (__bf16 *)v_dev, c.n_kv_heads, n_tokens, c.slot_capacity, sl8,     \
                     (long)ctx->slot_stride, sc_slot, dhs, 0)
    if (kToStore) {
      if (c.head_dim == 128) PC_KV8(kv_quant_kernel, 128); else PC_KV8(kv_quant_kernel, 64);
    } else {
      if (c.head_dim == 128) PC_KV8(kv_dequant_kernel, 128); else PC_KV8(kv_dequant_kernel, 64);
    }
#undef PC_KV8
    PC_HIP(ctx, hipGetLastError());
  }
  if (n16) {
    const size_t off = (size_t)layer * ctx->layer_stride;
    long total = (long)c.n_kv_heads * ((n_tokens + kKvTile - 1) / kKvTile) * kKvTile * c.head_dim / 8;
    int blocks = (int)((total + 255) / 256);
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(kv_copy_kernel<kToStore>, dim3(blocks, 2, n), dim3(256), 0, stream, (pc::u32x4 *)(ctx->k_store + off),
                       ctx->v_store + off, (pc::u32x4 *)k_dev, (__bf16 *)v_dev, c.n_kv_heads, n_tokens, c.head_dim,
                       c.slot_capacity, sl16, (long)ctx->slot_stride, dhs);
    PC_HIP(ctx, hipGetLastError());
  }
  return PC_OK;
}

}  // namespace

namespace pc {
pc_status launch_kv_store(percache_ctx *ctx, int layer, int slot, const __bf16 *k, const __bf16 *v, int n_tokens,
                          long dense_head_stride, hipStream_t stream) {
  return launch_copy<true>(ctx, layer, &slot, 1, (void *)k, (void *)v, n_tokens, stream, dense_head_stride);
}
pc_status launch_kv_append(percache_ctx *ctx, int layer, int slot, const __bf16 *k, const __bf16 *v, int off, int n_tokens,
                           long new_head_stride, hipStream_t stream) {
  const percache_config &c = ctx->cfg;
  if (ctx->is8(slot)) {
    const long sc_slot = (long)c.n_kv_heads * (c.slot_capacity / kKvTile);
    const size_t lo = (size_t)layer * ctx->layer_stride8, sc_off = (size_t)layer * ctx->n_slots8 * sc_slot;
    SlotList sl;
    for (int i = 0; i < 64; ++i) sl.slot[i] = i == 0 ? slot - ctx->n_slots16 : -1;
    const int total = off + n_tokens;
    dim3 grid((total + kKvTile - 1) / kKvTile - off / kKvTile, c.n_kv_heads, 1);
    if (c.head_dim == 128)
      hipLaunchKernelGGL((kv_quant_kernel<128>), grid, dim3(256), 0, stream, ctx->k8_store + lo, ctx->v8_store + lo,
                         ctx->k_scale + sc_off, ctx->v_scale + sc_off, k, v, c.n_kv_heads, total, c.slot_capacity, sl,
                         (long)ctx->slot_stride, sc_slot, new_head_stride, off);
    else
      hipLaunchKernelGGL((kv_quant_kernel<64>), grid, dim3(256), 0, stream, ctx->k8_store + lo, ctx->v8_store + lo,
                         ctx->k_scale + sc_off, ctx->v_scale + sc_off, k, v, c.n_kv_heads, total, c.slot_capacity, sl,
                         (long)ctx->slot_stride, sc_slot, new_head_stride, off);
    PC_HIP(ctx, hipGetLastError());
    return PC_OK;
  }
  const size_t at = (size_t)layer * ctx->layer_stride + (size_t)slot * ctx->slot_stride;
  const long work = (long)c.n_kv_heads * c.head_dim * ((n_tokens + kKvTile - 1) / kKvTile + 1) * kKvTile;
  int blocks = (int)((work + 255) / 256);
  if (blocks > 1024) blocks = 1024;
  hipLaunchKernelGGL(kv_append_kernel, dim3(blocks), dim3(256), 0, stream, ctx->k_store + at, ctx->v_store + at, k, v,
                     c.n_kv_heads, off, n_tokens, c.head_dim, c.slot_capacity, new_head_stride);
  PC_HIP(ctx, hipGetLastError());
  return PC_OK;
}
}  // namespace pc

extern "C" {

pc_status percache_kv_append(percache_ctx *ctx, int32_t layer, int32_t slot, const void *k_dev, const void *v_dev,
                             int32_t n_tokens, void *stream) {
  pc_status st = check_slot(ctx, layer, slot);
  if (st != PC_OK) return st;
  if (!k_dev || !v_dev) return pc::fail(ctx, PC_EINVAL, "k_dev / v_dev is NULL");
  if (((uintptr_t)k_dev | (uintptr_t)v_dev) % 16) return pc::fail(ctx, PC_EINVAL, "k_dev / v_dev must be 16-byte aligned");
  const percache_config &c = ctx->cfg;
  const int have = ctx->slot_len[(size_t)layer * c.n_slots + slot];
  if (n_tokens < 1 || have + n_tokens > c.slot_capacity)
    return pc::fail(ctx, PC_ELEN, "slot %d holds %d tokens: %d more do not fit the capacity %d", slot, have, n_tokens, c.slot_capacity);
  st = pc::launch_kv_append(ctx, layer, slot, (const __bf16 *)k_dev, (const __bf16 *)v_dev, have, n_tokens,
                            (long)n_tokens * c.head_dim, (hipStream_t)stream);
  if (st != PC_OK) return st;
  ctx->slot_len[(size_t)layer * c.n_slots + slot] = have + n_tokens;
  return PC_OK;
}

pc_status percache_kv_put(percache_ctx *ctx, int32_t layer, int32_t slot, const void *k_dev, const void *v_dev,
                          int32_t n_tokens, void *stream) {
  pc_status st = check_slot(ctx, layer, slot);
  if (st != PC_OK) return st;
  if (!k_dev || !v_dev) return pc::fail(ctx, PC_EINVAL, "k_dev / v_dev is NULL");
  if (((uintptr_t)k_dev | (uintptr_t)v_dev) % 16) return pc::fail(ctx, PC_EINVAL, "k_dev / v_dev must be 16-byte aligned");
  const percache_config &c = ctx->cfg;
  if (n_tokens < 1 || n_tokens > c.slot_capacity) return pc::fail(ctx, PC_ELEN, "n_tokens %d outside [1,%d]", n_tokens, c.slot_capacity);
  st = launch_copy<true>(ctx, layer, &slot, 1, (void *)k_dev, (void *)v_dev, n_tokens, (hipStream_t)stream);
  if (st != PC_OK) return st;
  ctx->slot_len[(size_t)layer * c.n_slots + slot] = n_tokens;
  return PC_OK;
}

pc_status percache_kv_put_batch(percache_ctx *ctx, int32_t layer, const int32_t *slots_host, int32_t n, const void *k_dev,
                                const void *v_dev, int32_t n_tokens, void *stream) {
  if (!ctx) return PC_EINVAL;
  if (!slots_host || n < 1) return pc::fail(ctx, PC_EINVAL, "slots_host is NULL or n < 1");
  if (!k_dev || !v_dev) return pc::fail(ctx, PC_EINVAL, "k_dev / v_dev is NULL");
  if (((uintptr_t)k_dev | (uintptr_t)v_dev) % 16) return pc::fail(ctx, PC_EINVAL, "k_dev / v_dev must be 16-byte aligned");
  const percache_config &c = ctx->cfg;
  if (n_tokens < 1 || n_tokens > c.slot_capacity) return pc::fail(ctx, PC_ELEN, "n_tokens %d outside [1,%d]", n_tokens, c.slot_capacity);
  for (int i = 0; i < n; ++i) {
    pc_status st = check_slot(ctx, layer, slots_host[i]);
    if (st != PC_OK) return st;
    for (int j = 0; j < i; ++j)
      if (slots_host[j] == slots_host[i]) return pc::fail(ctx, PC_EINVAL, "slot %d appears twice in the batch", slots_host[i]);
  }
  const size_t per_chunk = (size_t)c.n_kv_heads * n_tokens * c.head_dim;
  for (int i0 = 0; i0 < n; i0 += 64) {
    int cnt = n - i0 < 64 ? n - i0 : 64;
    pc_status st = launch_copy<true>(ctx, layer, slots_host + i0, cnt, (void *)((const __bf16 *)k_dev + per_chunk * i0),
                                     (void *)((const __bf16 *)v_dev + per_chunk * i0), n_tokens, (hipStream_t)stream);
    if (st != PC_OK) return st;
  }
  for (int i = 0; i < n; ++i) ctx->slot_len[(size_t)layer * c.n_slots + slots_host[i]] = n_tokens;
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
  st = launch_copy<false>(ctx, layer, &slot, 1, k_out_dev, v_out_dev, n_tokens, (hipStream_t)stream);
  if (st != PC_OK) return st;
  if (n_tokens_out_host) *n_tokens_out_host = n_tokens;
  return PC_OK;
}

pc_status percache_kv_get_batch(percache_ctx *ctx, int32_t layer, const int32_t *slots_host, int32_t n, void *k_out_dev,
                                void *v_out_dev, int32_t n_tokens, void *stream) {
  if (!ctx) return PC_EINVAL;
  if (!slots_host || n < 1) return pc::fail(ctx, PC_EINVAL, "slots_host is NULL or n < 1");
  if (!k_out_dev || !v_out_dev) return pc::fail(ctx, PC_EINVAL, "k_out_dev / v_out_dev is NULL");
  if (((uintptr_t)k_out_dev | (uintptr_t)v_out_dev) % 16) return pc::fail(ctx, PC_EINVAL, "outputs must be 16-byte aligned");
  const percache_config &c = ctx->cfg;
  if (n_tokens < 1 || n_tokens > c.slot_capacity) return pc::fail(ctx, PC_ELEN, "n_tokens %d outside [1,%d]", n_tokens, c.slot_capacity);
  for (int i = 0; i < n; ++i) {
    pc_status st = check_slot(ctx, layer, slots_host[i]);
    if (st != PC_OK) return st;
    const int have = ctx->slot_len[(size_t)layer * c.n_slots + slots_host[i]];
    if (have <= 0) return pc::fail(ctx, PC_ESLOT, "slot %d of layer %d is empty", slots_host[i], layer);
    if (have < n_tokens) return pc::fail(ctx, PC_ELEN, "slot %d holds %d tokens, %d asked for", slots_host[i], have, n_tokens);
  }
  const size_t per_chunk = (size_t)c.n_kv_heads * n_tokens * c.head_dim;
  for (int i0 = 0; i0 < n; i0 += 64) {
    const int cnt = n - i0 < 64 ? n - i0 : 64;
    pc_status st = launch_copy<false>(ctx, layer, slots_host + i0, cnt, (void *)((__bf16 *)k_out_dev + per_chunk * i0),
                                      (void *)((__bf16 *)v_out_dev + per_chunk * i0), n_tokens, (hipStream_t)stream);
    if (st != PC_OK) return st;
  }
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
