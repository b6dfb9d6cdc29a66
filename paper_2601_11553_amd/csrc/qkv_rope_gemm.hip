// Fresh-token Q/K/V projection with the RoPE of App. B.1 fused into the epilogue.
//
// Only the retained suffix of each query is projected (Sec. 4.2.2): Y = X W^T, X [M = B*T_f, H] bf16,
// W [(Hq+2Hkv)*D, H] bf16, fp32 accumulation on the bf16 matrix cores.  The position of fresh token i of
// query b is L_pre[b] + i: the position counter is advanced by the cached length before the sine/cosine
// table is read.  q and k are rotated on the fp32 accumulators and rounded to bf16 once.
//
// Tiling (64-wide wavefronts, 32x32x16 MFMA): a workgroup of 4 wavefronts computes 128 output features
// x (64 or 128) tokens.  The features are the M side of the MFMA and the tokens the N side, so a lane ends
// up holding 4 consecutive features of one token per accumulator quad (8-byte stores), and each wavefront
// owns a feature block together with its rotation partner (m, m + D/2): RoPE needs no cross-lane traffic.
#include "percache_internal.hpp"

namespace {
using pc::bf16x8;
using pc::f32x16;

constexpr int BK = 64;               // k elements per LDS stage
constexpr int LDS_ROW = BK * 2 + 16; // bytes per padded LDS row (conflict-free 16-byte reads)
constexpr int BF = 128;              // features per workgroup

__device__ __forceinline__ uint2 pack4(float a, float b, float c, float d) {
  pc::bf16x4 v = {(__bf16)a, (__bf16)b, (__bf16)c, (__bf16)d};
  return __builtin_bit_cast(uint2, v);
}

// NTB: 32-token blocks per wavefront (1 -> 64-token tile, 2 -> 128-token tile).
template <int D, int NTB>
__global__ __launch_bounds__(256) void qkv_rope_kernel(const __bf16 *__restrict__ X, const __bf16 *__restrict__ W, int M,
                                                       int H, int t_fresh, int Hq, int Hkv,
                                                       const int32_t *__restrict__ table, int tbl_stride,
                                                       const float2 *__restrict__ rope, __bf16 *__restrict__ Q,
                                                       __bf16 *__restrict__ K, __bf16 *__restrict__ V) {
  constexpr int BT = 64 * NTB;
  __shared__ __align__(16) char lds_w[2][BF * LDS_ROW];
  __shared__ __align__(16) char lds_x[2][BT * LDS_ROW];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wf = wave & 1, wt = wave >> 1;
  const int l32 = lane & 31, g = lane >> 5;
  const int f0 = blockIdx.x * BF;  // first feature of the tile
  const int m0 = blockIdx.y * BT;  // first token row of the tile

  // feature blocks (of 32) this wavefront owns: the low half of a rotation pair and its partner
  const int fb_lo = (D == 128) ? wf : 2 * wf;
  const int fb_hi = (D == 128) ? wf + 2 : 2 * wf + 1;

  // global -> LDS mapping: 8 threads per 128-byte row segment
  const int ld_row = tid >> 3, ld_col = tid & 7;
  pc::u32x4 rw[BF / 32], rx[BT / 32];
  auto load_global = [&](int kt) __attribute__((always_inline)) {
#pragma unroll
    for (int p = 0; p < BF / 32; ++p) {
      int row = f0 + ld_row + 32 * p;
      rw[p] = *(const pc::u32x4 *)(W + (size_t)row * H + kt * BK + ld_col * 8);
    }
#pragma unroll
    for (int p = 0; p < BT / 32; ++p) {
      int row = min(m0 + ld_row + 32 * p, M - 1);
      rx[p] = *(const pc::u32x4 *)(X + (size_t)row * H + kt * BK + ld_col * 8);
    }
  };
  auto store_lds = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
    for (int p = 0; p < BF / 32; ++p) *(pc::u32x4 *)(lds_w[buf] + (ld_row + 32 * p) * LDS_ROW + ld_col * 16) = rw[p];
#pragma unroll
    for (int p = 0; p < BT / 32; ++p) *(pc::u32x4 *)(lds_x[buf] + (ld_row + 32 * p) * LDS_ROW + ld_col * 16) = rx[p];
  };

  f32x16 acc[2][NTB];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int t = 0; t < NTB; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][t][r] = 0.f;

  const int nk = H / BK;
  load_global(0);
  store_lds(0);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < nk) load_global(kt + 1);
    const char *wl = lds_w[buf] + (fb_lo * 32 + l32) * LDS_ROW + g * 16;
    const char *wh = lds_w[buf] + (fb_hi * 32 + l32) * LDS_ROW + g * 16;
    const char *xb = lds_x[buf] + ((wt * NTB) * 32 + l32) * LDS_ROW + g * 16;
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 a_lo = *(const bf16x8 *)(wl + ks * 32);
      bf16x8 a_hi = *(const bf16x8 *)(wh + ks * 32);
#pragma unroll
      for (int t = 0; t < NTB; ++t) {
        bf16x8 b = *(const bf16x8 *)(xb + t * 32 * LDS_ROW + ks * 32);
        acc[0][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_lo, b, acc[0][t], 0, 0, 0);
        acc[1][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_hi, b, acc[1][t], 0, 0, 0);
      }
    }
    if (kt + 1 < nk) store_lds(buf ^ 1);
    __syncthreads();
  }

  // ---- epilogue: RoPE at position L_pre[b] + i on fp32, one rounding to bf16, head-major stores
  const int head = (D == 128) ? blockIdx.x : 2 * blockIdx.x + wf;
  const int m_base = (D == 128) ? wf * 32 : 0;  // index of the low element inside the head
  __bf16 *dst;
  int hh, n_heads;
  bool rotate = true;
  if (head < Hq) { dst = Q; hh = head; n_heads = Hq; }
  else if (head < Hq + Hkv) { dst = K; hh = head - Hq; n_heads = Hkv; }
  else { dst = V; hh = head - Hq - Hkv; n_heads = Hkv; rotate = false; }
#pragma unroll
  for (int t = 0; t < NTB; ++t) {
    const int m_raw = m0 + (wt * NTB + t) * 32 + l32;
    const bool m_ok = m_raw < M;
    const int m = m_ok ? m_raw : M - 1;
    const int b = m / t_fresh, i = m - b * t_fresh;
    const int pos = table[(size_t)b * tbl_stride + 1] + i;
    __bf16 *row = dst + (((size_t)b * n_heads + hh) * t_fresh + i) * D;
    const float2 *cs = rope + (size_t)pos * (D / 2);
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const int mm = m_base + q4 * 8 + g * 4;  // first of 4 consecutive pair indices
      float lo[4], hi[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float a = acc[0][t][q4 * 4 + e], c = acc[1][t][q4 * 4 + e];
        if (rotate) {
          float2 w = cs[mm + e];
          lo[e] = a * w.x - c * w.y;
          hi[e] = c * w.x + a * w.y;
        } else {
          lo[e] = a;
          hi[e] = c;
        }
      }
      if (m_ok) {
        *(uint2 *)(row + mm) = pack4(lo[0], lo[1], lo[2], lo[3]);
        *(uint2 *)(row + mm + D / 2) = pack4(hi[0], hi[1], hi[2], hi[3]);
      }
    }
  }
}

}  // namespace

namespace pc {

pc_status launch_qkv_rope(percache_ctx *ctx, const __bf16 *x, const __bf16 *w, int batch, int t_fresh,
                          const int32_t *table_dev, int tbl_stride, __bf16 *q, __bf16 *k, __bf16 *v,
                          hipStream_t stream) {
  const percache_config &c = ctx->cfg;
  const int M = batch * t_fresh;
  const int F = (c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim;
  if (F % BF) return fail(ctx, PC_ESHAPE, "(Hq + 2 Hkv) * D = %d must be a multiple of %d", F, BF);
  const float2 *rope = (const float2 *)ctx->rope;
  const bool big = M > 64 * 3;  // 128-token tiles once there are enough rows to fill them
  dim3 grid(F / BF, big ? (M + 127) / 128 : (M + 63) / 64);
#define PC_LAUNCH(DD, NN)                                                                                          \
  hipLaunchKernelGGL((qkv_rope_kernel<DD, NN>), grid, dim3(256), 0, stream, x, w, M, c.hidden, t_fresh, c.n_q_heads, \
                     c.n_kv_heads, table_dev, tbl_stride, rope, q, k, v)
  prof_begin(ctx, PC_KERNEL_QKV_ROPE, stream);
  if (c.head_dim == 128) {
    if (big) PC_LAUNCH(128, 2); else PC_LAUNCH(128, 1);
  } else {
    if (big) PC_LAUNCH(64, 2); else PC_LAUNCH(64, 1);
  }
#undef PC_LAUNCH
  prof_end(ctx, PC_KERNEL_QKV_ROPE, stream);
  PC_HIP(ctx, hipGetLastError());
  return PC_OK;
}

}  // namespace pc
