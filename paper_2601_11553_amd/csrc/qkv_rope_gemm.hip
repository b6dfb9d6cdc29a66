// Fresh-token Q/K/V projection with the RoPE of App. B.1 fused into the epilogue.
//
// Only the retained suffix of each query is projected (Sec. 4.2.2): Y = X W^T, X [M = B*T_f, H] bf16,
// W [(Hq+2Hkv)*D, H] bf16, fp32 accumulation on the bf16 matrix cores.  The position of fresh token i of
// query b is L_pre[b] + i: the position counter is advanced by the cached length before the sine/cosine
// table is read.  q and k are rotated on the fp32 accumulators and rounded to bf16 once.
//
// Tiling: the shared projection main loop (gemm_tile.hpp): a workgroup of 4 wavefronts computes 128 output
// features x (64 or 128) tokens, and each wavefront owns a feature block together with its rotation partner
// (m, m + D/2), so RoPE needs no cross-lane traffic.
#include "gemm_tile.hpp"

namespace {
using pc::f32x16;
using pc::gemm::BF;
using pc::gemm::pack4;

// NTB: 32-token blocks per wavefront (1 -> 64-token tile, 2 -> 128-token tile, 3 -> 192-token tile: 80 KB of LDS,
// still two workgroups per CU).
// EXTRA: the bias / head-norm variants (see QkvExtras) are compiled in.
// WIDE: 8 wavefronts on two heads (256 features) x the same token tile, one workgroup per CU (D = 128, no EXTRA).
template <int D, int NTB, bool EXTRA, bool WIDE = false>
__global__ __launch_bounds__(WIDE ? 512 : 256, WIDE ? 1 : 2) void qkv_rope_kernel(const __bf16 *__restrict__ X, const __bf16 *__restrict__ W, int M,
                                                          int H, int t_fresh, int Hq, int Hkv,
                                                          const int32_t *__restrict__ table, int tbl_stride,
                                                          const float2 *__restrict__ rope, __bf16 *__restrict__ Q,
                                                          __bf16 *__restrict__ K, __bf16 *__restrict__ V, pc::QkvExtras ex,
                                                          __bf16 *__restrict__ V_blk) {
  constexpr int BT = 64 * NTB;
  extern __shared__ __align__(16) char lds[];  // Shape<NTB>::LDS_BYTES

  static_assert(!WIDE || (D == 128 && !EXTRA), "the wide tile is built for head size 128 without the variants");
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wf = wave & 1, wt = (wave >> 1) & 1, half = wave >> 2;  // (half: which of the tile's two heads; 0 unless WIDE)
  const int l32 = lane & 31, g = lane >> 5;
  int bx = blockIdx.x, by = blockIdx.y;
  if constexpr (WIDE) {
    // One tile per CU: give each XCD (workgroup ids go round-robin over the 8) a compact patch of the tile grid, so
    // that the weight and token rows its tiles share are fetched into its L2 once.  Ids of one XCD become consecutive
    // positions, and positions walk strips of `sw` feature tiles, token tile by token tile.
    const int nx = gridDim.x, ny = gridDim.y, total = nx * ny;
    const int id = blockIdx.y * nx + blockIdx.x, xcd = id & 7;
    const int pos = xcd * (total >> 3) + min(xcd, total & 7) + (id >> 3);
    const int sw = nx % 5 == 0 ? 5 : nx % 4 == 0 ? 4 : nx % 3 == 0 ? 3 : nx % 2 == 0 ? 2 : 1;
    const int strip = pos / (sw * ny), within = pos - strip * (sw * ny);
    by = within / sw;
    bx = strip * sw + (within - by * sw);
  }
  const int f0 = bx * (WIDE ? 2 * BF : BF);  // first feature of the tile
  const int m0 = by * BT;                     // first token row of the tile

  // feature blocks (of 32) this wavefront owns: the low half of a rotation pair and its partner
  const int fb_lo = (D == 128) ? 4 * half + wf : 2 * wf;
  const int fb_hi = (D == 128) ? 4 * half + wf + 2 : 2 * wf + 1;

  f32x16 acc[2][NTB];
  if constexpr (WIDE)
    pc::gemm::mainloop_wide<NTB>(lds, [&](int row) __attribute__((always_inline)) { return W + (size_t)(f0 + row) * H; }, X, H, m0, M, H, fb_lo, fb_hi, wt, acc);
  else
    pc::gemm::mainloop<NTB>(lds, [&](int row) __attribute__((always_inline)) { return W + (size_t)(f0 + row) * H; }, X, H, m0, M, H, fb_lo, fb_hi, acc);

  // ---- epilogue: RoPE at position L_pre[b] + i on fp32, one rounding to bf16, head-major stores
  const int head = WIDE ? 2 * bx + half : (D == 128) ? bx : 2 * bx + wf;
  const int m_base = (D == 128) ? wf * 32 : 0;  // index of the low element inside the head
  __bf16 *dst;
  int hh, n_heads;
  bool rotate = true;
  if (head < Hq) { dst = Q; hh = head; n_heads = Hq; }
  else if (head < Hq + Hkv) { dst = K; hh = head - Hq; n_heads = Hkv; }
  else { dst = V; hh = head - Hq - Hkv; n_heads = Hkv; rotate = false; }
  if constexpr (EXTRA) {
    // bias on the accumulators; then, for q and k heads, RMSNorm over the head dimension: a token's head is spread over
    // the two lanes (l, l+32) and, at D = 128, over the wavefront pair (wf = 0, 1), which meet through LDS
    if (ex.bias) {
      const __bf16 *bl = ex.bias + (size_t)head * D + m_base + g * 4;
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float b_lo = (float)bl[q4 * 8 + e], b_hi = (float)bl[q4 * 8 + e + D / 2];
#pragma unroll
          for (int t = 0; t < NTB; ++t) { acc[0][t][q4 * 4 + e] += b_lo; acc[1][t][q4 * 4 + e] += b_hi; }
        }
    }
    const __bf16 *gain = head < Hq ? ex.q_norm : (head < Hq + Hkv ? ex.k_norm : nullptr);
    float ss[NTB];
#pragma unroll
    for (int t = 0; t < NTB; ++t) {
      ss[t] = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) ss[t] += acc[0][t][r] * acc[0][t][r] + acc[1][t][r] * acc[1][t][r];
      ss[t] += __shfl_xor(ss[t], 32, 64);
    }
    if (D == 128) {
      float *red = (float *)lds;  // [wt][NTB][32 tokens][wf]; the main loop is done with LDS (it ends in a barrier)
#pragma unroll
      for (int t = 0; t < NTB; ++t)
        if (g == 0) red[((wt * NTB + t) * 32 + l32) * 2 + wf] = ss[t];
      __syncthreads();
#pragma unroll
      for (int t = 0; t < NTB; ++t) ss[t] = red[((wt * NTB + t) * 32 + l32) * 2] + red[((wt * NTB + t) * 32 + l32) * 2 + 1];
    }
    if (gain) {
      const __bf16 *gl = gain + m_base + g * 4;
#pragma unroll
      for (int t = 0; t < NTB; ++t) {
        const float r = 1.0f / sqrtf(ss[t] / (float)D + ex.eps);
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            acc[0][t][q4 * 4 + e] *= r * (float)gl[q4 * 8 + e];
            acc[1][t][q4 * 4 + e] *= r * (float)gl[q4 * 8 + e + D / 2];
          }
      }
    }
  }
#pragma unroll
  for (int t = 0; t < NTB; ++t) {
    const int m_raw = m0 + (wt * NTB + t) * 32 + l32;
    const bool m_ok = m_raw < M;
    const int m = m_ok ? m_raw : M - 1;
    const int b = m / t_fresh, i = m - b * t_fresh;
    const int pos = table[(size_t)b * tbl_stride + 1] + i;
    __bf16 *row = dst + (((size_t)b * n_heads + hh) * t_fresh + i) * D;
    // all sixteen (cos, sin) pairs of this lane's token first (eight 16-byte loads in flight), then the math
    float4 cs[4][2];
    if (rotate) {
      const float4 *csp = (const float4 *)(rope + (size_t)pos * (D / 2) + m_base + g * 4);
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        cs[q4][0] = csp[q4 * 4];      // pairs mm, mm+1
        cs[q4][1] = csp[q4 * 4 + 1];  // pairs mm+2, mm+3
      }
    }
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const int mm = m_base + q4 * 8 + g * 4;  // first of 4 consecutive pair indices
      float lo[4], hi[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float a = acc[0][t][q4 * 4 + e], c = acc[1][t][q4 * 4 + e];
        if (rotate) {
          const float4 w4 = cs[q4][e >> 1];
          const float wc = (e & 1) ? w4.z : w4.x, ws = (e & 1) ? w4.w : w4.y;
          lo[e] = a * wc - c * ws;
          hi[e] = c * wc + a * ws;
        } else {
          lo[e] = a;
          hi[e] = c;
        }
      }
      if (m_ok) {
        *(uint2 *)(row + mm) = pack4(lo[0], lo[1], lo[2], lo[3]);
        *(uint2 *)(row + mm + D / 2) = pack4(hi[0], hi[1], hi[2], hi[3]);
        if (V_blk && !rotate) {
          // also as the 64-key blocks [D][64] the attention kernel reads for the fresh part (t_fresh is a multiple of
          // 64 here: no padding to write); the 32 lanes of a half wavefront hold 32 consecutive tokens of one feature
          const int tin = i & 63;
          __bf16 *vb = V_blk + ((((size_t)b * n_heads + hh) * (t_fresh >> 6) + (i >> 6)) * D) * 64 + (tin & ~15) + pc::blocked_key(tin & 15);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            vb[(size_t)(mm + e) * 64] = (__bf16)lo[e];
            vb[(size_t)(mm + e + D / 2) * 64] = (__bf16)hi[e];
          }
        }
      }
    }
  }
}

// Few token rows (one or two 128-token tiles) without the bias / head-norm variants: one pass, no slices.  A workgroup
// owns 32 weight rows = 16 rotation pairs of one head (rows j and j + 16 of the tile are features m and m + D/2), which a
// lane finds in its accumulators r and r + 8, and all token rows of its tile (gemm_tile.hpp: mainloop_skinny).
template <int D>
__global__ __launch_bounds__(256, 2) void qkv_rope_skinny_kernel(const __bf16 *__restrict__ X, const __bf16 *__restrict__ W,
                                                                 int M, int H, int t_fresh, int Hq, int Hkv,
                                                                 const int32_t *__restrict__ table, int tbl_stride,
                                                                 const float2 *__restrict__ rope, __bf16 *__restrict__ Q,
                                                                 __bf16 *__restrict__ K, __bf16 *__restrict__ V,
                                                                 __bf16 *__restrict__ V_blk) {
  constexpr int NS = 5, TPH = D / 32;  // stages; tiles per head
  __shared__ __align__(16) char lds[NS * pc::gemm::Skinny::STAGE];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l32 = lane & 31, g = lane >> 5;
  const int head = blockIdx.x / TPH, sub = blockIdx.x % TPH;
  const int m0 = blockIdx.y * 128;
  f32x16 acc;
  pc::gemm::mainloop_skinny<NS>(
      lds,
      [&](int row) __attribute__((always_inline)) {
        return W + (size_t)(head * D + (row < 16 ? 0 : D / 2 - 16) + sub * 16 + row) * H;
      },
      X, H, m0, M, H, acc);
  __bf16 *dst;
  int hh, n_heads;
  bool rotate = true;
  if (head < Hq) { dst = Q; hh = head; n_heads = Hq; }
  else if (head < Hq + Hkv) { dst = K; hh = head - Hq; n_heads = Hkv; }
  else { dst = V; hh = head - Hq - Hkv; n_heads = Hkv; rotate = false; }
  const int m_raw = m0 + wave * 32 + l32;
  if (m_raw >= M) return;
  const int b = m_raw / t_fresh, i = m_raw - b * t_fresh;
  const int pos = table[(size_t)b * tbl_stride + 1] + i;
  __bf16 *row = dst + (((size_t)b * n_heads + hh) * t_fresh + i) * D;
#pragma unroll
  for (int q2 = 0; q2 < 2; ++q2) {
    const int mm = sub * 16 + q2 * 8 + g * 4;  // first of this lane's 4 consecutive pair indices
    float lo[4], hi[4];
    float4 cs[2];
    if (rotate) {
      const float4 *csp = (const float4 *)(rope + (size_t)pos * (D / 2) + mm);
      cs[0] = csp[0];
      cs[1] = csp[1];
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float a = acc[q2 * 4 + e], c = acc[8 + q2 * 4 + e];
      if (rotate) {
        const float4 w4 = cs[e >> 1];
        const float wc = (e & 1) ? w4.z : w4.x, ws = (e & 1) ? w4.w : w4.y;
        lo[e] = a * wc - c * ws;
        hi[e] = c * wc + a * ws;
      } else {
        lo[e] = a;
        hi[e] = c;
      }
    }
    *(uint2 *)(row + mm) = pack4(lo[0], lo[1], lo[2], lo[3]);
    *(uint2 *)(row + mm + D / 2) = pack4(hi[0], hi[1], hi[2], hi[3]);
    if (V_blk && !rotate) {
      // the 64-key blocks [D][64] the attention kernel reads for the fresh part (t_fresh is a multiple of 64 here:
      // no padding to write), saving the repack launch
      const int tin = i & 63;
      __bf16 *vb = V_blk + ((((size_t)b * n_heads + hh) * (t_fresh >> 6) + (i >> 6)) * D) * 64 + (tin & ~15) + pc::blocked_key(tin & 15);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        vb[(size_t)(mm + e) * 64] = (__bf16)lo[e];
        vb[(size_t)(mm + e + D / 2) * 64] = (__bf16)hi[e];
      }
    }
  }
}

// Epilogue of the split-k path (few token rows): adds the fp32 slices P[s][m][f] in a fixed order, rotates q and k
// exactly as above, rounds once.  One thread per (token, head, 4 consecutive rotation pairs).
template <int D>
__global__ __launch_bounds__(256) void reduce_rope_kernel(const float *__restrict__ P, int n_k, int M, int F, int t_fresh, int Hq,
                                                          int Hkv, const int32_t *__restrict__ table, int tbl_stride,
                                                          const float2 *__restrict__ rope, __bf16 *__restrict__ Q,
                                                          __bf16 *__restrict__ K, __bf16 *__restrict__ V, pc::QkvExtras ex,
                                                          __bf16 *__restrict__ V_blk) {
  constexpr int QUADS = D / 8;
  const long gid = (long)blockIdx.x * blockDim.x + threadIdx.x;
  const int n_heads_all = Hq + 2 * Hkv;
  if (gid >= (long)M * n_heads_all * QUADS) return;
  const int j = (int)(gid % QUADS);
  const long r = gid / QUADS;
  const int head = (int)(r % n_heads_all), m = (int)(r / n_heads_all);
  const int mm = 4 * j;
  const size_t slice = (size_t)M * F, at = (size_t)m * F + (size_t)head * D + mm;
  float4 lo = *(const float4 *)(P + at), hi = *(const float4 *)(P + at + D / 2);
#pragma unroll 4
  for (int s = 1; s < n_k; ++s) {
    const float4 a = *(const float4 *)(P + s * slice + at), c = *(const float4 *)(P + s * slice + at + D / 2);
    lo.x += a.x; lo.y += a.y; lo.z += a.z; lo.w += a.w;
    hi.x += c.x; hi.y += c.y; hi.z += c.z; hi.w += c.w;
  }
  const int b = m / t_fresh, i = m - b * t_fresh;
  __bf16 *dst;
  int hh, n_heads;
  bool rotate = true;
  if (head < Hq) { dst = Q; hh = head; n_heads = Hq; }
  else if (head < Hq + Hkv) { dst = K; hh = head - Hq; n_heads = Hkv; }
  else { dst = V; hh = head - Hq - Hkv; n_heads = Hkv; rotate = false; }
  float l4[4] = {lo.x, lo.y, lo.z, lo.w}, h4[4] = {hi.x, hi.y, hi.z, hi.w};
  if (ex.bias) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      l4[e] += (float)ex.bias[(size_t)head * D + mm + e];
      h4[e] += (float)ex.bias[(size_t)head * D + mm + e + D / 2];
    }
  }
  const __bf16 *gain = head < Hq ? ex.q_norm : (head < Hq + Hkv ? ex.k_norm : nullptr);
  if (ex.q_norm || ex.k_norm) {  // uniform: the QUADS consecutive threads of a (token, head) reduce together
    float ss = 0.f;
#pragma unroll
    for (int e = 0; e < 4; ++e) ss += l4[e] * l4[e] + h4[e] * h4[e];
#pragma unroll
    for (int o = 1; o < QUADS; o <<= 1) ss += __shfl_xor(ss, o, 64);
    if (gain) {
      const float rr = 1.0f / sqrtf(ss / (float)D + ex.eps);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        l4[e] *= rr * (float)gain[mm + e];
        h4[e] *= rr * (float)gain[mm + e + D / 2];
      }
    }
  }
  if (rotate) {
    const int pos = table[(size_t)b * tbl_stride + 1] + i;
    const float4 *csp = (const float4 *)(rope + (size_t)pos * (D / 2) + mm);
    const float4 c01 = csp[0], c23 = csp[1];  // (cos, sin) of pairs mm, mm+1 and mm+2, mm+3
    const float wc[4] = {c01.x, c01.z, c23.x, c23.z}, wsn[4] = {c01.y, c01.w, c23.y, c23.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float a = l4[e], c = h4[e];
      l4[e] = a * wc[e] - c * wsn[e];
      h4[e] = c * wc[e] + a * wsn[e];
    }
  }
  __bf16 *row = dst + (((size_t)b * n_heads + hh) * t_fresh + i) * D;
  *(uint2 *)(row + mm) = pack4(l4[0], l4[1], l4[2], l4[3]);
  *(uint2 *)(row + mm + D / 2) = pack4(h4[0], h4[1], h4[2], h4[3]);
  if (V_blk && !rotate) {  // also as the 64-key blocks [D][64] of the attention kernel (t_fresh is a multiple of 64 here)
    const int tin = i & 63;
    __bf16 *vb = V_blk + ((((size_t)b * n_heads + hh) * (t_fresh >> 6) + (i >> 6)) * D) * 64 + (tin & ~15) + pc::blocked_key(tin & 15);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      vb[(size_t)(mm + e) * 64] = (__bf16)l4[e];
      vb[(size_t)(mm + e + D / 2) * 64] = (__bf16)h4[e];
    }
  }
}

}  // namespace

namespace pc {

pc_status launch_qkv_rope(percache_ctx *ctx, const __bf16 *x, const __bf16 *w, int batch, int t_fresh,
                          const int32_t *table_dev, int tbl_stride, __bf16 *q, __bf16 *k, __bf16 *v,
                          hipStream_t stream, float *gemm_part, const QkvExtras &extras, __bf16 *v_blk, bool *v_blk_done) {
  if (v_blk_done) *v_blk_done = false;
  const percache_config &c = ctx->cfg;
  const int M = batch * t_fresh;
  const int F = (c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim;
  if (F % BF) return fail(ctx, PC_ESHAPE, "(Hq + 2 Hkv) * D = %d must be a multiple of %d", F, BF);
  if ((long)F * c.hidden >= (1L << 31) || (long)M * c.hidden >= (1L << 31))
    return fail(ctx, PC_ESHAPE, "operand larger than 2^31 elements");
  const float2 *rope = (const float2 *)ctx->rope;
  if (gemm_part && splitk_applies(M) && M > 64 && !extras.any()) {
    // one or two 128-token tiles: weight-stream bound; one pass with 32 weight rows per workgroup (with at most 64
    // rows the slices below are faster: they do not pay for a 128-token tile)
    dim3 sgrid(F / 32, (M + 127) / 128);
    __bf16 *vb = (v_blk && v_blk_done && t_fresh % 64 == 0) ? v_blk : nullptr;  // also lay V out for the attention kernel
    if (vb) *v_blk_done = true;
    prof_begin(ctx, PC_KERNEL_QKV_ROPE, stream);
    if (c.head_dim == 128)
      hipLaunchKernelGGL(qkv_rope_skinny_kernel<128>, sgrid, dim3(256), 0, stream, x, w, M, c.hidden, t_fresh, c.n_q_heads,
                         c.n_kv_heads, table_dev, tbl_stride, rope, q, k, v, vb);
    else
      hipLaunchKernelGGL(qkv_rope_skinny_kernel<64>, sgrid, dim3(256), 0, stream, x, w, M, c.hidden, t_fresh, c.n_q_heads,
                         c.n_kv_heads, table_dev, tbl_stride, rope, q, k, v, vb);
    prof_end(ctx, PC_KERNEL_QKV_ROPE, stream);
    PC_HIP(ctx, hipGetLastError());
    return PC_OK;
  }
  if (gemm_part && splitk_applies(M)) {
    // few token rows with the bias / head-norm variants: contraction cut into slices (see block.hip)
    const int nk = choose_split_k(ctx->n_cu, F / BF * (M > 128 ? 2 : 1), c.hidden / pc::gemm::BK);
    prof_begin(ctx, PC_KERNEL_QKV_ROPE, stream);
    pc_status st = launch_splitk_partial(ctx, x, c.hidden, w, w, F, c.hidden, gemm_part, M, F, c.hidden, nk, stream);
    if (st != PC_OK) return st;
    const long threads = (long)M * (c.n_q_heads + 2 * c.n_kv_heads) * (c.head_dim / 8);
    const dim3 rgrid((unsigned)((threads + 255) / 256));
    __bf16 *vb = (v_blk && v_blk_done && t_fresh % 64 == 0) ? v_blk : nullptr;  // also lay V out for the attention kernel
    if (vb) *v_blk_done = true;
    if (c.head_dim == 128)
      hipLaunchKernelGGL(reduce_rope_kernel<128>, rgrid, dim3(256), 0, stream, gemm_part, nk, M, F, t_fresh, c.n_q_heads,
                         c.n_kv_heads, table_dev, tbl_stride, rope, q, k, v, extras, vb);
    else
      hipLaunchKernelGGL(reduce_rope_kernel<64>, rgrid, dim3(256), 0, stream, gemm_part, nk, M, F, t_fresh, c.n_q_heads,
                         c.n_kv_heads, table_dev, tbl_stride, rope, q, k, v, extras, vb);
    prof_end(ctx, PC_KERNEL_QKV_ROPE, stream);
    PC_HIP(ctx, hipGetLastError());
    return PC_OK;
  }
  // Token tile: two workgroups share a CU, so a launch runs in rounds of 2 * n_cu tiles and a tile's time grows with
  // its token blocks; take the width with the fewest block-rounds (the wider one on a tie: fewer operand reads per
  // MFMA).  64-token tiles while there are too few rows to fill wider ones.
  int ntb = 1;
  if (M > 64 * 3) {
    long best = -1;
    for (int cand = 3; cand >= 2; --cand) {
      const long tiles = (long)(F / BF) * ((M + 64 * cand - 1) / (64 * cand));
      const long cost = (tiles + 2L * ctx->n_cu - 1) / (2L * ctx->n_cu) * cand;
      if (best < 0 || cost < best) { best = cost; ntb = cand; }
    }
  }
  // Two heads per workgroup (8 wavefronts, one workgroup per CU) when all its tiles fit one round: the token rows
  // are brought into LDS once for twice the features.
  const int n_heads_all = c.n_q_heads + 2 * c.n_kv_heads;
  __bf16 *vb_large = (v_blk && v_blk_done && t_fresh % 64 == 0) ? v_blk : nullptr;  // the large tiles lay V out for the attention kernel too
  if (vb_large) *v_blk_done = true;
  if (c.head_dim == 128 && !extras.any() && n_heads_all % 2 == 0 && M >= 1024 &&
      (long)(n_heads_all / 2) * ((M + 191) / 192) <= ctx->n_cu) {
    constexpr int lds_bytes = pc::gemm::WideShape<3>::LDS_BYTES;
    PC_HIP(ctx, hipFuncSetAttribute((const void *)qkv_rope_kernel<128, 3, false, true>, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes));
    prof_begin(ctx, PC_KERNEL_QKV_ROPE, stream);
    hipLaunchKernelGGL((qkv_rope_kernel<128, 3, false, true>), dim3(n_heads_all / 2, (M + 191) / 192), dim3(512), lds_bytes, stream, x, w, M,
                       c.hidden, t_fresh, c.n_q_heads, c.n_kv_heads, table_dev, tbl_stride, rope, q, k, v, extras, vb_large);
    prof_end(ctx, PC_KERNEL_QKV_ROPE, stream);
    PC_HIP(ctx, hipGetLastError());
    return PC_OK;
  }
  dim3 grid(F / BF, (M + 64 * ntb - 1) / (64 * ntb));
#define PC_LAUNCH_E(DD, NN, EE)                                                                                        \
  do {                                                                                                                \
    constexpr int lds_bytes = pc::gemm::Shape<NN>::LDS_BYTES;                                                         \
    if (lds_bytes > 64 * 1024) /* above the default limit: opt in */                                                  \
      PC_HIP(ctx, hipFuncSetAttribute((const void *)qkv_rope_kernel<DD, NN, EE>, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes)); \
    hipLaunchKernelGGL((qkv_rope_kernel<DD, NN, EE>), grid, dim3(256), lds_bytes, stream, x, w, M, c.hidden, t_fresh,  \
                       c.n_q_heads, c.n_kv_heads, table_dev, tbl_stride, rope, q, k, v, extras, vb_large);            \
  } while (0)
#define PC_LAUNCH(DD, NN)                                                                                             \
  do {                                                                                                                \
    if (extras.any()) PC_LAUNCH_E(DD, NN, true); else PC_LAUNCH_E(DD, NN, false);                                      \
  } while (0)
  prof_begin(ctx, PC_KERNEL_QKV_ROPE, stream);
  if (c.head_dim == 128) {
    if (ntb == 3) PC_LAUNCH(128, 3); else if (ntb == 2) PC_LAUNCH(128, 2); else PC_LAUNCH(128, 1);
  } else {
    if (ntb == 3) PC_LAUNCH(64, 3); else if (ntb == 2) PC_LAUNCH(64, 2); else PC_LAUNCH(64, 1);
  }
#undef PC_LAUNCH
#undef PC_LAUNCH_E
  prof_end(ctx, PC_KERNEL_QKV_ROPE, stream);
  PC_HIP(ctx, hipGetLastError());
  return PC_OK;
}

}  // namespace pc
