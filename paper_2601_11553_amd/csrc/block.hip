// The rest of a pre-norm transformer block around the cache-reusing attention module, on the retained (fresh)
// rows only, so that a stack of layers can be chained (App. B.1: after the attention module the computation
// goes on as in an ordinary block; the cached rows' activations are never needed again because the next layer
// crops them once more):
//   h' = h + (attention(RMSNorm(h) ...)) Wo^T,   h'' = h' + (silu(n Wgate^T) * (n Wup^T)) Wdown^T,  n = RMSNorm(h').
// Kernels: a row-wise RMSNorm, and the shared projection main loop with two epilogues (residual add; SwiGLU on a
// gate/up feature pair held by the same lane); for few token rows, where the weight stream bounds a projection,
// slices of the contraction + small reduce kernels (few features, long contraction) or a one-pass kernel with 32
// weight rows per workgroup (many features).  percache_stack_reuse chains the layers; percache_kv_slice is the
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
  pc::gemm::mainloop<NTB>(lds, [&](int row) __attribute__((always_inline)) { return W + (size_t)(f0 + row) * K; }, A, K, m0, M,
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
      lds, [&](int row) __attribute__((always_inline)) { return (row < 64 ? Wg : Wu) + (size_t)(f0 + (row & 63)) * K; }, A, K, m0, M, K,
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

// ---------------------------------------------------------------------------------------------------
// Few token rows (one or two token tiles): the projections are bound by the stream of the weights, and N/128
// workgroups cannot pull it.  The contraction is therefore cut into n_k slices computed by separate workgroups:
//   P[s][m][n] = sum over k in slice s of A[m][k] W[n][k]     (fp32, [n_k][M][N])
// and a small second kernel adds the slices in a fixed order (deterministic) and applies the epilogue.
// The weight rows may come from two matrices (rows >= n_split from W1): gate and up projections in one launch.
// ---------------------------------------------------------------------------------------------------
template <int NTB, int NS>
__global__ __launch_bounds__(256, 2) void splitk_partial_kernel(const __bf16 *__restrict__ A, int lda,
                                                                const __bf16 *__restrict__ W0, const __bf16 *__restrict__ W1,
                                                                int n_split, int ldw, float *__restrict__ P, int M, int N,
                                                                int k_slice) {
  constexpr int BT = 64 * NTB;
  __shared__ __align__(16) char lds[NS * pc::gemm::Shape<NTB>::STAGE];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wf = wave & 1, wt = wave >> 1;
  const int l32 = lane & 31, g = lane >> 5;
  const int f0 = blockIdx.x * BF, m0 = blockIdx.z * BT;
  const int k0 = blockIdx.y * k_slice;
  f32x16 acc[2][NTB];
  pc::gemm::mainloop_deep<NTB, true, NS>(  // one token tile: every weight row is read by exactly one workgroup
      lds,
      [&](int row) __attribute__((always_inline)) {
        const int n = f0 + row;
        return (n < n_split ? W0 + (size_t)n * ldw : W1 + (size_t)(n - n_split) * ldw) + k0;
      },
      A + k0, lda, m0, M, k_slice, 2 * wf, 2 * wf + 1, acc);
  float *Ps = P + (size_t)blockIdx.y * M * N;
#pragma unroll
  for (int t = 0; t < NTB; ++t) {
    const int m_raw = m0 + (wt * NTB + t) * 32 + l32;
    const bool ok = m_raw < M;
    const int m = ok ? m_raw : M - 1;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const float4 v = {acc[a][t][q4 * 4 + 0], acc[a][t][q4 * 4 + 1], acc[a][t][q4 * 4 + 2], acc[a][t][q4 * 4 + 3]};
        if (ok) *(float4 *)(Ps + (size_t)m * N + f0 + (2 * wf + a) * 32 + q4 * 8 + g * 4) = v;
      }
  }
}

// One or two 128-token tiles and many features (the gate / up projections): one pass, no slices.  A workgroup owns 16
// gate rows and the 16 up rows of the same features (tile rows j and j + 16), which a lane finds in its accumulators
// r and r + 8, and all token rows of its tile (gemm_tile.hpp: mainloop_skinny).
__global__ __launch_bounds__(256, 2) void swiglu_skinny_kernel(const __bf16 *__restrict__ A, const __bf16 *__restrict__ Wg,
                                                               const __bf16 *__restrict__ Wu, __bf16 *__restrict__ Y, int M,
                                                               int F, int K) {
  constexpr int NS = 5;
  __shared__ __align__(16) char lds[NS * pc::gemm::Skinny::STAGE];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l32 = lane & 31, g = lane >> 5;
  const int f0 = blockIdx.x * 16, m0 = blockIdx.y * 128;
  f32x16 acc;
  pc::gemm::mainloop_skinny<NS>(
      lds, [&](int row) __attribute__((always_inline)) { return (row < 16 ? Wg : Wu) + (size_t)(f0 + (row & 15)) * K; }, A, K, m0, M, K,
      acc);
  const int m = m0 + wave * 32 + l32;
  if (m >= M) return;
#pragma unroll
  for (int q2 = 0; q2 < 2; ++q2) {
    float o[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float gate = acc[q2 * 4 + e], up = acc[8 + q2 * 4 + e];
      o[e] = gate / (1.0f + __expf(-gate)) * up;
    }
    *(uint2 *)(Y + (size_t)m * F + f0 + q2 * 8 + g * 4) = pack4(o[0], o[1], o[2], o[3]);
  }
}

// y = sum of slices + residual (rounded to bf16), and optionally n = RMSNorm(y) * gain on the rounded values.
// One workgroup per row, four columns per thread and pass.
__global__ __launch_bounds__(256) void reduce_residual_norm_kernel(const float *__restrict__ P, int n_k, int M, int N,
                                                                   const __bf16 *__restrict__ R, __bf16 *__restrict__ Y,
                                                                   const __bf16 *__restrict__ gain, __bf16 *__restrict__ Yn,
                                                                   float eps) {
  __shared__ float red[4];
  const int row = blockIdx.x, tid = threadIdx.x;
  const size_t slice = (size_t)M * N;
  float ss = 0.f;
  for (int c = tid * 4; c < N; c += 1024) {
    const size_t at = (size_t)row * N + c;
    float4 sum = *(const float4 *)(P + at);
#pragma unroll 4
    for (int s = 1; s < n_k; ++s) {
      const float4 v = *(const float4 *)(P + s * slice + at);
      sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
    }
    float res[4];
    unpack4(*(const uint2 *)(R + at), res);
    const uint2 packed = pack4(sum.x + res[0], sum.y + res[1], sum.z + res[2], sum.w + res[3]);
    *(uint2 *)(Y + at) = packed;
    float y[4];
    unpack4(packed, y);
    ss += y[0] * y[0] + y[1] * y[1] + y[2] * y[2] + y[3] * y[3];
  }
  if (!gain) return;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
  if ((tid & 63) == 0) red[tid >> 6] = ss;
  __syncthreads();
  const float r = 1.0f / sqrtf((red[0] + red[1] + red[2] + red[3]) / (float)N + eps);
  for (int c = tid * 4; c < N; c += 1024) {
    const size_t at = (size_t)row * N + c;
    float y[4], gq[4];
    unpack4(*(const uint2 *)(Y + at), y);  // this thread's own stores
    unpack4(*(const uint2 *)(gain + c), gq);
    *(uint2 *)(Yn + at) = pack4(y[0] * r * gq[0], y[1] * r * gq[1], y[2] * r * gq[2], y[3] * r * gq[3]);
  }
}

// act[m][f] = silu(sum of gate slices) * (sum of up slices); slices are [n_k][M][2F] with the up half at column F.
__global__ __launch_bounds__(256) void reduce_swiglu_kernel(const float *__restrict__ P, int n_k, int M, int F,
                                                            __bf16 *__restrict__ Y) {
  const long gid = (long)blockIdx.x * blockDim.x + threadIdx.x;
  const int per_row = F / 4;
  if (gid >= (long)M * per_row) return;
  const int m = (int)(gid / per_row), f = (int)(gid - (long)m * per_row) * 4;
  const size_t slice = (size_t)M * 2 * F, at = (size_t)m * 2 * F + f;
  float4 gt = *(const float4 *)(P + at), up = *(const float4 *)(P + at + F);
#pragma unroll 4
  for (int s = 1; s < n_k; ++s) {
    const float4 a = *(const float4 *)(P + s * slice + at), b = *(const float4 *)(P + s * slice + at + F);
    gt.x += a.x; gt.y += a.y; gt.z += a.z; gt.w += a.w;
    up.x += b.x; up.y += b.y; up.z += b.z; up.w += b.w;
  }
  *(uint2 *)(Y + (size_t)m * F + f) = pack4(gt.x / (1.0f + __expf(-gt.x)) * up.x, gt.y / (1.0f + __expf(-gt.y)) * up.y,
                                            gt.z / (1.0f + __expf(-gt.z)) * up.z, gt.w / (1.0f + __expf(-gt.w)) * up.w);
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

pc_status launch_reduce_residual_norm(percache_ctx *ctx, const float *part, int n_k, int M, int N, const __bf16 *res, __bf16 *y,
                                      const __bf16 *gain, __bf16 *yn, float eps, hipStream_t s) {
  hipLaunchKernelGGL(reduce_residual_norm_kernel, dim3(M), dim3(256), 0, s, part, n_k, M, N, res, y, gain, yn, eps);
  PC_HIP(ctx, hipGetLastError());
  return PC_OK;
}
pc_status launch_reduce_swiglu(percache_ctx *ctx, const float *part, int n_k, int M, int F, __bf16 *y, hipStream_t s) {
  const long threads = (long)M * (F / 4);
  hipLaunchKernelGGL(reduce_swiglu_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s, part, n_k, M, F, y);
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
  float *part;     // split-k slices of the block projections (few token rows only)
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
  const size_t widest = (size_t)(2 * ffn > c.hidden ? 2 * ffn : c.hidden);
  w.part = (float *)take(pc::splitk_applies((int)M) ? (size_t)pc::kMaxSplitK * M * widest * sizeof(float) : 0);
  w.total = off;
  return w;
}

}  // namespace

namespace pc {

// Largest number of slices that divides the k steps, leaves every workgroup at least two of them and keeps the
// launch within one workgroup per CU (more slices only add fp32 partials to write and read back).
int choose_split_k(int n_cu, int n_tiles, int k_steps) {
  int best = 1;
  for (int d = 1; d <= kMaxSplitK; ++d)
    if (k_steps % d == 0 && k_steps / d >= 2 && (long)n_tiles * d <= n_cu) best = d;
  return best;
}

pc_status launch_splitk_partial(percache_ctx *ctx, const __bf16 *a, int lda, const __bf16 *w0, const __bf16 *w1, int n_split,
                                int ldw, float *part, int M, int N, int K, int n_k, hipStream_t stream) {
  if (N % BF || n_split % BF || K % (pc::gemm::BK * n_k)) return fail(ctx, PC_ESHAPE, "split-k projection: N %d, K %d, slices %d", N, K, n_k);
  const int k_slice = K / n_k;
  // LDS stages: all k-steps of a workgroup in flight at once when there are up to four of them
  const bool deep = k_slice / pc::gemm::BK > 2;
#define PC_SPLITK(NTB, NS) \
  hipLaunchKernelGGL((splitk_partial_kernel<NTB, NS>), grid, dim3(256), 0, stream, a, lda, w0, w1, n_split, ldw, part, M, N, k_slice)
  if (M > 64) {
    dim3 grid(N / BF, n_k, (M + 127) / 128);
    if (deep) PC_SPLITK(2, 4); else PC_SPLITK(2, 2);
  } else {
    dim3 grid(N / BF, n_k, 1);
    if (deep) PC_SPLITK(1, 4); else PC_SPLITK(1, 2);
  }
#undef PC_SPLITK
  PC_HIP(ctx, hipGetLastError());
  return PC_OK;
}

}  // namespace pc

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

static pc_status run_stack(percache_ctx *ctx, const percache_block_weights *layers_host, int32_t n_layers, int32_t ffn,
                           float eps, const void *h_in_dev, int32_t batch, int32_t t_fresh,
                           const int32_t *slot_ids_host, const int32_t *used_len_host, const int32_t *n_chunks_host,
                           int32_t max_chunks, const int32_t *save_bounds_host, const int32_t *save_slots_host,
                           int32_t n_save, const int32_t *append_slots_host, void *h_out_dev, void *workspace_dev,
                           size_t workspace_bytes, void *stream, const int32_t *table_dev = nullptr,
                           const pc_table_shadow *shadow = nullptr) {
  if (!ctx) return PC_EINVAL;
  const percache_config &c = ctx->cfg;
  if (append_slots_host && batch >= 1 && t_fresh >= 1) {
    for (int b = 0; b < batch; ++b) {
      const int slot = append_slots_host[b];
      if (slot < 0) continue;
      if (slot >= c.n_slots) return pc::fail(ctx, PC_ESLOT, "append slot %d out of range [0,%d)", slot, c.n_slots);
      for (int bb = 0; bb < b; ++bb)
        if (append_slots_host[bb] == slot) return pc::fail(ctx, PC_EINVAL, "append slot %d appears twice", slot);
      for (int l = 0; l < n_layers && l < c.n_layers; ++l) {
        const int have = ctx->slot_len[(size_t)l * c.n_slots + slot];
        if (have != ctx->slot_len[slot]) return pc::fail(ctx, PC_ELEN, "append slot %d holds different lengths in layers 0 and %d", slot, l);
        if (have + t_fresh > c.slot_capacity)
          return pc::fail(ctx, PC_ELEN, "append slot %d holds %d tokens: %d more do not fit the capacity %d", slot, have, t_fresh, c.slot_capacity);
      }
    }
  }
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
    const void *opt[3] = {w.qkv_bias, w.q_norm, w.k_norm};
    for (const void *p : opt)
      if (p && !aligned16(p)) return pc::fail(ctx, PC_EINVAL, "layer %d: misaligned optional weight pointer", l);
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
  if (shadow && rows != shadow->rows)
    return pc::fail(ctx, PC_ELEN, "the slots' formats or lengths no longer match the device chunk table: put it again");
  const int formats = pc::table_formats(rows, pc::tbl_stride(max_chunks), batch);
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
  if (table_dev) {
    ws.pf.table = const_cast<int32_t *>(table_dev);  // the list is on the device already: nothing to copy
  } else {
    st = pc::upload_table(ctx, rows, ws.pf.table, s);
    if (st != PC_OK) return st;
  }
  const int H = c.hidden, A = c.n_q_heads * c.head_dim;
  const __bf16 *h_cur = (const __bf16 *)h_in_dev;
  __bf16 *h_out = (__bf16 *)h_out_dev;
  for (int l = 0; l < n_layers; ++l) {
    const percache_block_weights &w = layers_host[l];
#define PC_TRY(call) do { st = (call); if (st != PC_OK) return st; } while (0)
    // few token rows: split-k projections, whose reduce kernels also apply the residual and the next RMSNorm
    const bool skinny = pc::splitk_applies(M) && ffn % BF == 0;
    if (!skinny || l == 0) PC_TRY(launch_rmsnorm(ctx, h_cur, (const __bf16 *)w.gain1, ws.normed, (int)M, H, eps, s));
    bool v_blocked = false;
    pc::QkvExtras extras;
    extras.bias = (const __bf16 *)w.qkv_bias;
    extras.q_norm = (const __bf16 *)w.q_norm;
    extras.k_norm = (const __bf16 *)w.k_norm;
    extras.eps = eps;
    PC_TRY(pc::launch_qkv_rope(ctx, ws.normed, (const __bf16 *)w.wqkv, batch, t_fresh, ws.pf.table, stride, ws.pf.q, ws.pf.k, ws.pf.v, s,
                               skinny ? ws.pf.gemm_part : nullptr, extras, ws.pf.v_blk, &v_blocked));
    if (!v_blocked) PC_TRY(pc::launch_v_repack(ctx, ws.pf.v, ws.pf.v_blk, batch, t_fresh, s));
    PC_TRY(pc::launch_attention(ctx, l, ws.pf.q, ws.pf.k, ws.pf.v_blk, batch, t_fresh, ws.pf.table, stride, min_tiles, 0, ws.attn,
                                ws.pf.part_o, ws.pf.part_ml, s, formats));
    for (int b = 0; b < batch && n_save > 0; ++b)
      for (int j = 0; j < n_save; ++j) {
        const int slot = save_slots_host[(size_t)b * n_save + j];
        if (slot < 0) continue;
        const int lo = save_bounds_host[j], cnt = save_bounds_host[j + 1] - lo;
        const size_t at = ((size_t)b * c.n_kv_heads * t_fresh + lo) * c.head_dim;
        PC_TRY(pc::launch_kv_store(ctx, l, slot, ws.pf.k + at, ws.pf.v + at, cnt, (long)t_fresh * c.head_dim, s));
        ctx->slot_len[(size_t)l * c.n_slots + slot] = cnt;
      }
    for (int b = 0; b < batch && append_slots_host; ++b) {
      // after the attention launch in stream order: the keys it gathered from this slot are the older ones
      const int slot = append_slots_host[b];
      if (slot < 0) continue;
      const int have = ctx->slot_len[(size_t)l * c.n_slots + slot];
      const size_t at = (size_t)b * c.n_kv_heads * t_fresh * c.head_dim;
      PC_TRY(pc::launch_kv_append(ctx, l, slot, ws.pf.k + at, ws.pf.v + at, have, t_fresh, (long)t_fresh * c.head_dim, s));
      ctx->slot_len[(size_t)l * c.n_slots + slot] = have + t_fresh;
    }
    if (skinny) {
      const int m_tiles = M > 128 ? 2 : 1;
      const __bf16 *next_gain = l + 1 < n_layers ? (const __bf16 *)layers_host[l + 1].gain1 : nullptr;
      int nk = pc::choose_split_k(ctx->n_cu, H / BF * m_tiles, A / pc::gemm::BK);
      PC_TRY(pc::launch_splitk_partial(ctx, ws.attn, A, (const __bf16 *)w.wo, (const __bf16 *)w.wo, H, A, ws.part, (int)M, H, A, nk, s));
      PC_TRY(launch_reduce_residual_norm(ctx, ws.part, nk, (int)M, H, h_cur, ws.mid, (const __bf16 *)w.gain2, ws.normed, eps, s));
      if (M > 64 && ffn % 16 == 0) {
        // many features, short contraction: one pass with 32 weight rows per workgroup beats slices + a second kernel
        hipLaunchKernelGGL(swiglu_skinny_kernel, dim3(ffn / 16, m_tiles), dim3(256), 0, s, ws.normed, (const __bf16 *)w.w_gate,
                           (const __bf16 *)w.w_up, ws.act, (int)M, ffn, H);
        PC_HIP(ctx, hipGetLastError());
      } else {
        nk = pc::choose_split_k(ctx->n_cu, 2 * ffn / BF * m_tiles, H / pc::gemm::BK);
        PC_TRY(pc::launch_splitk_partial(ctx, ws.normed, H, (const __bf16 *)w.w_gate, (const __bf16 *)w.w_up, ffn, H, ws.part, (int)M, 2 * ffn, H, nk, s));
        PC_TRY(launch_reduce_swiglu(ctx, ws.part, nk, (int)M, ffn, ws.act, s));
      }
      nk = pc::choose_split_k(ctx->n_cu, H / BF * m_tiles, ffn / pc::gemm::BK);
      PC_TRY(pc::launch_splitk_partial(ctx, ws.act, ffn, (const __bf16 *)w.w_down, (const __bf16 *)w.w_down, H, ffn, ws.part, (int)M, H, ffn, nk, s));
      PC_TRY(launch_reduce_residual_norm(ctx, ws.part, nk, (int)M, H, ws.mid, h_out, next_gain, ws.normed, eps, s));
    } else {
      PC_TRY(launch_linear_residual(ctx, ws.attn, (const __bf16 *)w.wo, h_cur, ws.mid, (int)M, H, A, s));
      PC_TRY(launch_rmsnorm(ctx, ws.mid, (const __bf16 *)w.gain2, ws.normed, (int)M, H, eps, s));
      PC_TRY(launch_linear_swiglu(ctx, ws.normed, (const __bf16 *)w.w_gate, (const __bf16 *)w.w_up, ws.act, (int)M, ffn, H, s));
      PC_TRY(launch_linear_residual(ctx, ws.act, (const __bf16 *)w.w_down, ws.mid, h_out, (int)M, H, ffn, s));
    }
#undef PC_TRY
    h_cur = h_out;
  }
  return PC_OK;
}

pc_status percache_stack_reuse(percache_ctx *ctx, const percache_block_weights *layers_host, int32_t n_layers, int32_t ffn,
                               float eps, const void *h_in_dev, int32_t batch, int32_t t_fresh,
                               const int32_t *slot_ids_host, const int32_t *used_len_host, const int32_t *n_chunks_host,
                               int32_t max_chunks, const int32_t *save_bounds_host, const int32_t *save_slots_host,
                               int32_t n_save, void *h_out_dev, void *workspace_dev, size_t workspace_bytes, void *stream) {
  return run_stack(ctx, layers_host, n_layers, ffn, eps, h_in_dev, batch, t_fresh, slot_ids_host, used_len_host, n_chunks_host,
                   max_chunks, save_bounds_host, save_slots_host, n_save, nullptr, h_out_dev, workspace_dev, workspace_bytes, stream);
}

pc_status percache_stack_reuse_table(percache_ctx *ctx, const percache_block_weights *layers_host, int32_t n_layers,
                                     int32_t ffn, float eps, const void *h_in_dev, int32_t batch, int32_t t_fresh,
                                     const void *table_dev, void *h_out_dev, void *workspace_dev, size_t workspace_bytes,
                                     void *stream) {
  if (!ctx) return PC_EINVAL;
  const pc_table_shadow *sh = pc::find_table(ctx, table_dev, batch);
  if (!sh) return PC_EINVAL;
  return run_stack(ctx, layers_host, n_layers, ffn, eps, h_in_dev, batch, t_fresh, sh->ids.data(), sh->used.data(),
                   sh->n_chunks.data(), sh->max_chunks, nullptr, nullptr, 0, nullptr, h_out_dev, workspace_dev, workspace_bytes,
                   stream, (const int32_t *)table_dev, sh);
}

pc_status percache_stack_decode(percache_ctx *ctx, const percache_block_weights *layers_host, int32_t n_layers, int32_t ffn,
                                float eps, const void *h_in_dev, int32_t batch, int32_t n_new,
                                const int32_t *slot_ids_host, const int32_t *used_len_host, const int32_t *n_chunks_host,
                                int32_t max_chunks, const int32_t *append_slots_host, void *h_out_dev, void *workspace_dev,
                                size_t workspace_bytes, void *stream) {
  if (!ctx) return PC_EINVAL;
  if (!append_slots_host) return pc::fail(ctx, PC_EINVAL, "append_slots_host is NULL");
  return run_stack(ctx, layers_host, n_layers, ffn, eps, h_in_dev, batch, n_new, slot_ids_host, used_len_host, n_chunks_host,
                   max_chunks, nullptr, nullptr, 0, append_slots_host, h_out_dev, workspace_dev, workspace_bytes, stream);
}

}  // extern "C"
