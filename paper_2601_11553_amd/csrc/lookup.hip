// Query-level match (Sec. 4.2.1): cosine top-1 of probe embeddings against every row of the QA bank's
// embedding matrix, and the hit flag against tau_query.
//
// The bank is streamed from HBM exactly once per pass of up to 64 probes.  The dot products run on the
// fp16 matrix cores (16x16x32, fp32 accumulate) only because they perform the cross-lane reduction for
// free; the kernel is bound by the HBM stream of the bank, not by arithmetic.
#include <climits>

#include "percache_internal.hpp"

namespace {
using pc::f16x8;
using pc::f32x4;
using pc::u32x4;

struct Best {
  float s;
  int idx;
};
__device__ __forceinline__ bool better(float s1, int i1, float s2, int i2) { return s1 > s2 || (s1 == s2 && i1 < i2); }

// ---------------------------------------------------------------------------------------------------
// Inverse L2 norms of newly written bank rows; one wavefront per row.  Also copies the rows into the
// bank when the source is elsewhere.
// ---------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void bank_put_kernel(const _Float16 *__restrict__ src, _Float16 *__restrict__ dst,
                                                       float *__restrict__ inv_norm, int n, int d) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= n) return;
  const u32x4 *s = (const u32x4 *)(src + (size_t)row * d);
  u32x4 *t = (u32x4 *)(dst + (size_t)row * d);
  float ss = 0.f;
  for (int v = lane; v < d / 8; v += 64) {
    u32x4 raw = s[v];
    t[v] = raw;
    f16x8 h = __builtin_bit_cast(f16x8, raw);
#pragma unroll
    for (int e = 0; e < 8; ++e) ss += (float)h[e] * (float)h[e];
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
  if (lane == 0) inv_norm[row] = ss > 0.f ? 1.0f / sqrtf(ss) : 0.f;
}

// ---------------------------------------------------------------------------------------------------
// Streaming pass.  Workgroup = 4 wavefronts; workgroup b owns a contiguous range of 16-row blocks (at most
// kMaxBlocksPerWg), its wavefronts take them round-robin.  For one row block a wavefront issues, per step,
// one 16-byte load per lane: lane (r = lane%16, g = lane/16) reads elements [32 step + 8 g, +8) of row r,
// i.e. the four lanes of a row cover 64 contiguous bytes and consecutive steps walk along the row.  Loads
// are grouped in chunks of CS steps; the chunk after the one being multiplied is always in flight (two
// register sets, all indices compile-time, so the only waits are partial vmcnt waits).  The probes of the
// pass (NPB blocks of 16, zero padded) and the inverse norms of the workgroup's rows sit in LDS.
// Result lane layout of the 16x16 product: lane holds probe (lane%16), rows 4*(lane/16) + 0..3.
// ---------------------------------------------------------------------------------------------------
constexpr int kMaxBlocksPerWg = 256;  // 4096 rows: bounds the LDS copy of the inverse norms (16 KB)

template <int NPB, int CS>
__global__ __launch_bounds__(256) void lookup_stream_kernel(const _Float16 *__restrict__ bank,
                                                            const float *__restrict__ inv_norm, int N, int d,
                                                            const _Float16 *__restrict__ probes, int n_probes,
                                                            int per_wg, Best *__restrict__ partial) {
  extern __shared__ __align__(16) char smem[];
  const int row_bytes = d * 2 + 64;  // padded probe row in LDS
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r16 = lane & 15, g = lane >> 4;

  const int n_blocks = (N + 15) / 16;
  const int rb_begin = blockIdx.x * per_wg;
  const int rb_end = min(n_blocks, rb_begin + per_wg);

  // stage probes (zero rows beyond n_probes) and this workgroup's inverse norms (zero beyond N)
  const int vec_per_row = d / 8;
  for (int v = tid; v < NPB * 16 * vec_per_row; v += 256) {
    int p = v / vec_per_row, c = v - p * vec_per_row;
    u32x4 val = {0, 0, 0, 0};
    if (p < n_probes) val = ((const u32x4 *)(probes + (size_t)p * d))[c];
    *(u32x4 *)(smem + (size_t)p * row_bytes + c * 16) = val;
  }
  float *inv_lds = (float *)(smem + (size_t)NPB * 16 * row_bytes);
  for (int r = tid; r < per_wg * 16; r += 256) {
    int row = rb_begin * 16 + r;
    inv_lds[r] = row < N ? inv_norm[row] : 0.f;
  }
  __syncthreads();

  const int chunks = d / (32 * CS);

  float best_s[NPB][4];
  int best_i[NPB][4];
#pragma unroll
  for (int pb = 0; pb < NPB; ++pb)
#pragma unroll
    for (int r = 0; r < 4; ++r) { best_s[pb][r] = -INFINITY; best_i[pb][r] = INT_MAX; }

  u32x4 a0[CS], a1[CS];
  auto issue = [&](int rb, int chunk, u32x4 (&dst)[CS]) __attribute__((always_inline)) {
    int row = min(rb * 16 + r16, N - 1);
    const u32x4 *src = (const u32x4 *)(bank + (size_t)row * d + chunk * (CS * 32) + g * 8);
#pragma unroll
    for (int s = 0; s < CS; ++s) dst[s] = __builtin_nontemporal_load(src + s * 4);
  };
  f32x4 acc[NPB];
  auto clear = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int pb = 0; pb < NPB; ++pb) acc[pb] = f32x4{0.f, 0.f, 0.f, 0.f};
  };
  auto compute = [&](int chunk, const u32x4 (&src)[CS]) __attribute__((always_inline)) {
    const char *pbase = smem + (size_t)r16 * row_bytes + (chunk * CS * 32 + g * 8) * 2;
#pragma unroll
    for (int s = 0; s < CS; ++s) {
      f16x8 av = __builtin_bit_cast(f16x8, src[s]);
#pragma unroll
      for (int pb = 0; pb < NPB; ++pb) {
        f16x8 bv = *(const f16x8 *)(pbase + (size_t)pb * 16 * row_bytes + s * 64);
        acc[pb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(av, bv, acc[pb], 0, 0, 0);
      }
    }
  };
  // scale by the rows' inverse norms and keep the running best (strict >: the lowest row wins ties)
  auto epilogue = [&](int rb) __attribute__((always_inline)) {
    const f32x4 inv4 = *(const f32x4 *)(inv_lds + (rb - rb_begin) * 16 + g * 4);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int row = rb * 16 + g * 4 + r;
      const bool ok = row < N;
#pragma unroll
      for (int pb = 0; pb < NPB; ++pb) {
        float s = acc[pb][r] * inv4[r];
        if (ok && s > best_s[pb][r]) { best_s[pb][r] = s; best_i[pb][r] = row; }
      }
    }
  };
  auto advance = [&](int &rb_, int &c_) __attribute__((always_inline)) {
    if (++c_ == chunks) { c_ = 0; rb_ += 4; }
  };

  // flat software pipeline over (row block, chunk): one chunk of loads is always in flight ahead.  The
  // prefetch is issued unconditionally (past the end it re-reads the wavefront's last block and is never
  // used), so the loop body is straight-line code and every wait is an exact partial vmcnt wait.
  int rb = rb_begin + wave, c = 0;
  int prb = rb, pch = 0;
  const int rb_last = rb_end - 1;
  if (rb < rb_end) {
    issue(prb, pch, a0);
    clear();
    while (true) {
      advance(prb, pch);
      issue(min(prb, rb_last), pch, a1);
      compute(c, a0);
      if (c == chunks - 1) { epilogue(rb); clear(); }
      advance(rb, c);
      if (rb >= rb_end) break;
      advance(prb, pch);
      issue(min(prb, rb_last), pch, a0);
      compute(c, a1);
      if (c == chunks - 1) { epilogue(rb); clear(); }
      advance(rb, c);
      if (rb >= rb_end) break;
    }
  }

  // lane-local over r, then the four lanes that share a probe, then the four wavefronts
  __syncthreads();  // probes no longer needed: reuse LDS for the cross-wave step
  Best *red = (Best *)smem;  // [4 waves][NPB*16]
#pragma unroll
  for (int pb = 0; pb < NPB; ++pb) {
    float s = best_s[pb][0];
    int i = best_i[pb][0];
#pragma unroll
    for (int r = 1; r < 4; ++r)
      if (better(best_s[pb][r], best_i[pb][r], s, i)) { s = best_s[pb][r]; i = best_i[pb][r]; }
#pragma unroll
    for (int o = 16; o < 64; o <<= 1) {
      float s2 = __shfl_xor(s, o, 64);
      int i2 = __shfl_xor(i, o, 64);
      if (better(s2, i2, s, i)) { s = s2; i = i2; }
    }
    if (g == 0) red[wave * (NPB * 16) + pb * 16 + r16] = Best{s, i};
  }
  __syncthreads();
  if (tid < NPB * 16) {
    Best b = red[tid];
#pragma unroll
    for (int w = 1; w < 4; ++w) {
      Best o = red[w * (NPB * 16) + tid];
      if (better(o.s, o.idx, b.s, b.idx)) b = o;
    }
    partial[(size_t)blockIdx.x * (NPB * 16) + tid] = b;
  }
}

// ---------------------------------------------------------------------------------------------------
// Per probe: merge the workgroup partials, divide by the probe's norm, compare with tau.
// One workgroup (one wavefront) per probe.
// ---------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void lookup_finalize_kernel(const Best *__restrict__ partial, int n_partials,
                                                             int partial_stride, const _Float16 *__restrict__ probes,
                                                             int d, float tau, int32_t *__restrict__ idx_out,
                                                             float *__restrict__ sim_out, uint8_t *__restrict__ hit_out) {
  const int p = blockIdx.x, lane = threadIdx.x;
  float ss = 0.f;
  const u32x4 *src = (const u32x4 *)(probes + (size_t)p * d);
  for (int v = lane; v < d / 8; v += 64) {
    f16x8 h = __builtin_bit_cast(f16x8, src[v]);
#pragma unroll
    for (int e = 0; e < 8; ++e) ss += (float)h[e] * (float)h[e];
  }
  float s = -INFINITY;
  int i = INT_MAX;
  for (int w = lane; w < n_partials; w += 64) {
    Best b = partial[(size_t)w * partial_stride + p];
    if (better(b.s, b.idx, s, i)) { s = b.s; i = b.idx; }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    ss += __shfl_xor(ss, o, 64);
    float s2 = __shfl_xor(s, o, 64);
    int i2 = __shfl_xor(i, o, 64);
    if (better(s2, i2, s, i)) { s = s2; i = i2; }
  }
  if (lane == 0) {
    float inv = ss > 0.f ? 1.0f / sqrtf(ss) : 0.f;
    float sim = s * inv;
    idx_out[p] = i;
    sim_out[p] = sim;
    hit_out[p] = sim > tau ? 1 : 0;
  }
}

__global__ void lookup_empty_kernel(int n, int32_t *idx_out, float *sim_out, uint8_t *hit_out) {
  int p = blockIdx.x * blockDim.x + threadIdx.x;
  if (p < n) { idx_out[p] = -1; sim_out[p] = -INFINITY; hit_out[p] = 0; }
}

constexpr int kPassProbes = 64;

// Workgroups of one pass and 16-row blocks per workgroup.
void stream_shape(const percache_ctx *ctx, int npb, int N, int &grid, int &per_wg) {
  const int per_cu = npb >= 4 ? 1 : (npb == 2 ? 2 : 4);  // bounded by the LDS copy of the probes
  const int n_blocks = (N + 15) / 16;
  grid = ctx->n_cu * per_cu;
  const int need = (n_blocks + 3) / 4;  // at least one block per wavefront
  if (grid > need) grid = need > 0 ? need : 1;
  per_wg = (n_blocks + grid - 1) / grid;
  if (per_wg > kMaxBlocksPerWg) {
    per_wg = kMaxBlocksPerWg;
    grid = (n_blocks + per_wg - 1) / per_wg;
  }
}
int max_stream_grid(const percache_ctx *ctx) {
  int by_rows = (ctx->cfg.bank_capacity / 16 + kMaxBlocksPerWg) / kMaxBlocksPerWg;
  int by_cu = ctx->n_cu * 4;
  return by_rows > by_cu ? by_rows : by_cu;
}

template <int NPB, int CS>
pc_status launch_stream(percache_ctx *ctx, int grid, int per_wg, size_t lds, hipStream_t st, int N, int d,
                        const _Float16 *pp, int np, Best *partial) {
  if (lds > 64 * 1024) {
    static bool big_lds_set = false;  // dynamic LDS above 64 KB must be opted into once per kernel
    if (!big_lds_set) {
      PC_HIP(ctx, hipFuncSetAttribute((const void *)lookup_stream_kernel<NPB, CS>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
      big_lds_set = true;
    }
  }
  hipLaunchKernelGGL((lookup_stream_kernel<NPB, CS>), dim3(grid), dim3(256), lds, st, ctx->bank, ctx->bank_inv, N, d, pp, np,
                     per_wg, partial);
  return PC_OK;
}

}  // namespace

extern "C" {

pc_status percache_bank_put(percache_ctx *ctx, int32_t index, const void *emb_dev, int32_t n, void *stream) {
  if (!ctx) return PC_EINVAL;
  const percache_config &c = ctx->cfg;
  if (c.bank_capacity <= 0) return pc::fail(ctx, PC_ESHAPE, "context was created without a bank");
  if (!emb_dev) return pc::fail(ctx, PC_EINVAL, "emb_dev is NULL");
  if ((uintptr_t)emb_dev % 16) return pc::fail(ctx, PC_EINVAL, "emb_dev must be 16-byte aligned");
  if (n < 1) return pc::fail(ctx, PC_EINVAL, "n must be positive");
  if (index < 0 || index > ctx->bank_size) return pc::fail(ctx, PC_EINVAL, "index %d outside [0,%d] (no holes allowed)", index, ctx->bank_size);
  if ((long)index + n > c.bank_capacity) return pc::fail(ctx, PC_ENOMEM, "rows [%d,%ld) exceed bank capacity %d", index, (long)index + n, c.bank_capacity);
  hipLaunchKernelGGL(bank_put_kernel, dim3((n + 3) / 4), dim3(256), 0, (hipStream_t)stream, (const _Float16 *)emb_dev,
                     ctx->bank + (size_t)index * c.emb_dim, ctx->bank_inv + index, n, c.emb_dim);
  PC_HIP(ctx, hipGetLastError());
  if (index + n > ctx->bank_size) ctx->bank_size = index + n;
  return PC_OK;
}

size_t percache_lookup_workspace_bytes(const percache_ctx *ctx, int32_t n_probes) {
  if (!ctx || n_probes < 0) return 0;
  return pc::align_up((size_t)max_stream_grid(ctx) * kPassProbes * sizeof(Best));
}

pc_status percache_lookup(percache_ctx *ctx, const void *probes_dev, int32_t n_probes, float tau, int32_t *idx_out_dev,
                          float *sim_out_dev, uint8_t *hit_out_dev, void *workspace_dev, size_t workspace_bytes,
                          void *stream) {
  if (!ctx) return PC_EINVAL;
  const percache_config &c = ctx->cfg;
  if (c.bank_capacity <= 0) return pc::fail(ctx, PC_ESHAPE, "context was created without a bank");
  if (n_probes < 0) return pc::fail(ctx, PC_EINVAL, "n_probes is negative");
  if (n_probes == 0) return PC_OK;
  if (!probes_dev || !idx_out_dev || !sim_out_dev || !hit_out_dev) return pc::fail(ctx, PC_EINVAL, "NULL probe or output pointer");
  if ((uintptr_t)probes_dev % 16) return pc::fail(ctx, PC_EINVAL, "probes_dev must be 16-byte aligned");
  if (!(tau == tau)) return pc::fail(ctx, PC_EINVAL, "tau is NaN");
  hipStream_t st = (hipStream_t)stream;
  const int N = ctx->bank_size, d = c.emb_dim;
  if (N == 0) {
    hipLaunchKernelGGL(lookup_empty_kernel, dim3((n_probes + 255) / 256), dim3(256), 0, st, n_probes, idx_out_dev, sim_out_dev, hit_out_dev);
    PC_HIP(ctx, hipGetLastError());
    return PC_OK;
  }
  if (!workspace_dev || workspace_bytes < percache_lookup_workspace_bytes(ctx, n_probes))
    return pc::fail(ctx, PC_ENOMEM, "lookup workspace has %zu bytes, need %zu", workspace_bytes, percache_lookup_workspace_bytes(ctx, n_probes));
  if ((uintptr_t)workspace_dev % 16) return pc::fail(ctx, PC_EINVAL, "workspace must be 16-byte aligned");
  Best *partial = (Best *)workspace_dev;
  const _Float16 *probes = (const _Float16 *)probes_dev;
  for (int p0 = 0; p0 < n_probes; p0 += kPassProbes) {
    int np = n_probes - p0 < kPassProbes ? n_probes - p0 : kPassProbes;
    int npb = np <= 16 ? 1 : (np <= 32 ? 2 : 4);
    int grid, per_wg;
    stream_shape(ctx, npb, N, grid, per_wg);
    size_t lds = (size_t)npb * 16 * (d * 2 + 64) + (size_t)per_wg * 16 * sizeof(float);
    const _Float16 *pp = probes + (size_t)p0 * d;
    pc::prof_begin(ctx, PC_KERNEL_LOOKUP, st);
    pc_status ls;
#define PC_STREAM(NPB_)                                                                                        \
  (d == 64    ? launch_stream<NPB_, 2>(ctx, grid, per_wg, lds, st, N, d, pp, np, partial)                       \
   : d == 128 ? launch_stream<NPB_, 4>(ctx, grid, per_wg, lds, st, N, d, pp, np, partial)                       \
              : launch_stream<NPB_, 8>(ctx, grid, per_wg, lds, st, N, d, pp, np, partial))
    if (npb == 1) ls = PC_STREAM(1);
    else if (npb == 2) ls = PC_STREAM(2);
    else ls = PC_STREAM(4);
#undef PC_STREAM
    if (ls != PC_OK) return ls;
    pc::prof_end(ctx, PC_KERNEL_LOOKUP, st);
    PC_HIP(ctx, hipGetLastError());
    hipLaunchKernelGGL(lookup_finalize_kernel, dim3(np), dim3(64), 0, st, partial, grid, npb * 16, pp, d, tau,
                       idx_out_dev + p0, sim_out_dev + p0, hit_out_dev + p0);
    PC_HIP(ctx, hipGetLastError());
  }
  return PC_OK;
}

}  // extern "C"
