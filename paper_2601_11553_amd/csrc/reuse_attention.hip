// Attention of the fresh rows over [cached chunk K/V gathered by slot id ; fresh K/V] (Sec. 4.2.2,
// App. B.1: the loaded tensors are put in front of the projected ones along the sequence axis and the
// attention module then proceeds as usual).  The concatenation is never materialised: the kernel walks
// the query's chunk list, streams each (slot, kv head) run of the store tile by tile through LDS, and
// finishes with the fresh keys under the causal mask.
//
// Shape of the computation (64-wide wavefronts, bf16 32x32x16 MFMA, fp32 softmax state):
//   - the G = Hq/Hkv query heads of one kv head are stacked: R = G*T_f rows share every K/V tile;
//   - a workgroup of 4 wavefronts owns 128 rows, a wavefront 32 rows, and loops over 64-key tiles;
//   - scores are computed transposed, S^T = K Q^T, so that a lane's 32 accumulators all belong to ONE
//     query row: the row max/sum are lane-local plus a single exchange with lane+32, and the bf16
//     probabilities are already in the B-operand layout of O^T += V^T P^T (no LDS round trip for P);
//   - V is transposed on its way into LDS; within each group of 16 keys the columns are stored in the
//     order the accumulator layout delivers them, so each A operand is one 16-byte LDS read;
//   - the key axis can be partitioned over workgroups (split-KV); partial (max, sum, output) triples are
//     merged by a small second kernel with the usual log-sum-exp rule.
#include "percache_internal.hpp"

namespace {
using pc::bf16x8;
using pc::f32x16;
using pc::kKvTile;
using pc::kTblHeader;

constexpr int TK = kKvTile;  // keys per tile
constexpr int QROWS = 128;   // query rows per workgroup

template <int D>
struct Lds {
  static constexpr int K_ROW = D * 2 + 16;   // bytes per key row (padded: conflict-free 16-byte reads)
  static constexpr int V_ROW = TK * 2 + 16;  // bytes per V^T row (one head-dim index, TK keys)
  static constexpr int K_BYTES = TK * K_ROW;
  static constexpr int V_BYTES = D * V_ROW;
  static constexpr int STAGE = K_BYTES + V_BYTES;
};

// position of key t (0..15) of a 16-key group inside its V^T row segment: lane group g = (t/4)%2 of the
// score accumulators holds keys {4g..4g+3, 8+4g..8+4g+3}; they are stored contiguously at [8g, 8g+8).
__device__ __forceinline__ int vt_pos16(int t) { return 8 * ((t >> 2) & 1) + 4 * (t >> 3) + (t & 3); }

// 2^x on the hardware transcendental unit; arguments here are <= 0 (or -inf), results in [0, 1].
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <int D>
__global__ __launch_bounds__(256, 2) void reuse_attention_kernel(
    const __bf16 *__restrict__ Q, const __bf16 *__restrict__ Kf, const __bf16 *__restrict__ Vf,
    const __bf16 *__restrict__ k_store, const __bf16 *__restrict__ v_store, const int32_t *__restrict__ table,
    int tbl_stride, int T, int Hq, int Hkv, int C, int n_splits, float scale_log2e, __bf16 *__restrict__ out,
    float *__restrict__ part_o, float *__restrict__ part_ml) {
  using L = Lds<D>;
  constexpr int KS = D / 16;  // k-steps of the QK^T contraction
  constexpr int DB = D / 32;  // 32-wide blocks of the head dim (rows of O^T)
  __shared__ __align__(16) char lds[2 * L::STAGE];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, g2 = lane >> 5;
  const int G = Hq / Hkv, R = G * T;
  const int qt = blockIdx.x, gkv = blockIdx.y;
  const int b = blockIdx.z / n_splits, split = blockIdx.z - b * n_splits;

  const int32_t *trow = table + (size_t)b * tbl_stride;
  const int n_chunks = trow[0];
  const int n_cached_tiles = trow[2];

  // rows of this workgroup and the fresh tiles they can see
  const int row_first = qt * QROWS;
  const int row_last = min(row_first + QROWS, R) - 1;
  const int i_max = (row_first / T == row_last / T) ? (row_last % T) : (T - 1);
  const int n_tiles = n_cached_tiles + i_max / TK + 1;
  const int tile_begin = (int)((long)split * n_tiles / n_splits);
  const int tile_end = (int)((long)(split + 1) * n_tiles / n_splits);

  // this lane's query row (as column of S^T / O^T)
  const int my_row = row_first + wave * 32 + l32;
  const bool row_ok = my_row < R;
  const int row_c = row_ok ? my_row : R - 1;
  const int hg = row_c / T, my_i = row_c - hg * T;
  const int head = gkv * G + hg;

  // Q fragments (B operand): lane holds q[row][16 ks + 8 g2 .. +7]
  bf16x8 qf[KS];
  {
    const __bf16 *qrow = Q + (((size_t)b * Hq + head) * T + my_i) * D + g2 * 8;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[ks] = *(const bf16x8 *)(qrow + ks * 16);
  }

  f32x16 o_acc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) o_acc[db][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  // ---- tile cursor over the chunk list
  int cur_chunk = 0, cur_off = 0;  // chunk index, tile index inside the chunk
  {
    int rem = tile_begin;
    while (cur_chunk < n_chunks) {
      int ntc = (trow[kTblHeader + 2 * cur_chunk + 1] + TK - 1) / TK;
      if (rem < ntc) break;
      rem -= ntc;
      ++cur_chunk;
    }
    cur_off = rem;  // for fresh tiles: tile index inside the fresh part
  }

  // ---- global -> register staging of one tile
  constexpr int K_PASS = TK * (D / 8) / 256;  // 16-byte loads per thread for the K tile
  constexpr int TPR = D / 8;                  // threads per key row
  pc::u32x4 rk[K_PASS], rv[2][2];
  // V items: wavefront w transposes keys [16w, 16w+16); lane group lg and item it pick the key pair
  const int v_lg = lane >> 4, v_dc0 = lane & 15;
  struct TileDesc { const __bf16 *k, *v; int valid; int t0; bool fresh; };
  auto describe = [&](int chunk, int off, TileDesc &td) __attribute__((always_inline)) {
    if (chunk < n_chunks) {
      int slot = trow[kTblHeader + 2 * chunk], used = trow[kTblHeader + 2 * chunk + 1];
      size_t base = (((size_t)slot * Hkv + gkv) * C + (size_t)off * TK) * D;
      td.k = k_store + base;
      td.v = v_store + base;
      td.valid = min(TK, used - off * TK);
      td.t0 = 0;
      td.fresh = false;
    } else {
      size_t base = (((size_t)b * Hkv + gkv) * T + (size_t)off * TK) * D;
      td.k = Kf + base;
      td.v = Vf + base;
      td.valid = min(TK, T - off * TK);
      td.t0 = off * TK;
      td.fresh = true;
    }
  };
  auto advance = [&]() __attribute__((always_inline)) {
    ++cur_off;
    if (cur_chunk < n_chunks) {
      int ntc = (trow[kTblHeader + 2 * cur_chunk + 1] + TK - 1) / TK;
      if (cur_off >= ntc) {
        cur_off = 0;
        ++cur_chunk;
        // skip chunks with no used tokens
        while (cur_chunk < n_chunks && trow[kTblHeader + 2 * cur_chunk + 1] == 0) ++cur_chunk;
      }
    }
  };
  auto load_tile = [&](const TileDesc &td) __attribute__((always_inline)) {
#pragma unroll
    for (int p = 0; p < K_PASS; ++p) {
      int row = min(tid / TPR + p * (256 / TPR), td.valid - 1);
      rk[p] = *(const pc::u32x4 *)(td.k + (size_t)row * D + (tid % TPR) * 8);
    }
    if (D == 128 || v_dc0 < 8) {
#pragma unroll
      for (int it = 0; it < 2; ++it) {
        int x = (v_lg & 1) + 4 * (v_lg >> 1) + 2 * it;  // key-pair index inside the 16-key group
        int t = wave * 16 + 2 * x;
        int ra = min(t, td.valid - 1), rb = min(t + 1, td.valid - 1);
        rv[it][0] = *(const pc::u32x4 *)(td.v + (size_t)ra * D + v_dc0 * 8);
        rv[it][1] = *(const pc::u32x4 *)(td.v + (size_t)rb * D + v_dc0 * 8);
      }
    }
  };
  auto store_tile = [&](int buf) __attribute__((always_inline)) {
    char *kb = lds + buf * L::STAGE;
    char *vb = kb + L::K_BYTES;
#pragma unroll
    for (int p = 0; p < K_PASS; ++p) {
      int row = tid / TPR + p * (256 / TPR);
      *(pc::u32x4 *)(kb + row * L::K_ROW + (tid % TPR) * 16) = rk[p];
    }
    if (D == 128 || v_dc0 < 8) {
#pragma unroll
      for (int it = 0; it < 2; ++it) {
        // item `it` of lane group v_lg is the key pair stored in 32-bit word (4 it + v_lg) of the 16-key
        // group, i.e. word v_lg of 16-byte chunk (2 wave + it) of the V^T row
        const uint32_t wa[4] = {rv[it][0].x, rv[it][0].y, rv[it][0].z, rv[it][0].w};
        const uint32_t wc[4] = {rv[it][1].x, rv[it][1].y, rv[it][1].z, rv[it][1].w};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          uint32_t w = (e & 1) ? ((wa[e >> 1] >> 16) | (wc[e >> 1] & 0xffff0000u))
                               : ((wa[e >> 1] & 0xffffu) | (wc[e >> 1] << 16));
          int d = v_dc0 * 8 + e;
          int chunk = (2 * wave + it) ^ ((d >> 4) & 7);  // XOR swizzle: conflict-free writes and reads
          *(uint32_t *)(vb + d * L::V_ROW + chunk * 16 + v_lg * 4) = w;
        }
      }
    }
  };

  TileDesc td;
  if (tile_begin < tile_end) {
    // skip leading empty chunks
    while (cur_chunk < n_chunks && trow[kTblHeader + 2 * cur_chunk + 1] == 0) ++cur_chunk;
    describe(cur_chunk, cur_off, td);
    load_tile(td);
    store_tile(0);
  }
  __syncthreads();

  for (int tt = tile_begin; tt < tile_end; ++tt) {
    const int buf = (tt - tile_begin) & 1;
    const TileDesc cur = td;
    const bool has_next = tt + 1 < tile_end;
    if (has_next) {
      advance();
      describe(cur_chunk, cur_off, td);
      load_tile(td);
    }
    const char *kb = lds + buf * L::STAGE;
    const char *vb = kb + L::K_BYTES;

    // ---- S^T = K Q^T : two 32-key blocks
    f32x16 s_acc[2];
#pragma unroll
    for (int kbk = 0; kbk < 2; ++kbk) {
#pragma unroll
      for (int r = 0; r < 16; ++r) s_acc[kbk][r] = 0.f;
      const char *krow = kb + (kbk * 32 + l32) * L::K_ROW + g2 * 16;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        bf16x8 a = *(const bf16x8 *)(krow + ks * 32);
        s_acc[kbk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[ks], s_acc[kbk], 0, 0, 0);
      }
    }

    // ---- mask (ragged tile end, causal part) and online softmax in the log2 domain
    const bool need_mask = cur.valid < TK || (cur.fresh && cur.t0 + TK - 1 > my_i);
    float mx = -INFINITY;
#pragma unroll
    for (int kbk = 0; kbk < 2; ++kbk)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float s = s_acc[kbk][r] * scale_log2e;
        if (need_mask) {
          int t = kbk * 32 + (r >> 2) * 8 + g2 * 4 + (r & 3);
          bool vis = t < cur.valid && (!cur.fresh || cur.t0 + t <= my_i);
          s = vis ? s : -INFINITY;
        }
        s_acc[kbk][r] = s;
        mx = fmaxf(mx, s);
      }
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx);
    const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
    const float alpha = fast_exp2(m_run - m_use);
    m_run = m_new;
    float psum = 0.f;
    bf16x8 pf[2][2];
#pragma unroll
    for (int kbk = 0; kbk < 2; ++kbk)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          float p = fast_exp2(s_acc[kbk][j * 8 + e] - m_use);
          psum += p;
          pf[kbk][j][e] = (__bf16)p;
        }
    l_run = l_run * alpha + psum;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) o_acc[db][r] *= alpha;

    // ---- O^T += V^T P^T
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      const int dd = db * 32 + l32;
      const char *vrow = vb + dd * L::V_ROW;
      const int sw = (dd >> 4) & 7;
#pragma unroll
      for (int kbk = 0; kbk < 2; ++kbk)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          bf16x8 a = *(const bf16x8 *)(vrow + (((kbk * 4 + j * 2 + g2) ^ sw) * 16));
          o_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[kbk][j], o_acc[db], 0, 0, 0);
        }
    }

    if (has_next) store_tile(buf ^ 1);
    __syncthreads();
  }

  // ---- finish: combine the two lanes of a row, normalise, write
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
  if (!row_ok) return;
  if (n_splits == 1) {
    __bf16 *orow = out + ((size_t)b * T + my_i) * ((size_t)Hq * D) + (size_t)head * D;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        pc::bf16x4 v = {(__bf16)(o_acc[db][q4 * 4 + 0] * inv), (__bf16)(o_acc[db][q4 * 4 + 1] * inv),
                        (__bf16)(o_acc[db][q4 * 4 + 2] * inv), (__bf16)(o_acc[db][q4 * 4 + 3] * inv)};
        *(pc::bf16x4 *)(orow + db * 32 + q4 * 8 + g2 * 4) = v;
      }
  } else {
    const size_t prow = (((size_t)b * Hkv + gkv) * R + my_row) * n_splits + split;
    float *po = part_o + prow * D;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        float4 v = make_float4(o_acc[db][q4 * 4 + 0] * inv, o_acc[db][q4 * 4 + 1] * inv, o_acc[db][q4 * 4 + 2] * inv,
                               o_acc[db][q4 * 4 + 3] * inv);
        *(float4 *)(po + db * 32 + q4 * 8 + g2 * 4) = v;
      }
    if (g2 == 0) {
      part_ml[prow * 2] = m_run;
      part_ml[prow * 2 + 1] = l_tot;
    }
  }
}

// Merge of the split-KV partials: m = max m_s, w_s = l_s 2^(m_s - m), o = sum w_s o_s / sum w_s.
// One thread per (row, 4 head-dim elements).
template <int D>
__global__ __launch_bounds__(256) void splitkv_combine_kernel(const float *__restrict__ part_o,
                                                              const float *__restrict__ part_ml, int n_splits, int T,
                                                              int Hq, int Hkv, long total_rows,
                                                              __bf16 *__restrict__ out) {
  constexpr int VPR = D / 4;
  long gid = (long)blockIdx.x * blockDim.x + threadIdx.x;
  long prow = gid / VPR;
  int dv = (int)(gid - prow * VPR);
  if (prow >= total_rows) return;
  const int G = Hq / Hkv, R = G * T;
  long bg = prow / R;
  int row = (int)(prow - bg * R);
  int b = (int)(bg / Hkv), gkv = (int)(bg - (long)b * Hkv);
  int hg = row / T, i = row - hg * T;
  int head = gkv * G + hg;
  const float *ml = part_ml + prow * n_splits * 2;
  float m = -INFINITY;
  for (int s = 0; s < n_splits; ++s) m = fmaxf(m, ml[2 * s]);
  float wsum = 0.f;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int s = 0; s < n_splits; ++s) {
    float ms = ml[2 * s], ls = ml[2 * s + 1];
    if (ls <= 0.f) continue;
    float w = ls * exp2f(ms - m);
    float4 o = *(const float4 *)(part_o + (prow * n_splits + s) * D + dv * 4);
    acc.x += w * o.x; acc.y += w * o.y; acc.z += w * o.z; acc.w += w * o.w;
    wsum += w;
  }
  float inv = wsum > 0.f ? 1.0f / wsum : 0.f;
  pc::bf16x4 v = {(__bf16)(acc.x * inv), (__bf16)(acc.y * inv), (__bf16)(acc.z * inv), (__bf16)(acc.w * inv)};
  *(pc::bf16x4 *)(out + ((size_t)b * T + i) * ((size_t)Hq * D) + (size_t)head * D + dv * 4) = v;
}

}  // namespace

namespace pc {

pc_status launch_attention(percache_ctx *ctx, int layer, const __bf16 *q, const __bf16 *kf, const __bf16 *vf,
                           int batch, int t_fresh, const int32_t *table_dev, int tbl_stride, int min_tiles,
                           int n_splits, __bf16 *out, float *part_o, float *part_ml, hipStream_t stream) {
  const percache_config &c = ctx->cfg;
  const int G = c.n_q_heads / c.n_kv_heads, R = G * t_fresh;
  const int q_tiles = (R + QROWS - 1) / QROWS;
  if (n_splits <= 0) {
    long base = (long)batch * c.n_kv_heads * q_tiles;
    long want = 2L * ctx->n_cu;
    n_splits = (int)((want + base - 1) / base);
    int cap = min_tiles / 4;  // keep at least 4 tiles per partition
    if (n_splits > cap) n_splits = cap;
    if (n_splits < 1) n_splits = 1;
  }
  {
    int cap = max_splits_for(c, ctx->n_cu, batch, t_fresh);
    if (n_splits > cap) n_splits = cap;
  }
  const __bf16 *ks = ctx->k_store + (size_t)layer * ctx->layer_stride;
  const __bf16 *vs = ctx->v_store + (size_t)layer * ctx->layer_stride;
  const float scale_log2e = 1.4426950408889634f / sqrtf((float)c.head_dim);
  dim3 grid(q_tiles, c.n_kv_heads, batch * n_splits);
  prof_begin(ctx, PC_KERNEL_ATTENTION, stream);
  if (c.head_dim == 128)
    hipLaunchKernelGGL(reuse_attention_kernel<128>, grid, dim3(256), 0, stream, q, kf, vf, ks, vs, table_dev, tbl_stride,
                       t_fresh, c.n_q_heads, c.n_kv_heads, c.slot_capacity, n_splits, scale_log2e, out, part_o, part_ml);
  else
    hipLaunchKernelGGL(reuse_attention_kernel<64>, grid, dim3(256), 0, stream, q, kf, vf, ks, vs, table_dev, tbl_stride,
                       t_fresh, c.n_q_heads, c.n_kv_heads, c.slot_capacity, n_splits, scale_log2e, out, part_o, part_ml);
  prof_end(ctx, PC_KERNEL_ATTENTION, stream);
  PC_HIP(ctx, hipGetLastError());
  if (n_splits > 1) {
    long total_rows = (long)batch * c.n_kv_heads * R;
    long threads = total_rows * (c.head_dim / 4);
    int blocks = (int)((threads + 255) / 256);
    if (c.head_dim == 128)
      hipLaunchKernelGGL(splitkv_combine_kernel<128>, dim3(blocks), dim3(256), 0, stream, part_o, part_ml, n_splits,
                         t_fresh, c.n_q_heads, c.n_kv_heads, total_rows, out);
    else
      hipLaunchKernelGGL(splitkv_combine_kernel<64>, dim3(blocks), dim3(256), 0, stream, part_o, part_ml, n_splits,
                         t_fresh, c.n_q_heads, c.n_kv_heads, total_rows, out);
    PC_HIP(ctx, hipGetLastError());
  }
  return PC_OK;
}

}  // namespace pc
