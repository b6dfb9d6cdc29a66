// Query-level match (Sec. 4.2.1): cosine top-1 of probe embeddings against every row of the QA bank's
// embedding matrix, and the hit flag against tau_query.
//
// The bank is streamed from HBM exactly once per pass of up to 32 probes.  The dot products run on the
// fp16 matrix cores (16x16x32, fp32 accumulate) only because they perform the cross-lane reduction for
// free; the kernel is bound by the HBM stream of the bank, not by arithmetic.
#include <climits>
#include <cmath>

#include "gemm_tile.hpp"

namespace {
using pc::f16x8;
using pc::f32x4;
using pc::u32x4;

struct Best {
  float s;
  int idx;
};
__device__ __forceinline__ bool better(float s1, int i1, float s2, int i2) { return s1 > s2 || (s1 == s2 && i1 < i2); }

// Sorted list of the K best (similarity, row) pairs, best first; ties go to the lower row.
template <int K>
struct TopK {
  float s[K];
  int i[K];
  __device__ __forceinline__ void clear() {
#pragma unroll
    for (int j = 0; j < K; ++j) { s[j] = -INFINITY; i[j] = INT_MAX; }
  }
  __device__ __forceinline__ void insert(float cs, int ci) {
    if (!better(cs, ci, s[K - 1], i[K - 1])) return;
    s[K - 1] = cs;
    i[K - 1] = ci;
#pragma unroll
    for (int j = K - 1; j > 0; --j) {
      const bool up = better(s[j], i[j], s[j - 1], i[j - 1]);
      const float ts = s[j]; const int ti = i[j];
      s[j] = up ? s[j - 1] : ts;   i[j] = up ? i[j - 1] : ti;
      s[j - 1] = up ? ts : s[j - 1]; i[j - 1] = up ? ti : i[j - 1];
    }
  }
  // drops the head if this list owns it
  __device__ __forceinline__ void pop_if(bool mine) {
#pragma unroll
    for (int j = 0; j < K - 1; ++j) { s[j] = mine ? s[j + 1] : s[j]; i[j] = mine ? i[j + 1] : i[j]; }
    s[K - 1] = mine ? -INFINITY : s[K - 1];
    i[K - 1] = mine ? INT_MAX : i[K - 1];
  }
};

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
// kMaxBlocksPerWg), its wavefronts take them round-robin.  Each wavefront streams its row blocks through a
// PRIVATE ring of LDS stages with direct global->LDS loads: one stage holds 16 rows x CHB bytes (a chunk of
// CHB/2 elements per row), one load instruction brings 1 KB that is contiguous in memory (whole 128-byte
// lines, requested once), and NSTG-1 chunks are always in flight per wavefront.  No workgroup barrier is
// needed in the loop: a ring is written and read by one wavefront only.  The 16-byte chunks of a row are
// XOR-swizzled inside the stage so that the MFMA operand reads (lane (r = lane%16, g = lane/16) reads
// elements [32 step + 8 g, +8) of row r) are bank-conflict free.  The probes of the pass (NPB blocks of 16,
// zero padded) and the inverse norms of the workgroup's rows sit in LDS too.
// Result lane layout of the 16x16 product: lane holds probe (lane%16), rows 4*(lane/16) + 0..3.
// ---------------------------------------------------------------------------------------------------
// cache policy of the bank stream (aux operand of the global->LDS load): 2 = non-temporal, the rows are used once
constexpr int kBankLoadAux = 2;
constexpr int kProbePad = 32;  // bytes added to every probe row in LDS (measured: 16 leaves 4 conflict cycles per operand read, 32 none)
constexpr int kMaxBlocksPerWg = 128;  // 2048 rows: bounds the LDS copy of the inverse norms (8 KB)
#define PC_LOOKUP_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 0xf) | (7 << 4) | (15 << 8) | ((((n) >> 4) & 3) << 14))

template <int CHB>
__device__ __forceinline__ int row_swz(int row) { return CHB >= 256 ? (row & 15) : ((row >> 1) & 7); }

// Merge of the per-lane lists of one workgroup: the four lanes that share a probe (K rounds of "best head wins and
// is popped"), then the four wavefronts through LDS; the workgroup's lists go to partial[blockIdx.x][NPB*16][KL].
template <int NPB, int KL>
__device__ __forceinline__ void merge_workgroup_lists(TopK<KL> (&best)[NPB], char *smem, Best *__restrict__ partial) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r16 = lane & 15, g = lane >> 4;
  __syncthreads();  // probes no longer needed: reuse LDS for the cross-wave step
  Best *red = (Best *)smem;  // [4 waves][NPB*16][KL]
#pragma unroll
  for (int pb = 0; pb < NPB; ++pb) {
#pragma unroll
    for (int j = 0; j < KL; ++j) {
      float s = best[pb].s[0];
      int i = best[pb].i[0];
#pragma unroll
      for (int o = 16; o < 64; o <<= 1) {
        float s2 = __shfl_xor(s, o, 64);
        int i2 = __shfl_xor(i, o, 64);
        if (better(s2, i2, s, i)) { s = s2; i = i2; }
      }
      best[pb].pop_if(i != INT_MAX && best[pb].i[0] == i);  // rows are unique: at most one lane owns the winner
      if (g == 0) red[(wave * (NPB * 16) + pb * 16 + r16) * KL + j] = Best{s, i};
    }
  }
  __syncthreads();
  if (tid < NPB * 16) {
    int head[4] = {0, 0, 0, 0};
    for (int j = 0; j < KL; ++j) {
      Best b = Best{-INFINITY, INT_MAX};
      int from = -1;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        if (head[w] >= KL) continue;
        Best o = red[(w * (NPB * 16) + tid) * KL + head[w]];
        if (o.idx != INT_MAX && better(o.s, o.idx, b.s, b.idx)) { b = o; from = w; }
      }
#pragma unroll
      for (int w = 0; w < 4; ++w) head[w] += (w == from);
      partial[((size_t)blockIdx.x * (NPB * 16) + tid) * KL + j] = b;
    }
  }
}

// Arguments of the per-row mode (K == 0): instead of the best rows per probe, the best PROBE per bank row is
// written (cache refresh, Sec. 4.1.3: does any new chunk enter a stored query's top-k?).
struct RowScan {
  const float *probe_inv;  // [n_probes] inverse norms of the probes
  const float *kth;        // [N] similarity a new chunk must exceed for row j (the row's current k-th best)
  float *best_sim;         // [N] out: best similarity over all new chunks so far
  int32_t *best_new;       // [N] out: index of that chunk
  uint8_t *stale;          // [N] out: best_sim > kth
  int p0;                  // index of this pass's first probe
  int first;               // 1: first pass (outputs are overwritten), 0: merged with the previous passes
};

template <int NPB, int CHB, int NSTG, int K>
__global__ __launch_bounds__(256) void lookup_stream_kernel(const _Float16 *__restrict__ bank,
                                                            const float *__restrict__ inv_norm, int N, int d,
                                                            const _Float16 *__restrict__ probes, int n_probes,
                                                            int per_wg, int ring_off, Best *__restrict__ partial, RowScan rs) {
  extern __shared__ __align__(16) char smem[];
  constexpr int CS = CHB / 64;           // MFMA k-steps (32 elements) per chunk
  constexpr int STG = 16 * CHB;          // bytes per stage
  constexpr int IPS = STG / 1024;        // load instructions per stage
  constexpr int LPR = CHB / 16;          // lanes (16-byte chunks) per row
  constexpr int AHEAD = NSTG - 1;
  // probe rows in LDS are padded by kProbePad = 32 bytes (a row is a multiple of 128 bytes): lane (probe r16, k-group g)
  // then reads at (32 r16 + 16 g) modulo 256.  With 16 bytes of padding -- 16 (r16 + g) modulo 256 -- the counters showed
  // four bank-conflict cycles per operand read, with 32 none
  const int row_bytes = d * 2 + kProbePad;
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

  const int chunks = d * 2 / CHB;
  char *ring = smem + ring_off + wave * (NSTG * STG);

  constexpr int KL = K > 0 ? K : 1;
  TopK<KL> best[NPB];  // this lane's best rows for probe pb*16 + r16
#pragma unroll
  for (int pb = 0; pb < NPB; ++pb) best[pb].clear();
  // per-row mode: the product is taken the other way round (probes on the M side), so a lane holds ONE row (r16) and
  // the probes pb*16 + 4g + 0..3; their inverse norms (-inf marks padding probes)
  float pinv[NPB][4];
#pragma unroll
  for (int pb = 0; pb < NPB; ++pb)
#pragma unroll
    for (int e = 0; e < 4; ++e) pinv[pb][e] = (K == 0 && pb * 16 + g * 4 + e < n_probes) ? rs.probe_inv[pb * 16 + g * 4 + e] : -INFINITY;

  // load instruction i of a stage: lane lands at stage byte 1024 i + 16 lane = (row, physical chunk)
  int ld_row[IPS], ld_col[IPS];
#pragma unroll
  for (int i = 0; i < IPS; ++i) {
    const int row = i * (1024 / CHB) + lane / LPR, pc = lane % LPR;
    ld_row[i] = row;
    ld_col[i] = (pc ^ row_swz<CHB>(row)) * 8;  // element offset of the logical chunk inside the row's chunk
  }
  auto issue = [&](int rb, int chunk, int st) __attribute__((always_inline)) {
    const _Float16 *base = bank + chunk * (CHB / 2);
#pragma unroll
    for (int i = 0; i < IPS; ++i) {
      const int row = min(rb * 16 + ld_row[i], N - 1);
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(base + (size_t)row * d + ld_col[i]),
                                       (__attribute__((address_space(3))) void *)(ring + st * STG + i * 1024), 16, 0, kBankLoadAux);
    }
  };
  // swizzled byte offsets of this lane's operand reads inside a stage
  int rd_off[CS];
#pragma unroll
  for (int s = 0; s < CS; ++s) rd_off[s] = r16 * CHB + (((4 * s + g) ^ row_swz<CHB>(r16)) * 16);

  f32x4 acc[NPB];
  auto clear = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int pb = 0; pb < NPB; ++pb) acc[pb] = f32x4{0.f, 0.f, 0.f, 0.f};
  };
  auto compute = [&](int chunk, int st) __attribute__((always_inline)) {
    const char *pbase = smem + (size_t)r16 * row_bytes + (chunk * (CHB / 2) + g * 8) * 2;
    const char *abase = ring + st * STG;
#pragma unroll
    for (int s = 0; s < CS; ++s) {
      f16x8 av = *(const f16x8 *)(abase + rd_off[s]);
#pragma unroll
      for (int pb = 0; pb < NPB; ++pb) {
        f16x8 bv = *(const f16x8 *)(pbase + (size_t)pb * 16 * row_bytes + s * 64);
        // (both operands have the same lane layout -- index lane%16, elements 8*(lane/16).. -- so swapping them
        // transposes the result: lane holds row r16 and probes 4g + 0..3)
        acc[pb] = K == 0 ? __builtin_amdgcn_mfma_f32_16x16x32_f16(bv, av, acc[pb], 0, 0, 0)
                         : __builtin_amdgcn_mfma_f32_16x16x32_f16(av, bv, acc[pb], 0, 0, 0);
      }
    }
  };
  // scale by the rows' inverse norms and keep the running best list (the lowest row wins ties)
  auto epilogue = [&](int rb) __attribute__((always_inline)) {
    if (K > 0) {
      const f32x4 inv4 = *(const f32x4 *)(inv_lds + (rb - rb_begin) * 16 + g * 4);
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int row = rb * 16 + g * 4 + r;
        const bool ok = row < N;
#pragma unroll
        for (int pb = 0; pb < NPB; ++pb) {
          const float s = acc[pb][r] * inv4[r];
          if (ok) best[pb].insert(s, row);
        }
      }
    } else {
      // best probe of row r16: this lane's probes first (ascending, so the lowest wins ties), then the four lanes
      // that hold the row
      const int row = rb * 16 + r16;
      const float inv = inv_lds[(rb - rb_begin) * 16 + r16];
      float s = -INFINITY;
      int pi = INT_MAX;
#pragma unroll
      for (int pb = 0; pb < NPB; ++pb)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float c = pinv[pb][e] == -INFINITY ? -INFINITY : acc[pb][e] * inv * pinv[pb][e];
          const int p = rs.p0 + pb * 16 + g * 4 + e;
          if (better(c, p, s, pi)) { s = c; pi = p; }
        }
#pragma unroll
      for (int o = 16; o < 64; o <<= 1) {
        const float s2 = __shfl_xor(s, o, 64);
        const int p2 = __shfl_xor(pi, o, 64);
        if (better(s2, p2, s, pi)) { s = s2; pi = p2; }
      }
      if (row < N && g == 0) {
        if (!rs.first && !better(s, pi, rs.best_sim[row], rs.best_new[row])) { s = rs.best_sim[row]; pi = rs.best_new[row]; }
        rs.best_sim[row] = s;
        rs.best_new[row] = pi;
        rs.stale[row] = s > rs.kth[row] ? 1 : 0;
      }
    }
  };
  auto advance = [&](int &rb_, int &c_) __attribute__((always_inline)) {
    if (++c_ == chunks) { c_ = 0; rb_ += 4; }
  };

  // flat pipeline over this wavefront's (row block, chunk) items.  Loads are issued unconditionally (past the
  // end they re-read the last block into a stage nobody will read), so exactly AHEAD items are outstanding
  // behind the one about to be multiplied and a partial vmcnt wait is exact.
  int rb = rb_begin + wave, c = 0;
  int prb = rb, pch = 0;
  const int rb_last = rb_end - 1;
  if (rb < rb_end) {
    int st = 0, ist = 0;
#pragma unroll
    for (int k = 0; k < AHEAD; ++k) {
      issue(min(prb, rb_last), pch, ist);
      advance(prb, pch);
      ist = ist + 1 == NSTG ? 0 : ist + 1;
    }
    clear();
    while (true) {
      issue(min(prb, rb_last), pch, ist);  // overwrites the stage multiplied in the previous iteration
      advance(prb, pch);
      ist = ist + 1 == NSTG ? 0 : ist + 1;
      PC_LOOKUP_WAIT_VMCNT(AHEAD * IPS);
      asm volatile("" ::: "memory");
      compute(c, st);
      if (c == chunks - 1) { epilogue(rb); clear(); }
      advance(rb, c);
      st = st + 1 == NSTG ? 0 : st + 1;
      if (rb >= rb_end) break;
    }
    PC_LOOKUP_WAIT_VMCNT(0);
  }

  if (K == 0) return;  // per-row mode: everything has been written
  merge_workgroup_lists<NPB, KL>(best, smem, partial);
}

// ---------------------------------------------------------------------------------------------------
// Per probe: merge the workgroup partial lists, divide by the probe's norm, compare the best with tau.
// One workgroup of four wavefronts per probe, one thread per partial list (a thread takes its first list as it
// stands -- the lists are sorted, best first -- and inserts any further ones); then k rounds of "the best head of
// all threads wins and its owner pops it".  k <= K entries are written per probe.
// ---------------------------------------------------------------------------------------------------
constexpr int kFinalizeThreads = 256;
template <int K>
__global__ __launch_bounds__(kFinalizeThreads) void lookup_finalize_kernel(const Best *__restrict__ partial, int n_partials,
                                                                           int partial_stride, const _Float16 *__restrict__ probes,
                                                                           int d, float tau, int k, int32_t *__restrict__ idx_out,
                                                                           float *__restrict__ sim_out, uint8_t *__restrict__ hit_out) {
  constexpr int NWV = kFinalizeThreads / 64;
  __shared__ float norm_part[NWV];
  __shared__ float red_s[2][NWV];
  __shared__ int red_i[2][NWV];
  const int p = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  float ss = 0.f;
  const u32x4 *src = (const u32x4 *)(probes + (size_t)p * d);
  for (int v = tid; v < d / 8; v += kFinalizeThreads) {
    f16x8 h = __builtin_bit_cast(f16x8, src[v]);
#pragma unroll
    for (int e = 0; e < 8; ++e) ss += (float)h[e] * (float)h[e];
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
  if (lane == 0) norm_part[wave] = ss;
  TopK<K> mine;
  mine.clear();
  if (tid < n_partials) {
    const Best *lst = partial + ((size_t)tid * partial_stride + p) * K;
#pragma unroll
    for (int j = 0; j < K; ++j) {
      const Best b = lst[j];
      mine.s[j] = b.idx != INT_MAX ? b.s : -INFINITY;
      mine.i[j] = b.idx;
    }
  }
  for (int w = tid + kFinalizeThreads; w < n_partials; w += kFinalizeThreads) {
    const Best *lst = partial + ((size_t)w * partial_stride + p) * K;
#pragma unroll
    for (int j = 0; j < K; ++j) {
      Best b = lst[j];
      if (b.idx != INT_MAX) mine.insert(b.s, b.idx);
    }
  }
  __syncthreads();
  float tot = 0.f;
#pragma unroll
  for (int w = 0; w < NWV; ++w) tot += norm_part[w];
  const float inv = tot > 0.f ? 1.0f / sqrtf(tot) : 0.f;
  for (int j = 0; j < k; ++j) {
    float s = mine.s[0];
    int i = mine.i[0];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      float s2 = __shfl_xor(s, o, 64);
      int i2 = __shfl_xor(i, o, 64);
      if (better(s2, i2, s, i)) { s = s2; i = i2; }
    }
    if (lane == 0) { red_s[j & 1][wave] = s; red_i[j & 1][wave] = i; }
    __syncthreads();  // (the buffer of round j is written again in round j + 2, behind the barrier of round j + 1)
    s = red_s[j & 1][0];
    i = red_i[j & 1][0];
#pragma unroll
    for (int w = 1; w < NWV; ++w) {
      const float s2 = red_s[j & 1][w];
      const int i2 = red_i[j & 1][w];
      if (better(s2, i2, s, i)) { s = s2; i = i2; }
    }
    mine.pop_if(i != INT_MAX && mine.i[0] == i);
    if (tid == 0) {
      const float sim = i == INT_MAX ? -INFINITY : s * inv;
      idx_out[(size_t)p * k + j] = i == INT_MAX ? -1 : i;
      sim_out[(size_t)p * k + j] = sim;
      if (hit_out && j == 0) hit_out[p] = sim > tau ? 1 : 0;
    }
  }
}

// ---------------------------------------------------------------------------------------------------
// Many probes at once (more than the one-pass kernels take): the scan is a matrix product E P^T and is bound by the
// matrix cores, not by the stream of the bank.  Tiles of 256 bank rows x PT probes (256, or 128 where that pads less
// and for top-k calls, whose sorted lists need the registers) per workgroup of 8 wavefronts, one workgroup per CU,
// which walks a group of consecutive bank tiles; the bank rows are the M side, so a lane holds, for ONE probe, 32 rows
// per tile, scales them by the rows' inverse norms and keeps its best (or a running sorted list of K).  A CU takes in
// at most 64 bytes per clock from L2, which a 128 x 128 tile would need for as long as its MFMAs run; at 256 x 256
// the operand bytes per flop halve.
// Wavefront (wa, wb) owns bank-row blocks 2 wa, 2 wa + 1 and probe blocks NB wb .. NB wb + NB - 1 (NB = PT / 64).
// LDS stages of 64 k-elements (128-byte rows, chunk ^= (row >> 1) & 7) in a ring of NSTG: as many as fit (two of
// 64 KB at PT = 256, three of 48 KB at PT = 128); a request has NSTG - 1 k-steps to land in.  (128-row tiles with a
// ring of five for up to 128 probes were tried: 0.104 ms against 0.097, a k-step of so little arithmetic is all
// barrier.)  One software pipeline runs over all the k-steps of all the
// workgroup's tiles: the operands of the next 16 k-elements are read from LDS while the MFMAs of the current ones
// run, and the one barrier of a k-step sits before its last quarter -- there every wavefront has read the rest of the
// current stage into registers (so the stage can be requested again, NSTG k-steps ahead) and the next stage has
// landed (its first operands are read under that last quarter's MFMAs).
// ---------------------------------------------------------------------------------------------------
constexpr int kBigRows = 256;
template <int PT>
struct BigTile {
  static constexpr int A_BYTES = kBigRows * 128, B_BYTES = PT * 128, STAGE = A_BYTES + B_BYTES;
  static constexpr int NSTG = 160 * 1024 / STAGE;
  static constexpr int LDS = NSTG * STAGE;
  static constexpr int A_PER = A_BYTES / 1024 / 4, B_PER = B_BYTES / 1024 / 4;  // request instructions per wavefront and stage
  static_assert((PT == 256 || PT == 128) && NSTG >= 2 && NSTG <= 5, "tile");
};

template <int PT, int K>
__global__ __launch_bounds__(512, 1) void lookup_big_kernel(const _Float16 *__restrict__ bank, const float *__restrict__ inv_norm,
                                                            int N, int d, const _Float16 *__restrict__ probes, int n_probes,
                                                            int p_pad, int n_groups, int p_tiles, Best *__restrict__ partial) {
  extern __shared__ __align__(16) char smem[];
  using BT = BigTile<PT>;
  constexpr int ROW = 128, RT = kBigRows, NSTG = BT::NSTG, STAGE = BT::STAGE, NA = RT / 128, NB = PT / 64;
  // the probe tiles of one bank group run next to each other on ONE XCD (workgroup ids go round-robin over the 8):
  // the group's rows come from HBM once and are re-read from that XCD's L2
  const int xcd = blockIdx.x & 7, jj = blockIdx.x >> 3;
  const int group = (jj / p_tiles) * 8 + xcd, p_tile = jj % p_tiles;
  if (group >= n_groups) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wa = wave & 3, wb = wave >> 2;
  const int l32 = lane & 31, g = lane >> 5;
  const int n_tiles = (N + RT - 1) / RT;
  const int tile_begin = (int)((long)group * n_tiles / n_groups), tile_end = (int)((long)(group + 1) * n_tiles / n_groups);
  const int m0 = p_tile * PT;
  const int nk = d / 64;

  // requests: instruction i of a half-stage fills its bytes [1024 i, 1024 i + 1024), i.e. rows 8 i .. 8 i + 7;
  // wavefronts 0-3 bring the bank rows (A_PER instructions each), 4-7 the probes (B_PER each)
  const bool loads_bank = wave < 4;
  const int per = loads_bank ? BT::A_PER : BT::B_PER;
  const int my_row = (wave & 3) * per * 8 + (lane >> 3);  // + 8 k
  const int my_chunk = lane & 7;
  const _Float16 *src[8];
  int f_tile = tile_begin, f_kt = 0;  // what the next request brings
  auto aim = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const int row = my_row + 8 * (k < per ? k : 0);
      const size_t at = loads_bank ? (size_t)min(f_tile * RT + row, N - 1) : (size_t)min(m0 + row, n_probes - 1);
      src[k] = (loads_bank ? bank : probes) + at * d + ((my_chunk ^ pc::gemm::swz128(row)) * 8);
    }
  };
  char *const dst = smem + (loads_bank ? 0 : BT::A_BYTES) + (wave & 3) * per * 1024;
  // instructions k0 .. k1 - 1 of the request for k-step (f_tile, f_kt) into ring slot `slot` (a wavefront has A_PER
  // or B_PER of them: the surplus is skipped)
  auto request_part = [&](int slot, int k0, int k1) __attribute__((always_inline)) {
    if (loads_bank) {
#pragma unroll
      for (int k = k0; k < (k1 < BT::A_PER ? k1 : BT::A_PER); ++k)
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(src[k] + f_kt * 64),
                                         (__attribute__((address_space(3))) void *)(dst + slot * STAGE + k * 1024), 16, 0, 0);
    } else {
#pragma unroll
      for (int k = k0; k < (k1 < BT::B_PER ? k1 : BT::B_PER); ++k)
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(src[k] + f_kt * 64),
                                         (__attribute__((address_space(3))) void *)(dst + slot * STAGE + k * 1024), 16, 0, 0);
    }
  };
  // on to the next k-step; past the last one the cursor stays on valid rows (requests made then land in a slot that
  // nobody reads any more)
  auto advance = [&]() __attribute__((always_inline)) {
    if (++f_kt == nk) {
      f_kt = 0;
      if (f_tile + 1 < tile_end) {
        ++f_tile;
        if (loads_bank) aim();
      }
    }
  };
  // operand reads: this lane's row inside a 32-row block is l32; k-quarter q of a stage is chunk 2 q + g
  int rd[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) rd[q] = ((2 * q + g) ^ pc::gemm::swz128(l32)) * 16;
  const int a_off = (NA * wa * 32 + l32) * ROW, b_off = BT::A_BYTES + (NB * wb * 32 + l32) * ROW;
  f16x8 oa[2][NA], ob[2][NB];  // two register sets
  auto read_ops = [&](int set, int slot, int q) __attribute__((always_inline)) {
    const char *base = smem + slot * STAGE + rd[q];
#pragma unroll
    for (int a = 0; a < NA; ++a) oa[set][a] = *(const f16x8 *)(base + a_off + a * 32 * ROW);
#pragma unroll
    for (int t = 0; t < NB; ++t) ob[set][t] = *(const f16x8 *)(base + b_off + t * 32 * ROW);
  };
  pc::f32x16 acc[NA][NB];
  auto mma_ops = [&](int set) __attribute__((always_inline)) {
#pragma unroll
    for (int t = 0; t < NB; ++t)
#pragma unroll
      for (int a = 0; a < NA; ++a) acc[a][t] = pc::gemm::mma(oa[set][a], ob[set][t], acc[a][t]);
  };
  // one MFMA, one LDS read, ... : the reads of the next quarter go out under the MFMAs of this one, and so do
  // `loads` request instructions (a CU's 64 per k-step issued in one burst hold every wavefront in the issue queue
  // for the thousand cycles the texture path needs for them)
  auto interleave = [&](int loads) __attribute__((always_inline)) {
    constexpr int READS = NA + NB, MMAS = NA * NB;
#pragma unroll
    for (int i = 0; i < (READS < MMAS ? READS : MMAS); ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      if ((i & 1) == 0 && i / 2 < loads) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
    }
    if (MMAS > READS) __builtin_amdgcn_sched_group_barrier(0x008, MMAS - READS, 0);
  };

  static_assert(K == 1 || PT == 128, "the sorted lists of a top-k call need the registers that 256-probe tiles take");
  TopK<K> best[NB];  // this lane's rows for probes m0 + (NB wb + t) * 32 + l32
#pragma unroll
  for (int t = 0; t < NB; ++t) best[t].clear();

  if (tile_begin < tile_end) {  // the first k-step, then whole requests for the next NSTG - 2 and the first part of one more
    aim();
    request_part(0, 0, 8);
    advance();
    pc::gemm::wait_vmcnt0();
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
#pragma unroll
    for (int s2 = 1; s2 < NSTG - 1; ++s2) {
      request_part(s2, 0, 8);
      advance();
    }
    request_part(NSTG - 1, 0, 3);  // (the rest of it under the first two quarters below)
    read_ops(0, 0, 0);
  }
  int slot = 0;  // ring slot of this k-step
  for (int tile = tile_begin; tile < tile_end; ++tile) {
#pragma unroll
    for (int a = 0; a < NA; ++a)
#pragma unroll
      for (int t = 0; t < NB; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[a][t][r] = 0.f;
    const int row_mine = tile * RT + NA * wa * 32 + lane;
    const float inv_mine = row_mine < N && lane < NA * 32 ? inv_norm[row_mine] : __builtin_nanf("");  // (in flight under the tile's k-steps)
    for (int kt = 0; kt < nk; ++kt) {
      const int slot_prev = slot == 0 ? NSTG - 1 : slot - 1, slot_next = slot == NSTG - 1 ? 0 : slot + 1;
      // a request was begun behind the last barrier, into the slot that k-step gave up: the rest of its instructions
      request_part(slot_prev, 3, 6);
      read_ops(1, slot, 1);
      mma_ops(0);
      interleave(3);
      request_part(slot_prev, 6, 8);
      read_ops(0, slot, 2);
      mma_ops(1);
      interleave(2);
      advance();
      read_ops(1, slot, 3);
      mma_ops(0);
      interleave(0);
      // every read of this stage is in registers and this wavefront's part of the next stage has landed: all of its
      // requests but the NSTG - 2 latest ones, which are for later k-steps
      constexpr int LEAVE_A = (NSTG - 2) * BT::A_PER, LEAVE_B = (NSTG - 2) * BT::B_PER;  // (vmcnt: bits 3:0 and 15:14)
      static_assert(LEAVE_A < 64 && LEAVE_B < 64, "vmcnt");
      if (loads_bank) __builtin_amdgcn_s_waitcnt((LEAVE_A & 0xf) | (7 << 4) | ((LEAVE_A >> 4) << 14));
      else __builtin_amdgcn_s_waitcnt((LEAVE_B & 0xf) | (7 << 4) | ((LEAVE_B >> 4) << 14));
      asm volatile("" ::: "memory");
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
      request_part(slot, 0, 3);       // the k-step NSTG ahead (past the end: see advance())
      read_ops(0, slot_next, 0);      // (past the last k-step: whatever that slot holds, never multiplied)
      mma_ops(1);
      interleave(3);
      slot = slot_next;
    }
    // cosines of this tile's rows (up to the probe's own norm, which the finalize kernel divides by)
    const int r0 = tile * RT;
    if constexpr (K == 1) {
      // Lane L of the wavefront has fetched the inverse norm of the wavefront's row L (of NA * 32) while the tile was
      // multiplied -- NaN past the end of the bank, which no comparison below ever prefers -- and a lane takes the
      // ones of its own rows from there.  Its 32 rows are visited in rising order, so "greater" alone keeps the
      // lowest row among equals, within the tile and against earlier tiles.
      float ls[NB];
      int lc[NB];
#pragma unroll
      for (int t = 0; t < NB; ++t) { ls[t] = -INFINITY; lc[t] = 0; }
#pragma unroll
      for (int a = 0; a < NA; ++a)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          float inv[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) inv[e] = __shfl(inv_mine, a * 32 + q4 * 8 + g * 4 + e, 64);
#pragma unroll
          for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int t = 0; t < NB; ++t) {
              const float v = acc[a][t][q4 * 4 + e] * inv[e];
              lc[t] = v > ls[t] ? a * 16 + q4 * 4 + e : lc[t];
              ls[t] = fmaxf(ls[t], v);
            }
          __builtin_amdgcn_sched_barrier(0);  // (four exchanged norms live at a time, not thirty-two)
        }
#pragma unroll
      for (int t = 0; t < NB; ++t) {
        const int row = r0 + (NA * wa + (lc[t] >> 4)) * 32 + ((lc[t] >> 2) & 3) * 8 + g * 4 + (lc[t] & 3);
        const bool up = ls[t] > best[t].s[0];
        best[t].s[0] = up ? ls[t] : best[t].s[0];
        best[t].i[0] = up ? row : best[t].i[0];
      }
    } else {
      // the k best: the same exchanged norms, every scaled product offered to the lane's sorted list (an insertion
      // happens only when it beats the list's last entry; NaN, past the end of the bank, never does)
#pragma unroll
      for (int a = 0; a < NA; ++a)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          float inv[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) inv[e] = __shfl(inv_mine, a * 32 + q4 * 8 + g * 4 + e, 64);
#pragma unroll
          for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int t = 0; t < NB; ++t)
              best[t].insert(acc[a][t][q4 * 4 + e] * inv[e], r0 + (NA * wa + a) * 32 + q4 * 8 + g * 4 + e);
          __builtin_amdgcn_sched_barrier(0);
        }
    }
  }
  // the two lanes of a probe, then the four wavefronts (wa) that hold other rows of the same probes: K rounds of
  // "the best head wins and is popped" between the lanes, then a merge of the four sorted lists
  __builtin_amdgcn_s_waitcnt(7 << 4);
  __syncthreads();
  Best *red = (Best *)smem;  // [wb][wa][NB * 32][K]
#pragma unroll
  for (int t = 0; t < NB; ++t) {
#pragma unroll
    for (int j = 0; j < K; ++j) {
      float s = best[t].s[0];
      int i = best[t].i[0];
      const float s2 = __shfl_xor(s, 32, 64);
      const int i2 = __shfl_xor(i, 32, 64);
      if (better(s2, i2, s, i)) { s = s2; i = i2; }
      if constexpr (K > 1) best[t].pop_if(i != INT_MAX && best[t].i[0] == i);
      if (g == 0) red[((wb * 4 + wa) * (NB * 32) + t * 32 + l32) * K + j] = Best{s, i};
    }
  }
  __syncthreads();
  if (tid < PT) {  // one thread per probe of the tile: probe wb2 * NB * 32 + within
    const int wb2 = tid / (NB * 32), within = tid % (NB * 32);
    const Best *lst[4];
    int head[4];
#pragma unroll
    for (int w = 0; w < 4; ++w) { lst[w] = red + ((wb2 * 4 + w) * (NB * 32) + within) * K; head[w] = 0; }
    Best *out = partial + ((size_t)group * p_pad + m0 + tid) * K;
    for (int j = 0; j < K; ++j) {
      Best b{-INFINITY, INT_MAX};
      int from = 0;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const Best c = head[w] < K ? lst[w][head[w]] : Best{-INFINITY, INT_MAX};
        if (c.idx != INT_MAX && (b.idx == INT_MAX || better(c.s, c.idx, b.s, b.idx))) { b = c; from = w; }
      }
      out[j] = b;
#pragma unroll
      for (int w = 0; w < 4; ++w) head[w] += (w == from && b.idx != INT_MAX);
    }
  }
}

// ---------------------------------------------------------------------------------------------------
// Up to 128 probes in one pass of the bank (embedding widths of 512, 768 and 1024 elements).
// One workgroup per CU; wavefront w keeps ITS 32 probes in registers as the N-side operands of the 32x32x16 product
// (d/4 registers per lane: one wavefront per SIMD), and all four wavefronts multiply the same 32-row blocks of the
// bank, which stream through a ring of LDS stages shared by the workgroup (32 rows x 512 bytes per stage; every
// load instruction brings two contiguous 512-byte runs; NSTG - 1 stages in flight).  One barrier per stage: it
// publishes the stage that has landed and retires the one just multiplied.  A lane ends up with 16 rows of one
// probe per block, scales them by the rows' inverse norms and keeps a running sorted list, as in the kernel above.
// ---------------------------------------------------------------------------------------------------
constexpr int kWideProbes = 128;
constexpr int kWideStages = 8;
constexpr int kWideChunk = 512;             // bytes of a row per stage
constexpr int kWideMaxBlocksPerWg = 192;    // 6144 rows: bounds the LDS copy of the inverse norms (24 KB)

template <int D_EMB, int K>
__global__ __launch_bounds__(256, 1) void lookup_wide_kernel(const _Float16 *__restrict__ bank, const float *__restrict__ inv_norm,
                                                             int N, const _Float16 *__restrict__ probes, int n_probes, int per_wg,
                                                             Best *__restrict__ partial) {
  extern __shared__ __align__(16) char smem[];
  constexpr int CHB = kWideChunk, NSTG = kWideStages;
  constexpr int CHUNKS = D_EMB * 2 / CHB;  // stages per row block
  constexpr int CS = CHB / 32;             // MFMA k-steps (16 elements) per stage
  constexpr int STG = 32 * CHB;            // bytes per stage
  constexpr int IPS = STG / 1024 / 4;      // load instructions per stage and wavefront
  static_assert(D_EMB * 2 % CHB == 0, "row must be a whole number of chunks");
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, g2 = lane >> 5;
  const int n_blocks = (N + 31) / 32;
  const int rb_begin = blockIdx.x * per_wg, rb_end = min(n_blocks, rb_begin + per_wg);

  // inverse norms of this workgroup's rows (zero beyond N), then the ring
  float *inv_lds = (float *)smem;
  char *ring = smem + kWideMaxBlocksPerWg * 32 * sizeof(float);
  for (int r = tid; r < per_wg * 32; r += 256) {
    const int row = rb_begin * 32 + r;
    inv_lds[r] = row < N ? inv_norm[row] : 0.f;
  }
  // this lane's probe: elements [16 ks + 8 g2, +8) for every k-step (zero for a padding probe)
  f16x8 pq[D_EMB / 16];
  {
    const int p = wave * 32 + l32;
    const u32x4 *src = (const u32x4 *)(probes + (size_t)min(p, n_probes - 1) * D_EMB);
#pragma unroll
    for (int ks = 0; ks < D_EMB / 16; ++ks) {
      u32x4 raw = src[2 * ks + g2];
      if (p >= n_probes) raw = u32x4{0, 0, 0, 0};
      pq[ks] = __builtin_bit_cast(f16x8, raw);
    }
  }
  // (the probes' loads must not be counted by the ring's partial waits below)
#pragma unroll
  for (int ks = 0; ks < D_EMB / 16; ++ks) asm volatile("" : "+v"(pq[ks]));
  PC_LOOKUP_WAIT_VMCNT(0);
  __syncthreads();

  // load instruction i of a stage (i = wave + 4 k): stage bytes [1024 i, +1024) = rows 2i, 2i+1
  int ld_row[IPS], ld_col[IPS];
#pragma unroll
  for (int k = 0; k < IPS; ++k) {
    const int row = (wave + 4 * k) * 2 + (lane >> 5), pc = lane & 31;
    ld_row[k] = row;
    ld_col[k] = (pc ^ (row & 15)) * 8;  // element offset of the logical 16-byte chunk this lane fetches
  }
  auto issue = [&](int rb, int chunk, int st) __attribute__((always_inline)) {
    const _Float16 *base = bank + chunk * (CHB / 2);
#pragma unroll
    for (int k = 0; k < IPS; ++k) {
      const int row = min(rb * 32 + ld_row[k], N - 1);
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(base + (size_t)row * D_EMB + ld_col[k]),
                                       (__attribute__((address_space(3))) void *)(ring + st * STG + (wave + 4 * k) * 1024), 16, 0, kBankLoadAux);
    }
  };
  int rd_off[CS];  // swizzled byte offsets of this lane's operand reads inside a stage
#pragma unroll
  for (int s = 0; s < CS; ++s) rd_off[s] = l32 * CHB + (((2 * s + g2) ^ (l32 & 15)) * 16);

  TopK<K> best;
  best.clear();
  const int rb_last = rb_end - 1;
  if (rb_begin < rb_end) {
    // flat sequence of (row block, chunk) items; loads go out unconditionally (past the end they repeat the last
    // block into a stage nobody reads), so the count of loads in flight is the same at every wait
    int prb = rb_begin, pch = 0, ist = 0, st = 0;
    auto advance = [&](int &rb_, int &c_) __attribute__((always_inline)) {
      if (++c_ == CHUNKS) { c_ = 0; ++rb_; }
    };
#pragma unroll
    for (int k = 0; k < NSTG - 1; ++k) {
      issue(min(prb, rb_last), pch, ist);
      advance(prb, pch);
      ist = ist + 1 == NSTG ? 0 : ist + 1;
    }
    for (int rb = rb_begin; rb < rb_end; ++rb) {
      pc::f32x16 acc[2];  // two accumulation chains: an MFMA does not wait for the one before it
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[a][r] = 0.f;
#pragma unroll
      for (int c = 0; c < CHUNKS; ++c) {
        // the oldest stage in flight has landed (mine), then (barrier) everyone's; the barrier also says that the
        // stage multiplied last is free for the next load
        PC_LOOKUP_WAIT_VMCNT((NSTG - 2) * IPS);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        issue(min(prb, rb_last), pch, ist);
        advance(prb, pch);
        ist = ist + 1 == NSTG ? 0 : ist + 1;
        // all of the stage's operands are asked for before its first MFMA (left to itself the compiler reads one
        // operand, waits, multiplies: one LDS latency per MFMA instead of one per stage)
        const char *abase = ring + st * STG;
        f16x8 av[CS];
#pragma unroll
        for (int s = 0; s < CS; ++s) av[s] = *(const f16x8 *)(abase + rd_off[s]);
#pragma unroll
        for (int s = 0; s < CS; ++s) acc[s & 1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(av[s], pq[c * CS + s], acc[s & 1], 0, 0, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, CS, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, CS, 0);
        st = st + 1 == NSTG ? 0 : st + 1;
      }
      // element r of the product: row (r/4)*8 + 4*g2 + r%4 of the block, probe wave*32 + l32
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int rin = q4 * 8 + g2 * 4;
        const f32x4 inv4 = *(const f32x4 *)(inv_lds + (rb - rb_begin) * 32 + rin);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int row = rb * 32 + rin + e;
          if (row < N) best.insert((acc[0][q4 * 4 + e] + acc[1][q4 * 4 + e]) * inv4[e], row);
        }
      }
    }
    PC_LOOKUP_WAIT_VMCNT(0);
  }
  // the two lanes of a probe hold different rows: merge (K rounds of "best head wins and is popped")
  Best *out = partial + ((size_t)blockIdx.x * kWideProbes + wave * 32 + l32) * K;
#pragma unroll
  for (int j = 0; j < K; ++j) {
    float s = best.s[0];
    int i = best.i[0];
    const float s2 = __shfl_xor(s, 32, 64);
    const int i2 = __shfl_xor(i, 32, 64);
    if (better(s2, i2, s, i)) { s = s2; i = i2; }
    best.pop_if(i != INT_MAX && best.i[0] == i);
    if (g2 == 0) out[j] = Best{s, i};
  }
}

// inverse L2 norms of n embedding rows (0 for a zero row); one wavefront per row
__global__ __launch_bounds__(256) void inv_norm_kernel(const _Float16 *__restrict__ src, float *__restrict__ inv_norm, int n, int d) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= n) return;
  const u32x4 *s = (const u32x4 *)(src + (size_t)row * d);
  float ss = 0.f;
  for (int v = lane; v < d / 8; v += 64) {
    f16x8 h = __builtin_bit_cast(f16x8, s[v]);
#pragma unroll
    for (int e = 0; e < 8; ++e) ss += (float)h[e] * (float)h[e];
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
  if (lane == 0) inv_norm[row] = ss > 0.f ? 1.0f / sqrtf(ss) : 0.f;
}

__global__ void lookup_empty_kernel(int n_out, int n_probes, int32_t *idx_out, float *sim_out, uint8_t *hit_out) {
  int p = blockIdx.x * blockDim.x + threadIdx.x;
  if (p < n_out) { idx_out[p] = -1; sim_out[p] = -INFINITY; }
  if (hit_out && p < n_probes) hit_out[p] = 0;
}

constexpr int kPassProbes = 32;

// LDS bytes of one workgroup: probes, inverse norms, then (1 KB aligned) the four wavefront rings.
constexpr size_t kMaxLds = 160 * 1024;
struct StreamShape {
  int grid, per_wg, nstg, chb, ring_off;
  size_t lds;
};
StreamShape stream_shape(const percache_ctx *ctx, int npb, int N) {
  const int d = ctx->cfg.emb_dim;
  StreamShape s;
  s.chb = d * 2 % 512 == 0 ? 512 : d * 2 % 256 == 0 ? 256 : 128;  // widest chunk that divides a row
  const int n_blocks = (N + 15) / 16;
  s.grid = ctx->n_cu;  // the rings allow one workgroup per CU
  const int need = (n_blocks + 3) / 4;  // at least one block per wavefront
  if (s.grid > need) s.grid = need > 0 ? need : 1;
  s.per_wg = (n_blocks + s.grid - 1) / s.grid;
  if (s.per_wg > kMaxBlocksPerWg) {
    s.per_wg = kMaxBlocksPerWg;
    s.grid = (n_blocks + s.per_wg - 1) / s.per_wg;
  }
  size_t head = (size_t)npb * 16 * (d * 2 + kProbePad) + (size_t)s.per_wg * 16 * sizeof(float);
  s.ring_off = (int)((head + 1023) / 1024 * 1024);
  // three stages per wavefront for a single probe block if they fit beside the probes, else two
  s.nstg = npb == 1 && s.ring_off + (size_t)4 * 3 * 16 * s.chb <= kMaxLds ? 3 : 2;
  s.lds = s.ring_off + (size_t)4 * s.nstg * 16 * s.chb;
  return s;
}
int max_stream_grid(const percache_ctx *ctx) {
  int by_rows = (ctx->cfg.bank_capacity / 16 + kMaxBlocksPerWg) / kMaxBlocksPerWg;
  return by_rows > ctx->n_cu ? by_rows : ctx->n_cu;
}

constexpr int kMaxTopK = 8;
constexpr int kBatchedFrom = 32;  // more probes than one streaming pass takes: the 128-probe pass or the matrix-product kernel
constexpr int kWideUpTo = 128;    // one such pass; beyond it the matrix-product kernel is the faster one

// Launch shape of the 256-row kernel: probe tiles x groups of consecutive 256-row bank tiles, one workgroup per CU (a
// multiple of 8 groups, so that a group's probe tiles share an XCD), every group at least one tile.
struct BigShape {
  int p_tiles, groups;
};
BigShape big_shape(int n_cu, int N, int n_probes, int pt) {
  BigShape b;
  b.p_tiles = (n_probes + pt - 1) / pt;
  const int n_tiles = (N + kBigRows - 1) / kBigRows;
  b.groups = n_cu / b.p_tiles / 8 * 8;
  if (b.groups < 8) b.groups = 8;
  if (b.groups > n_tiles) b.groups = n_tiles;
  return b;
}
// whether 256-probe tiles are filled well enough to beat 128-probe ones (at most a third of padding)
bool big_tiles_pay(int n_probes) {
  if (n_probes <= kWideUpTo) return false;
  const long padded = (long)(n_probes + 255) / 256 * 256;
  return padded * 3 <= (long)n_probes * 4;
}

template <int NPB, int CHB, int NSTG, int K>
pc_status launch_stream(percache_ctx *ctx, const StreamShape &sh, hipStream_t st, int N, int d, const _Float16 *pp, int np,
                        Best *partial, const RowScan &rs) {
  static bool big_lds_set = false;  // dynamic LDS above 64 KB must be opted into once per kernel
  if (!big_lds_set) {
    PC_HIP(ctx, hipFuncSetAttribute((const void *)lookup_stream_kernel<NPB, CHB, NSTG, K>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kMaxLds));
    big_lds_set = true;
  }
  hipLaunchKernelGGL((lookup_stream_kernel<NPB, CHB, NSTG, K>), dim3(sh.grid), dim3(256), sh.lds, st, ctx->bank, ctx->bank_inv, N, d,
                     pp, np, sh.per_wg, sh.ring_off, partial, rs);
  return PC_OK;
}

template <int K>
pc_status launch_pass(percache_ctx *ctx, const StreamShape &sh, int npb, hipStream_t st, int N, int d, const _Float16 *pp, int np,
                      Best *partial, const RowScan &rs = RowScan{}) {
  if (npb == 1 && sh.nstg == 3)
    return sh.chb == 128   ? launch_stream<1, 128, 3, K>(ctx, sh, st, N, d, pp, np, partial, rs)
           : sh.chb == 256 ? launch_stream<1, 256, 3, K>(ctx, sh, st, N, d, pp, np, partial, rs)
                           : launch_stream<1, 512, 3, K>(ctx, sh, st, N, d, pp, np, partial, rs);
  if (npb == 1) return launch_stream<1, 512, 2, K>(ctx, sh, st, N, d, pp, np, partial, rs);  // only the widest rows (512-byte chunks) get here
  return sh.chb == 128   ? launch_stream<2, 128, 2, K>(ctx, sh, st, N, d, pp, np, partial, rs)
         : sh.chb == 256 ? launch_stream<2, 256, 2, K>(ctx, sh, st, N, d, pp, np, partial, rs)
                         : launch_stream<2, 512, 2, K>(ctx, sh, st, N, d, pp, np, partial, rs);
}

// k best rows per probe (k == 1: the query-level match with its hit flag; hit_out may be null otherwise)
pc_status run_lookup(percache_ctx *ctx, const void *probes_dev, int32_t n_probes, float tau, int k, int32_t *idx_out_dev,
                     float *sim_out_dev, uint8_t *hit_out_dev, void *workspace_dev, size_t workspace_bytes, void *stream) {
  if (!ctx) return PC_EINVAL;
  const percache_config &c = ctx->cfg;
  if (c.bank_capacity <= 0) return pc::fail(ctx, PC_ESHAPE, "context was created without a bank");
  if (n_probes < 0) return pc::fail(ctx, PC_EINVAL, "n_probes is negative");
  if (k < 1 || k > kMaxTopK) return pc::fail(ctx, PC_ESHAPE, "k = %d outside [1,%d]", k, kMaxTopK);
  if (n_probes == 0) return PC_OK;
  if (!probes_dev || !idx_out_dev || !sim_out_dev || (k == 1 && !hit_out_dev)) return pc::fail(ctx, PC_EINVAL, "NULL probe or output pointer");
  if ((uintptr_t)probes_dev % 16) return pc::fail(ctx, PC_EINVAL, "probes_dev must be 16-byte aligned");
  if (!(tau == tau)) return pc::fail(ctx, PC_EINVAL, "tau is NaN");
  hipStream_t st = (hipStream_t)stream;
  const int N = ctx->bank_size, d = c.emb_dim;
  if (N == 0) {
    const int n_out = n_probes * k;
    hipLaunchKernelGGL(lookup_empty_kernel, dim3((n_out + 255) / 256), dim3(256), 0, st, n_out, n_probes, idx_out_dev, sim_out_dev, hit_out_dev);
    PC_HIP(ctx, hipGetLastError());
    return PC_OK;
  }
  const size_t need = percache_lookup_workspace_bytes(ctx, n_probes);
  if (!workspace_dev || workspace_bytes < need) return pc::fail(ctx, PC_ENOMEM, "lookup workspace has %zu bytes, need %zu", workspace_bytes, need);
  if ((uintptr_t)workspace_dev % 16) return pc::fail(ctx, PC_EINVAL, "workspace must be 16-byte aligned");
  Best *partial = (Best *)workspace_dev;
  const _Float16 *probes = (const _Float16 *)probes_dev;
  if (n_probes > kBatchedFrom && n_probes <= kWideUpTo && (d == 512 || d == 768 || d == 1024)) {
    // up to 128 probes: one pass of the bank
    const int n_blocks = (N + 31) / 32;
    int grid = ctx->n_cu < n_blocks ? ctx->n_cu : n_blocks;
    int per_wg = (n_blocks + grid - 1) / grid;
    if (per_wg > kWideMaxBlocksPerWg) { per_wg = kWideMaxBlocksPerWg; grid = (n_blocks + per_wg - 1) / per_wg; }
    const size_t lds = (size_t)kWideMaxBlocksPerWg * 32 * sizeof(float) + (size_t)kWideStages * 32 * kWideChunk;
#define PC_WIDE(DD, KK)                                                                                               \
  do {                                                                                                                \
    PC_HIP(ctx, hipFuncSetAttribute((const void *)lookup_wide_kernel<DD, KK>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)); \
    hipLaunchKernelGGL((lookup_wide_kernel<DD, KK>), dim3(grid), dim3(256), lds, st, ctx->bank, ctx->bank_inv, N, pp, np, per_wg, partial); \
  } while (0)
    for (int p0 = 0; p0 < n_probes; p0 += kWideProbes) {
      const int np = n_probes - p0 < kWideProbes ? n_probes - p0 : kWideProbes;
      const _Float16 *pp = probes + (size_t)p0 * d;
      pc::prof_begin(ctx, PC_KERNEL_LOOKUP, st);
      if (k == 1) {
        if (d == 512) PC_WIDE(512, 1); else if (d == 768) PC_WIDE(768, 1); else PC_WIDE(1024, 1);
      } else {
        if (d == 512) PC_WIDE(512, kMaxTopK); else if (d == 768) PC_WIDE(768, kMaxTopK); else PC_WIDE(1024, kMaxTopK);
      }
      pc::prof_end(ctx, PC_KERNEL_LOOKUP, st);
      PC_HIP(ctx, hipGetLastError());
      uint8_t *hit = hit_out_dev ? hit_out_dev + p0 : nullptr;
      if (k == 1)
        hipLaunchKernelGGL(lookup_finalize_kernel<1>, dim3(np), dim3(kFinalizeThreads), 0, st, partial, grid, kWideProbes, pp, d, tau, 1,
                           idx_out_dev + p0, sim_out_dev + p0, hit);
      else
        hipLaunchKernelGGL(lookup_finalize_kernel<kMaxTopK>, dim3(np), dim3(kFinalizeThreads), 0, st, partial, grid, kWideProbes, pp, d, tau, k,
                           idx_out_dev + (size_t)p0 * k, sim_out_dev + (size_t)p0 * k, hit);
      PC_HIP(ctx, hipGetLastError());
    }
#undef PC_WIDE
    return PC_OK;
  }
  if (n_probes > kBatchedFrom) {  // (d is a multiple of 64: percache_create checks it)
    // many probes: the matrix-core product on 256-row tiles, one workgroup per CU; 256-probe tiles where the probes
    // fill them to three quarters (best match only: a top-k call's lists need their registers), else 128-probe tiles
    const int pt = k == 1 && big_tiles_pay(n_probes) ? 256 : 128;
    const BigShape bg = big_shape(ctx->n_cu, N, n_probes, pt);
    static bool big_lds_set = false;  // dynamic LDS above 64 KB must be opted into once
    if (!big_lds_set) {
      PC_HIP(ctx, hipFuncSetAttribute((const void *)lookup_big_kernel<256, 1>, hipFuncAttributeMaxDynamicSharedMemorySize, BigTile<256>::LDS));
      PC_HIP(ctx, hipFuncSetAttribute((const void *)lookup_big_kernel<128, 1>, hipFuncAttributeMaxDynamicSharedMemorySize, BigTile<128>::LDS));
      PC_HIP(ctx, hipFuncSetAttribute((const void *)lookup_big_kernel<128, kMaxTopK>, hipFuncAttributeMaxDynamicSharedMemorySize, BigTile<128>::LDS));
      big_lds_set = true;
    }
    const dim3 grid((unsigned)((bg.groups + 7) / 8 * 8 * bg.p_tiles));
    pc::prof_begin(ctx, PC_KERNEL_LOOKUP, st);
#define PC_BIG(PP, KK)                                                                                                 \
  hipLaunchKernelGGL((lookup_big_kernel<PP, KK>), grid, dim3(512), (BigTile<PP>::LDS), st, ctx->bank, ctx->bank_inv, N, d, probes, n_probes, \
                     bg.p_tiles * pt, bg.groups, bg.p_tiles, partial)
    if (k > 1) PC_BIG(128, kMaxTopK); else if (pt == 256) PC_BIG(256, 1); else PC_BIG(128, 1);
#undef PC_BIG
    pc::prof_end(ctx, PC_KERNEL_LOOKUP, st);
    PC_HIP(ctx, hipGetLastError());
    if (k == 1)
      hipLaunchKernelGGL(lookup_finalize_kernel<1>, dim3(n_probes), dim3(kFinalizeThreads), 0, st, partial, bg.groups, bg.p_tiles * pt, probes, d, tau, 1,
                         idx_out_dev, sim_out_dev, hit_out_dev);
    else
      hipLaunchKernelGGL(lookup_finalize_kernel<kMaxTopK>, dim3(n_probes), dim3(kFinalizeThreads), 0, st, partial, bg.groups, bg.p_tiles * pt, probes, d,
                         tau, k, idx_out_dev, sim_out_dev, hit_out_dev);
    PC_HIP(ctx, hipGetLastError());
    return PC_OK;
  }
  // two probe blocks per pass unless their LDS copy leaves no room for the rings (very wide embeddings)
  const int pass_probes = stream_shape(ctx, 2, N).lds <= kMaxLds ? kPassProbes : 16;
  {  // every pass shape of this call is checked before the first pass is enqueued
    const size_t lds1 = stream_shape(ctx, 1, N).lds;
    if (lds1 > kMaxLds) return pc::fail(ctx, PC_ESHAPE, "emb_dim %d needs %zu bytes of LDS per workgroup", d, lds1);
  }
  for (int p0 = 0; p0 < n_probes; p0 += pass_probes) {
    int np = n_probes - p0 < pass_probes ? n_probes - p0 : pass_probes;
    int npb = np <= 16 ? 1 : 2;
    StreamShape sh = stream_shape(ctx, npb, N);
    const _Float16 *pp = probes + (size_t)p0 * d;
    pc::prof_begin(ctx, PC_KERNEL_LOOKUP, st);
    pc_status ls = k == 1 ? launch_pass<1>(ctx, sh, npb, st, N, d, pp, np, partial) : launch_pass<kMaxTopK>(ctx, sh, npb, st, N, d, pp, np, partial);
    if (ls != PC_OK) return ls;
    pc::prof_end(ctx, PC_KERNEL_LOOKUP, st);
    PC_HIP(ctx, hipGetLastError());
    uint8_t *hit = hit_out_dev ? hit_out_dev + p0 : nullptr;
    if (k == 1)
      hipLaunchKernelGGL(lookup_finalize_kernel<1>, dim3(np), dim3(kFinalizeThreads), 0, st, partial, sh.grid, npb * 16, pp, d, tau, 1,
                         idx_out_dev + p0, sim_out_dev + p0, hit);
    else
      hipLaunchKernelGGL(lookup_finalize_kernel<kMaxTopK>, dim3(np), dim3(kFinalizeThreads), 0, st, partial, sh.grid, npb * 16, pp, d, tau, k,
                         idx_out_dev + (size_t)p0 * k, sim_out_dev + (size_t)p0 * k, hit);
    PC_HIP(ctx, hipGetLastError());
  }
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
  size_t lists = (size_t)max_stream_grid(ctx) * kPassProbes;
  if (n_probes > kBatchedFrom) {
    // the 256-row kernel: groups * p_tiles <= max(n_cu, 8 p_tiles) workgroups of at most 256 lists
    const size_t p_big = ((size_t)n_probes + 127) / 128;
    const size_t big = ((size_t)ctx->n_cu > 8 * p_big ? (size_t)ctx->n_cu : 8 * p_big) * 256;
    if (big > lists) lists = big;
    // the 128-probe pass: one list per workgroup and probe
    const size_t wide_grid = (size_t)ctx->cfg.bank_capacity / (32 * kWideMaxBlocksPerWg) + 1;
    const size_t wide = (wide_grid > (size_t)ctx->n_cu ? wide_grid : (size_t)ctx->n_cu) * kWideProbes;
    if (wide > lists) lists = wide;
  }
  return pc::align_up(lists * kMaxTopK * sizeof(Best));
}

pc_status percache_lookup(percache_ctx *ctx, const void *probes_dev, int32_t n_probes, float tau, int32_t *idx_out_dev,
                          float *sim_out_dev, uint8_t *hit_out_dev, void *workspace_dev, size_t workspace_bytes,
                          void *stream) {
  return run_lookup(ctx, probes_dev, n_probes, tau, 1, idx_out_dev, sim_out_dev, hit_out_dev, workspace_dev, workspace_bytes, stream);
}

pc_status percache_lookup_noalloc(percache_ctx *ctx, const void *probes_dev, int32_t n_probes, float tau,
                                  int32_t *idx_out_dev, float *sim_out_dev, uint8_t *hit_out_dev, void *stream) {
  if (!ctx) return PC_EINVAL;
  if (n_probes > kPassProbes)
    return pc::fail(ctx, PC_ESHAPE, "percache_lookup_noalloc takes at most %d probes per call, got %d", kPassProbes, n_probes);
  const size_t need = percache_lookup_workspace_bytes(ctx, n_probes < 0 ? 0 : n_probes);
  if (need > pc::kStaticScratchBytes)
    return pc::fail(ctx, PC_ESHAPE, "a bank of %d rows needs %zu bytes of scratch, the library's static scratch holds %zu",
                    ctx->cfg.bank_capacity, need, pc::kStaticScratchBytes);
  if (!ctx->static_scratch) return pc::fail(ctx, PC_EHIP, "static scratch was not resolved on this device");
  // nothing in the scratch has to start at zero: every workgroup of a pass writes all of its lists before the
  // finalize kernel (next on the stream) reads exactly those
  return run_lookup(ctx, probes_dev, n_probes, tau, 1, idx_out_dev, sim_out_dev, hit_out_dev, ctx->static_scratch,
                    pc::kStaticScratchBytes, stream);
}

pc_status percache_bank_refresh_scan(percache_ctx *ctx, const void *new_emb_dev, int32_t n_new, const float *kth_sim_dev,
                                     float *best_sim_out_dev, int32_t *best_new_out_dev, uint8_t *stale_out_dev,
                                     void *workspace_dev, size_t workspace_bytes, void *stream) {
  if (!ctx) return PC_EINVAL;
  const percache_config &c = ctx->cfg;
  if (c.bank_capacity <= 0) return pc::fail(ctx, PC_ESHAPE, "context was created without a bank");
  if (n_new < 1) return pc::fail(ctx, PC_EINVAL, "n_new must be positive");
  if (!new_emb_dev || !kth_sim_dev || !best_sim_out_dev || !best_new_out_dev || !stale_out_dev) return pc::fail(ctx, PC_EINVAL, "NULL pointer");
  if ((uintptr_t)new_emb_dev % 16) return pc::fail(ctx, PC_EINVAL, "new_emb_dev must be 16-byte aligned");
  const int N = ctx->bank_size, d = c.emb_dim;
  if (N == 0) return PC_OK;  // nothing to mark
  const size_t need = percache_lookup_workspace_bytes(ctx, n_new);
  if (!workspace_dev || workspace_bytes < need || (size_t)n_new * sizeof(float) > need)
    return pc::fail(ctx, PC_ENOMEM, "workspace has %zu bytes, need %zu (and at most %zu new rows per call)", workspace_bytes, need, need / sizeof(float));
  if ((uintptr_t)workspace_dev % 16) return pc::fail(ctx, PC_EINVAL, "workspace must be 16-byte aligned");
  {
    const size_t lds1 = stream_shape(ctx, 1, N).lds;
    if (lds1 > kMaxLds) return pc::fail(ctx, PC_ESHAPE, "emb_dim %d needs %zu bytes of LDS per workgroup", d, lds1);
  }
  hipStream_t st = (hipStream_t)stream;
  float *probe_inv = (float *)workspace_dev;
  const _Float16 *probes = (const _Float16 *)new_emb_dev;
  hipLaunchKernelGGL(inv_norm_kernel, dim3((n_new + 3) / 4), dim3(256), 0, st, probes, probe_inv, n_new, d);
  PC_HIP(ctx, hipGetLastError());
  const int pass_probes = stream_shape(ctx, 2, N).lds <= kMaxLds ? kPassProbes : 16;
  for (int p0 = 0; p0 < n_new; p0 += pass_probes) {
    const int np = n_new - p0 < pass_probes ? n_new - p0 : pass_probes;
    const int npb = np <= 16 ? 1 : 2;
    StreamShape sh = stream_shape(ctx, npb, N);
    RowScan rs{probe_inv + p0, kth_sim_dev, best_sim_out_dev, best_new_out_dev, stale_out_dev, p0, p0 == 0 ? 1 : 0};
    pc_status ls = launch_pass<0>(ctx, sh, npb, st, N, d, probes + (size_t)p0 * d, np, nullptr, rs);
    if (ls != PC_OK) return ls;
    PC_HIP(ctx, hipGetLastError());
  }
  return PC_OK;
}

pc_status percache_lookup_topk(percache_ctx *ctx, const void *probes_dev, int32_t n_probes, int32_t k, int32_t *idx_out_dev,
                               float *sim_out_dev, void *workspace_dev, size_t workspace_bytes, void *stream) {
  return run_lookup(ctx, probes_dev, n_probes, 0.f, k, idx_out_dev, sim_out_dev, nullptr, workspace_dev, workspace_bytes, stream);
}

}  // extern "C"
