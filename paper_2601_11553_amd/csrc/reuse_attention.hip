// Attention of the fresh rows over [cached chunk K/V gathered by slot id ; fresh K/V] (Sec. 4.2.2,
// App. B.1: the loaded tensors are put in front of the projected ones along the sequence axis and the
// attention module then proceeds as usual).  The concatenation is never materialised: the kernel walks
// the query's chunk list, streams each (slot, kv head) run of the store tile by tile through LDS, and
// finishes with the fresh keys under the causal mask.
//
// Shape of the computation (64-wide wavefronts, bf16 32x32x16 MFMA, fp32 softmax state):
//   - the G = Hq/Hkv query heads of one kv head are stacked: R = G*T_f rows share every K/V tile;
//   - a workgroup of 4 or 8 wavefronts owns 128 or 256 rows, a wavefront 32 rows, and loops over 64-key tiles;
//   - scores are computed transposed, S^T = K Q^T, so that a lane's 32 accumulators all belong to ONE
//     query row: the row max/sum are lane-local plus a single exchange with lane+32, and the bf16
//     probabilities are already in the B-operand layout of O^T += V^T P^T (no LDS round trip for P);
//   - V is kept in the store (and handed over for the fresh part) as 64-key blocks [D][64] whose key
//     order inside each group of 16 is the order the score accumulators deliver them, so K and V tiles
//     are both staged with direct global->LDS loads (no registers, no LDS store instructions) and every
//     MFMA operand is one 16-byte LDS read from an XOR-swizzled, conflict-free layout;
//   - the reference exponent is only refreshed when the sum of a lane's 32 probabilities of a tile exceeds
//     32 * 2^8 (so a single probability stays below 2^13, harmless in bf16/fp32), so the rescale of the
//     output accumulators is almost never run;
//   - the key axis can be partitioned over workgroups (split-KV); partial (max, sum, output) triples are
//     merged by a small second kernel with the usual log-sum-exp rule;
//   - workgroups that stream the same K/V run are placed on the same XCD (workgroup ids go round-robin
//     over the 8 XCDs), so the run is fetched into one L2 only.
#include "percache_internal.hpp"

namespace {
using pc::bf16x8;
using pc::f32x16;
using pc::kKvTile;
using pc::kTblHeader;
using pc::u32x4;

constexpr int TK = kKvTile;  // keys per tile
constexpr int kKvAux = 2;   // cache policy of the K/V tile loads (aux operand): 2 = non-temporal
constexpr float kLazy = 8.f; // log2 slack before the reference exponent is refreshed
constexpr float kSumLimit = 32.f * 256.f;  // 32 probabilities of a lane and tile, each at most 2^kLazy

// LDS stage = one K tile [TK][D] followed by one V block [D][TK], both unpadded (they are filled by
// direct global->LDS loads, which write 1 KB per wavefront instruction contiguously).  Bank conflicts are
// avoided by an XOR swizzle of the 16-byte chunk index inside each row, applied on the global-address side
// when loading and on the LDS-address side when reading:
//   rows of 256 bytes (16 chunks): chunk ^= row & 15;   rows of 128 bytes (8 chunks): chunk ^= (row >> 1) & 7.
template <int D>
struct Lds {
  static constexpr int K_ROW = D * 2;   // bytes per key row
  static constexpr int V_ROW = TK * 2;  // bytes per V^T row (one head-dim index, TK keys)
  static constexpr int K_BYTES = TK * K_ROW;
  static constexpr int V_BYTES = D * V_ROW;
  static constexpr int STAGE = K_BYTES + V_BYTES;
};
template <int ROW_BYTES>
__device__ __forceinline__ int swz(int row) { return ROW_BYTES == 256 ? (row & 15) : ((row >> 1) & 7); }

// s_waitcnt vmcnt(n) alone (expcnt / lgkmcnt fields left at "no wait")
#define PC_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 0xf) | (7 << 4) | (15 << 8) | ((((n) >> 4) & 3) << 14))

// 2^x on the hardware transcendental unit; arguments here are bounded above by kLazy.
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// max / sum over the two lanes (l, l+32) that share a query row
__device__ __forceinline__ float pair_max(float x) { return fmaxf(x, __shfl_xor(x, 32, 64)); }
__device__ __forceinline__ float pair_sum(float x) { return x + __shfl_xor(x, 32, 64); }

// eight E4M3 codes (two dwords) times a power-of-two scale -> the eight bf16 values of one MFMA operand (exact)
__device__ __forceinline__ bf16x8 codes_to_bf16(unsigned w0, unsigned w1, float scale) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  union { bf16x2 p[4]; bf16x8 v; } u;
  u.p[0] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w0, scale, false);
  u.p[1] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w0, scale, true);
  u.p[2] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w1, scale, false);
  u.p[3] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w1, scale, true);
  return u.v;
}

// NW wavefronts per workgroup (32 query rows each), NSTAGE LDS stages of one K tile + one V block.
// KV8: the store holds 8-bit slots (E4M3 codes, one power-of-two scale per kv head and 64-token block; layouts in
// kvstore.hip).  Such a tile takes half a stage; a lane's 16-byte LDS read then carries the operands of two
// consecutive k-steps, which are turned into bf16 (exactly) on the way to the MFMA.  For that the head dim is
// walked in the order  32 j + 16 g2 + 8 jj  (k-step 2 j + jj, lane half g2) by K, Q and the fresh bf16 K alike.
// The fresh tiles stay bf16.  KV8 kernels run with two stages.
// KSP = 2: two wavefronts share a 32-row block and take one 32-key block of every tile each (separate running
// maximum / sum / output, merged through LDS at the end); for the cases with few rows per kv head, where the per-tile
// chain of one wavefront, not the key stream, would set the pace.
template <int D, int NW, int NSTAGE, bool KV8 = false, int KSP = 1, bool MIXED = false>
__global__ __launch_bounds__(64 * NW, 2) void reuse_attention_kernel(
    const __bf16 *__restrict__ Q, const __bf16 *__restrict__ Kf, const __bf16 *__restrict__ Vf_blk,
    const void *__restrict__ k_store_any, const void *__restrict__ v_store_any, const float *__restrict__ k_scale,
    const float *__restrict__ v_scale, const __bf16 *__restrict__ k_store16, const __bf16 *__restrict__ v_store16, int n_slots16,
    const int32_t *__restrict__ table,
    int tbl_stride, int T, int Hq, int Hkv, int C, int n_splits, int q_tiles, int n_groups, float scale_log2e,
    __bf16 *__restrict__ out, __bf16 *__restrict__ part_o, float *__restrict__ part_ml) {
  static_assert(!KV8 || NSTAGE == 2, "8-bit slots: two stages (the waits assume one tile in flight)");
  const __bf16 *k_store = (const __bf16 *)k_store_any, *v_store = (const __bf16 *)v_store_any;
  const uint8_t *k8_store = (const uint8_t *)k_store_any, *v8_store = (const uint8_t *)v_store_any;
  using L = Lds<D>;
  constexpr int KS = D / 16;  // k-steps of the QK^T contraction
  constexpr int DB = D / 32;  // 32-wide blocks of the head dim (rows of O^T)
  constexpr int NT = 64 * NW;      // threads
  constexpr int QROWS = 32 * NW / KSP;   // query rows per workgroup
  constexpr int NKB = 2 / KSP;           // 32-key blocks of a tile per wavefront
  static_assert(KSP == 1 || (KSP == 2 && NW % 2 == 0), "key split over one or two wavefronts");
  constexpr int AHEAD = NSTAGE - 1;  // tiles in flight ahead of the one being computed
  __shared__ __align__(16) char lds[NSTAGE * L::STAGE];

  // workgroup -> (stream group, q tile): the q tiles of one stream group are consecutive on one XCD
  const int xcd = blockIdx.x & 7, jj = blockIdx.x >> 3;
  const int sg = (jj / q_tiles) * 8 + xcd, qt = jj % q_tiles;
  if (sg >= n_groups) return;
  const int split = sg % n_splits, bg = sg / n_splits;
  const int gkv = bg % Hkv, b = bg / Hkv;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, g2 = lane >> 5;
  const int G = Hq / Hkv, R = G * T;

  // Chunk list of this query.  Lane c keeps (slot, used length) of chunk c for the first 64 chunks, so that the
  // walk over the list costs one memory latency in all; chunks past the 64th are read from the table when met.
  const int32_t *trow = table + (size_t)b * tbl_stride;
  int my_slot = 0, my_used = 0;
  if (lane < (tbl_stride - kTblHeader) / 2) {
    const int2 e = *(const int2 *)(trow + kTblHeader + 2 * lane);
    my_slot = e.x;
    my_used = e.y;
  }
  const int n_chunks = trow[0];
  const int n_cached_tiles = trow[2];
  if (lane >= n_chunks) my_used = 0;
  const unsigned long long live = __ballot(my_used > 0);  // chunks (of the first 64) with keys to read

  // rows of this workgroup and the fresh tiles they can see
  const int row_first = qt * QROWS;
  const int row_last = min(row_first + QROWS, R) - 1;
  const int i_max = (row_first / T == row_last / T) ? (row_last % T) : (T - 1);
  const int n_tiles = n_cached_tiles + i_max / TK + 1;
  const int tile_begin = (int)((long)split * n_tiles / n_splits);
  const int tile_end = (int)((long)(split + 1) * n_tiles / n_splits);

  // this lane's query row (as column of S^T / O^T)
  const int kb0 = KSP == 2 ? (wave & 1) : 0;  // this wavefront's first key block inside a tile
  const int my_row = row_first + (wave / KSP) * 32 + l32;
  const bool row_ok = my_row < R;
  const bool wave_live = row_first + (wave / KSP) * 32 < R;  // wave-uniform: does this wavefront own any row?
  const int row_c = row_ok ? my_row : R - 1;
  const int hg = row_c / T, my_i = row_c - hg * T;
  const int head = gkv * G + hg;

  // Q fragments (B operand): lane holds q[row][16 ks + 8 g2 .. +7]  (8-bit slots: [32 (ks/2) + 16 g2 + 8 (ks%2) .. +7])
  bf16x8 qf[KS];
  {
    const __bf16 *qrow = Q + (((size_t)b * Hq + head) * T + my_i) * D;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[ks] = *(const bf16x8 *)(qrow + (KV8 ? 32 * (ks >> 1) + 16 * g2 + 8 * (ks & 1) : ks * 16 + g2 * 8));
  }

  f32x16 o_acc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) o_acc[db][r] = 0.f;
  float m_ref = -INFINITY, l_run = 0.f;  // m_ref: reference exponent (scaled, log2 domain)

  // ---- tile cursor over the chunk list.  The chunk's slot id and used length are kept in (scalar) registers and
  // re-read from the table only when the cursor enters another chunk.
  struct Cursor { int chunk, off, slot, used; };  // chunk index, tile index inside the chunk (or the fresh part)
  auto enter_chunk = [&](Cursor &c) __attribute__((always_inline)) {
    if (c.chunk < 64) {  // skip unused chunks
      const unsigned long long rest = live >> c.chunk;
      c.chunk = rest ? c.chunk + __builtin_ctzll(rest) : min(n_chunks, 64);
    }
    while (c.chunk >= 64 && c.chunk < n_chunks && trow[kTblHeader + 2 * c.chunk + 1] == 0) ++c.chunk;
    if (c.chunk < min(n_chunks, 64)) {
      const int ch = __builtin_amdgcn_readfirstlane(c.chunk);
      c.slot = __builtin_amdgcn_readlane(my_slot, ch);
      c.used = __builtin_amdgcn_readlane(my_used, ch);
    } else if (c.chunk < n_chunks) {
      c.slot = trow[kTblHeader + 2 * c.chunk];
      c.used = trow[kTblHeader + 2 * c.chunk + 1];
    }
  };
  Cursor cur = {0, 0, 0, 0};
  {
    // tiles of the chunks before each lane's chunk (exclusive scan over the lanes), then the chunk tile_begin is in
    const int my_tiles = (my_used + TK - 1) / TK;
    int incl = my_tiles;
#pragma unroll
    for (int sh = 1; sh < 64; sh <<= 1) {
      const int up = __shfl_up(incl, sh, 64);
      if (lane >= sh) incl += up;
    }
    cur.chunk = __popcll(__ballot(incl <= tile_begin && lane < n_chunks));
    int rem;
    if (cur.chunk < min(n_chunks, 64)) {
      rem = tile_begin - __builtin_amdgcn_readlane(incl - my_tiles, __builtin_amdgcn_readfirstlane(cur.chunk));
    } else {
      rem = tile_begin - __builtin_amdgcn_readlane(incl, 63);
      while (cur.chunk < n_chunks) {
        int ntc = (trow[kTblHeader + 2 * cur.chunk + 1] + TK - 1) / TK;
        if (rem < ntc) break;
        rem -= ntc;
        ++cur.chunk;
      }
    }
    cur.off = rem;
    enter_chunk(cur);
  }

  // ---- direct global -> LDS staging of one tile.  Wavefront instruction i writes bytes [1024 i, 1024 i + 1024)
  // of the K tile (or V block); lane l lands at byte 1024 i + 16 l, i.e. row (1024 i + 16 l) / ROW, physical
  // chunk ((1024 i + 16 l) % ROW) / 16, and therefore fetches the logical chunk (physical ^ swizzle(row)).
  static_assert(NSTAGE * L::STAGE <= 160 * 1024, "LDS stages exceed the 160 KB of a CU");
  constexpr int K_INSTR = L::K_BYTES / 1024 / NW;  // per wavefront
  constexpr int V_INSTR = L::V_BYTES / 1024 / NW;
  static_assert(K_INSTR >= 1 && V_INSTR >= 1, "tile too small for this many wavefronts");
  int k_row[K_INSTR], k_col[K_INSTR], v_goff[V_INSTR];
#pragma unroll
  for (int k = 0; k < K_INSTR; ++k) {
    const int byte = (wave + k * NW) * 1024 + lane * 16;
    const int row = byte / L::K_ROW, pc = (byte % L::K_ROW) / 16;
    k_row[k] = row;
    k_col[k] = (pc ^ swz<L::K_ROW>(row)) * 8;  // element offset inside the row
  }
#pragma unroll
  for (int k = 0; k < V_INSTR; ++k) {
    const int byte = (wave + k * NW) * 1024 + lane * 16;
    const int d = byte / L::V_ROW, pc = (byte % L::V_ROW) / 16;
    v_goff[k] = d * TK + (pc ^ swz<L::V_ROW>(d)) * 8;  // element offset inside the block
  }
  // swizzled byte offsets of this lane's MFMA operand reads inside its row
  int k_rd[KS], v_rd[4];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks)
    k_rd[ks] = ((KV8 ? 4 * (ks >> 1) + 2 * g2 + (ks & 1) : 2 * ks + g2) ^ swz<L::K_ROW>(l32)) * 16;
#pragma unroll
  for (int c4 = 0; c4 < 2 * NKB; ++c4) v_rd[c4] = ((2 * (2 * kb0 + c4) + g2) ^ swz<L::V_ROW>(l32)) * 16;
  // 8-bit tiles: K rows of D bytes, V^T rows of TK bytes; 16-byte chunk index XOR-swizzled by the row as above
  // (rows of 128 bytes: (row >> 1) & 7; rows of 64 bytes: (row >> 2) & 3)
  constexpr int K8_ROW = D, V8_ROW = TK;
  constexpr int K8_TOTAL = TK * K8_ROW / 1024, V8_TOTAL = D * V8_ROW / 1024;  // load instructions per tile (all wavefronts)
  constexpr int K8_INSTR = KV8 ? (K8_TOTAL + NW - 1) / NW : 1, V8_INSTR = KV8 ? (V8_TOTAL + NW - 1) / NW : 1;
  auto swz8 = [](int row_bytes, int row) { return row_bytes == 128 ? ((row >> 1) & 7) : ((row >> 2) & 3); };
  int k8_row[K8_INSTR], k8_col[K8_INSTR], v8_goff[V8_INSTR], k8_rd[KS / 2], v8_rd[2];
  if (KV8) {
#pragma unroll
    for (int k = 0; k < K8_INSTR; ++k) {
      const int byte = (wave + k * NW) * 1024 + lane * 16;
      const int row = byte / K8_ROW, pc = (byte % K8_ROW) / 16;
      k8_row[k] = row;
      k8_col[k] = (pc ^ swz8(K8_ROW, row)) * 16;
    }
#pragma unroll
    for (int k = 0; k < V8_INSTR; ++k) {
      const int byte = (wave + k * NW) * 1024 + lane * 16;
      const int d = byte / V8_ROW, pc = (byte % V8_ROW) / 16;
      v8_goff[k] = d * V8_ROW + (pc ^ swz8(V8_ROW, d)) * 16;
    }
#pragma unroll
    for (int j = 0; j < KS / 2; ++j) k8_rd[j] = ((2 * j + g2) ^ swz8(K8_ROW, l32)) * 16;
#pragma unroll
    for (int J = 0; J < NKB; ++J) v8_rd[J] = ((2 * (kb0 + J) + g2) ^ swz8(V8_ROW, l32)) * 16;
  }
  // is8: the tile holds 8-bit codes (a chunk in an 8-bit slot); fresh tiles and chunks in bf16 slots are bf16 tiles.
  // A context may hold slots of both formats: ids below n_slots16 are bf16 slots of k_store16 / v_store16.
  struct TileDesc { const __bf16 *k, *v; int valid; int t0; bool fresh; bool is8; float ks, vs; };
  auto describe = [&](const Cursor &c, TileDesc &td) __attribute__((always_inline)) {
    if (c.chunk < n_chunks) {
      // (no branch around the scale loads: a branch would make the wavefront wait for them here instead of at their
      // first use, a tile later)
      // MIXED: the call names chunks of both formats (else every chunk of a KV8 launch sits in an 8-bit slot, and the
      // compiler keeps the bf16 path out of the cached part of the loop)
      const bool is8 = KV8 && (!MIXED || c.slot >= n_slots16);
      const int s = is8 ? c.slot - n_slots16 : c.slot;
      const size_t base = (((size_t)s * Hkv + gkv) * C + (size_t)c.off * TK) * D;  // same offset in both layouts
      if (KV8) {
        td.k = is8 ? (const __bf16 *)(k8_store + base) : k_store16 + base;
        td.v = is8 ? (const __bf16 *)(v8_store + base) : v_store16 + base;
        const size_t sc = is8 ? ((size_t)s * Hkv + gkv) * (C / TK) + c.off : 0;
        const float lk = k_scale[sc], lv = v_scale[sc];
        td.ks = is8 ? lk : 1.f;
        td.vs = is8 ? lv : 1.f;
      } else {
        td.k = k_store + base;
        td.v = v_store + base;
        td.ks = td.vs = 1.f;
      }
      td.is8 = is8;
      td.valid = min(TK, c.used - c.off * TK);
      td.t0 = 0;
      td.fresh = false;
    } else {
      td.ks = td.vs = 1.f;
      td.is8 = false;
      const int ft = (T + TK - 1) / TK;
      td.k = Kf + (((size_t)b * Hkv + gkv) * T + (size_t)c.off * TK) * D;
      td.v = Vf_blk + (((size_t)b * Hkv + gkv) * ft + c.off) * (size_t)(TK * D);
      td.valid = min(TK, T - c.off * TK);
      td.t0 = c.off * TK;
      td.fresh = true;
    }
  };
  auto advance = [&](Cursor &c) __attribute__((always_inline)) {
    ++c.off;
    if (c.chunk < n_chunks && c.off * TK >= c.used) {
      c.off = 0;
      ++c.chunk;
      enter_chunk(c);
    }
  };
  auto fetch_tile = [&](const TileDesc &td, int st) __attribute__((always_inline)) {
    char *kb = lds + st * L::STAGE;
    if (KV8 && td.is8) {
      const uint8_t *k8 = (const uint8_t *)td.k, *v8 = (const uint8_t *)td.v;
#pragma unroll
      for (int k = 0; k < K8_INSTR; ++k)
        if ((wave + k * NW) < K8_TOTAL) {
          const int row = min(k8_row[k], td.valid - 1);
          __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(k8 + (size_t)row * K8_ROW + k8_col[k]),
                                           (__attribute__((address_space(3))) void *)(kb + (wave + k * NW) * 1024), 16, 0, kKvAux);
        }
#pragma unroll
      for (int k = 0; k < V8_INSTR; ++k)
        if ((wave + k * NW) < V8_TOTAL)
          __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(v8 + v8_goff[k]),
                                           (__attribute__((address_space(3))) void *)(kb + L::K_BYTES + (wave + k * NW) * 1024), 16, 0, kKvAux);
      return;
    }
#pragma unroll
    for (int k = 0; k < K_INSTR; ++k) {
      const int row = min(k_row[k], td.valid - 1);  // rows past a ragged end repeat the last valid row (masked later)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(td.k + (size_t)row * D + k_col[k]),
                                       (__attribute__((address_space(3))) void *)(kb + (wave + k * NW) * 1024), 16, 0, kKvAux);
    }
#pragma unroll
    for (int k = 0; k < V_INSTR; ++k)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(td.v + v_goff[k]),
                                       (__attribute__((address_space(3))) void *)(kb + L::K_BYTES + (wave + k * NW) * 1024), 16, 0, kKvAux);
  };

  // Pipeline: the tile computed in iteration t sits in stage t % NSTAGE; the loads of tile t+AHEAD are issued at
  // the top of iteration t into the stage that iteration t-1 finished reading (the barrier at its end says so).
  // At the end of iteration t the loads of tile t+1 must have landed: they are the oldest outstanding ones, so
  // waiting until at most (AHEAD-1) tiles' worth of loads remain is enough; then one barrier publishes them.
  // Two cursors walk the chunk list: cur for the tile being fetched, cmp for the one being computed.
  Cursor cmp = cur;
  int fetched = tile_begin;  // next tile to fetch
#pragma unroll
  for (int k = 0; k < AHEAD; ++k) {
    if (fetched < tile_end) {
      TileDesc t0d;
      describe(cur, t0d);
      fetch_tile(t0d, k);
      advance(cur);
      ++fetched;
    }
  }
  // Consume the Q fragments here, once (their latency has run beside the first tiles'): otherwise the loads are
  // still "pending" at the loop header in the compiler's wait-count model and every iteration waits on its own
  // K/V prefetch before the first MFMA.
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(qf[ks]));
  PC_WAIT_VMCNT(0);
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");

  int stage = 0;  // (tt - tile_begin) % NSTAGE
  for (int tt = tile_begin; tt < tile_end; ++tt) {
    const int buf = stage;
    int in_stage = stage + AHEAD;
    if (in_stage >= NSTAGE) in_stage -= NSTAGE;
    const bool has_next = fetched < tile_end;
    if (has_next) {
      TileDesc nxt;
      describe(cur, nxt);
      fetch_tile(nxt, in_stage);
      advance(cur);
      ++fetched;
    }
    TileDesc td;
    describe(cmp, td);
    advance(cmp);
    const char *kb = lds + buf * L::STAGE;
    const char *vb = kb + L::K_BYTES;

    if (wave_live) {  // (a wavefront without rows only helps to load the tiles)
    // ---- S^T = K Q^T : two 32-key blocks.  The K operands are requested from LDS in batches of eight ahead of
    // their MFMAs (the two accumulation chains alternating): one LDS latency per batch instead of one per MFMA.
    f32x16 s_acc[NKB];
#pragma unroll
    for (int kbk = 0; kbk < NKB; ++kbk)
#pragma unroll
      for (int r = 0; r < 16; ++r) s_acc[kbk][r] = 0.f;
    const char *kbw = kb + kb0 * 32 * (KV8 && td.is8 ? K8_ROW : L::K_ROW);  // this wavefront's key rows
    if (KV8 && td.is8) {
      // 8-bit tile: one 16-byte read per key block and pair of k-steps, turned into two bf16 operands
#pragma unroll
      for (int h = 0; h < KS / 4; ++h) {
        pc::u32x4 raw[NKB][2];
#pragma unroll
        for (int j2 = 0; j2 < 2; ++j2)
#pragma unroll
          for (int kbk = 0; kbk < NKB; ++kbk) raw[kbk][j2] = *(const pc::u32x4 *)(kbw + (kbk * 32 + l32) * K8_ROW + k8_rd[2 * h + j2]);
#pragma unroll
        for (int j2 = 0; j2 < 2; ++j2)
#pragma unroll
          for (int kbk = 0; kbk < NKB; ++kbk) {
            const bf16x8 a0 = codes_to_bf16(raw[kbk][j2][0], raw[kbk][j2][1], td.ks);
            const bf16x8 a1 = codes_to_bf16(raw[kbk][j2][2], raw[kbk][j2][3], td.ks);
            s_acc[kbk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, qf[4 * h + 2 * j2], s_acc[kbk], 0, 0, 0);
            s_acc[kbk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, qf[4 * h + 2 * j2 + 1], s_acc[kbk], 0, 0, 0);
          }
      }
    } else {
#pragma unroll
    for (int h = 0; h < KS / 4; ++h) {
      bf16x8 kop[NKB][4];
#pragma unroll
      for (int k4 = 0; k4 < 4; ++k4)
#pragma unroll
        for (int kbk = 0; kbk < NKB; ++kbk) kop[kbk][k4] = *(const bf16x8 *)(kbw + (kbk * 32 + l32) * L::K_ROW + k_rd[4 * h + k4]);
#pragma unroll
      for (int k4 = 0; k4 < 4; ++k4)
#pragma unroll
        for (int kbk = 0; kbk < NKB; ++kbk)
          s_acc[kbk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kop[kbk][k4], qf[4 * h + k4], s_acc[kbk], 0, 0, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 4 * NKB, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 4 * NKB, 0);
    }
    }

    // ---- mask: only tiles with a ragged end or in the causal part take this path (wave-uniform test)
    if (td.valid < TK || td.fresh) {
#pragma unroll
      for (int kbk = 0; kbk < NKB; ++kbk)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          int t = (kb0 + kbk) * 32 + (r >> 2) * 8 + g2 * 4 + (r & 3);
          bool vis = t < td.valid && (!td.fresh || td.t0 + t <= my_i);
          s_acc[kbk][r] = vis ? s_acc[kbk][r] : -INFINITY;
        }
    }

    // ---- online softmax in the log2 domain with a lazily refreshed reference exponent.  Common path: the
    // probabilities are taken against the current reference and only their sum is looked at -- a probability above
    // 2^kLazy shows up there, so no row maximum is needed.  The row sum is taken over the bf16-rounded
    // probabilities (the very values the PV product uses), two per instruction.
    bf16x8 pf[NKB][2];
    auto exponentials = [&](float neg_m) __attribute__((always_inline)) {
      typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
      const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
      float sum = 0.f;
#pragma unroll
      for (int kbk = 0; kbk < NKB; ++kbk)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int e = 0; e < 8; e += 2) {
            const float p0 = fast_exp2(__builtin_fmaf(s_acc[kbk][j * 8 + e], scale_log2e, neg_m));
            const float p1 = fast_exp2(__builtin_fmaf(s_acc[kbk][j * 8 + e + 1], scale_log2e, neg_m));
            const bf16x2 pr = {(__bf16)p0, (__bf16)p1};
            pf[kbk][j][e] = pr[0];
            pf[kbk][j][e + 1] = pr[1];
            sum = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, sum, false);
          }
      return sum;
    };
    float psum = 0.f;
    bool refresh = __builtin_amdgcn_ballot_w64(m_ref == -INFINITY) != 0;  // a row that has seen no key yet
    if (!refresh) {
      psum = exponentials(-m_ref);
      refresh = __builtin_amdgcn_ballot_w64(!(psum <= kSumLimit)) != 0;   // also catches inf / nan
    }
    if (refresh) {  // rare: row maxima, exchange between the two lanes of a row, rescale, probabilities again
      float mx = s_acc[0][0];
#pragma unroll
      for (int kbk = 0; kbk < NKB; ++kbk)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s_acc[kbk][r]);
      const float mc = pair_max(mx) * scale_log2e;
      const bool upd = mc > m_ref;  // (false for a row whose keys are all masked: mc = -inf)
      const float alpha = upd ? fast_exp2(m_ref - mc) : 1.0f;  // m_ref = -inf gives 0
      m_ref = upd ? mc : m_ref;
      l_run *= alpha;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o_acc[db][r] *= alpha;
      psum = exponentials((m_ref == -INFINITY) ? 0.f : -m_ref);
    }
    l_run += psum;

    // ---- O^T += V^T P^T, operands requested in batches of eight in the same way
    if (KV8 && td.is8) {
#pragma unroll
      for (int h = 0; h < NKB; ++h) {
        pc::u32x4 raw[DB];
#pragma unroll
        for (int db = 0; db < DB; ++db) raw[db] = *(const pc::u32x4 *)(vb + (db * 32 + l32) * V8_ROW + v8_rd[h]);
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          const bf16x8 a0 = codes_to_bf16(raw[db][0], raw[db][1], td.vs);
          const bf16x8 a1 = codes_to_bf16(raw[db][2], raw[db][3], td.vs);
          o_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, pf[h][0], o_acc[db], 0, 0, 0);
          o_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, pf[h][1], o_acc[db], 0, 0, 0);
        }
      }
    } else {
#pragma unroll
    for (int h = 0; h < NKB; ++h) {
      bf16x8 vop[DB][2];
#pragma unroll
      for (int c2 = 0; c2 < 2; ++c2)
#pragma unroll
        for (int db = 0; db < DB; ++db) vop[db][c2] = *(const bf16x8 *)(vb + (db * 32 + l32) * L::V_ROW + v_rd[2 * h + c2]);
#pragma unroll
      for (int c2 = 0; c2 < 2; ++c2)
#pragma unroll
        for (int db = 0; db < DB; ++db)
          o_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vop[db][c2], pf[h][c2], o_acc[db], 0, 0, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 2 * DB, 1);
      __builtin_amdgcn_sched_group_barrier(0x008, 2 * DB, 1);
    }
    }

    }  // wave_live

    // (when nothing was fetched in this iteration fewer tiles are in flight: wait for all of them)
    if (AHEAD == 1 || !has_next) PC_WAIT_VMCNT(0); else PC_WAIT_VMCNT((AHEAD - 1) * (K_INSTR + V_INSTR));
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    stage = stage + 1 == NSTAGE ? 0 : stage + 1;
  }

  if (KSP == 2) {
    // the wavefront of the odd key blocks hands its state over lane to lane (the loop's last barrier has retired the tiles)
    float *mine = (float *)lds + (size_t)(wave >> 1) * (DB * 16 + 2) * 64 + lane;
    if (kb0 == 1) {
      mine[0] = m_ref;
      mine[64] = l_run;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) mine[(2 + db * 16 + r) * 64] = o_acc[db][r];
    }
    __syncthreads();
    if (kb0 == 1) return;
    const float m1 = mine[0], l1 = mine[64];
    const float m = fmaxf(m_ref, m1);
    const float a0 = m_ref == -INFINITY ? 0.f : fast_exp2(m_ref - m), a1 = m1 == -INFINITY ? 0.f : fast_exp2(m1 - m);
    l_run = l_run * a0 + l1 * a1;
    m_ref = m;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) o_acc[db][r] = o_acc[db][r] * a0 + mine[(2 + db * 16 + r) * 64] * a1;
  }

  // ---- finish: combine the two lanes of a row, normalise, write
  const float l_tot = pair_sum(l_run);
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
    // partial outputs are normalised per split and kept in bf16: they are convex combinations of V rows, and the
    // merge weights them in fp32, so this costs one extra bf16 rounding and halves the merge traffic
    __bf16 *po = part_o + prow * D;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        pc::bf16x4 v = {(__bf16)(o_acc[db][q4 * 4 + 0] * inv), (__bf16)(o_acc[db][q4 * 4 + 1] * inv),
                        (__bf16)(o_acc[db][q4 * 4 + 2] * inv), (__bf16)(o_acc[db][q4 * 4 + 3] * inv)};
        *(pc::bf16x4 *)(po + db * 32 + q4 * 8 + g2 * 4) = v;
      }
    if (g2 == 0) {
      part_ml[prow * 2] = m_ref;
      part_ml[prow * 2 + 1] = l_tot;
    }
  }
}

// Long-context kernel: bf16 slots, 8 wavefronts x 32 rows per workgroup, chunk lists of at most 64 entries (both head
// sizes; the figures below are for head size 128).  The
// arithmetic is that of reuse_attention_kernel; the loop around it is pared down, because at 32 MFMAs per tile and
// wavefront the vector and scalar ports are nearly as busy as the matrix pipe and every instruction beside the
// arithmetic shows in the tile time (cycles per 64-key tile on the 16 x 1024-key, 256-row, batch-8 launch: 4100 for
// the general kernel, 3320 here, 3050-3150 for the bare tile arithmetic):
//   - three LDS stages; the requests for tile t+2 are issued at the END of iteration t by wavefronts 0..3 only, one
//     per SIMD, from 32-bit lane offsets computed once (a ragged tile takes a rarely used branch that clamps its rows);
//   - only those wavefronts walk the chunk list with pointers, and the walk moves on by adding a tile's size; the step
//     to the next chunk is a rarely taken branch.  Every wavefront keeps a second cursor of three integers (chunk,
//     keys left, first fresh token) that tells whether the tile it computes on needs a mask;
//   - mask and reference refresh are marked unlikely, so the usual tile is one fall-through path;
//   - the V operands of the first 32-key block are requested before the softmax arithmetic;
//   - the row sums are fp32 adds of the unrounded probabilities: the two-element bf16 dot instruction runs on the
//     matrix pipe and does not overlap with the other wavefront's MFMAs.  (The sum then differs from the sum of the
//     bf16 values the PV product multiplies by at most 2^-9 relative, the rounding of one probability.)
//   - LDS is touched by the requests and by operand reads only: with an ordinary LDS store or an LDS object of another
//     kind in the kernel, the compiler places a wait for all outstanding requests before the first operand read.
template <int D>
__global__ __launch_bounds__(512, 2) void reuse_attention_wide_kernel(
    const __bf16 *__restrict__ Q, const __bf16 *__restrict__ Kf, const __bf16 *__restrict__ Vf_blk,
    const __bf16 *__restrict__ k_store, const __bf16 *__restrict__ v_store, const int32_t *__restrict__ table,
    int tbl_stride, int T, int Hq, int Hkv, int C, int n_splits, int q_tiles, int n_groups, float scale_log2e,
    __bf16 *__restrict__ out, __bf16 *__restrict__ part_o, float *__restrict__ part_ml) {
  using L = Lds<D>;
  constexpr int NW = 8, NLD = 4, NSTAGE = 3, KS = D / 16, DB = D / 32, QROWS = 32 * NW;
  __shared__ __align__(16) char lds[NSTAGE * L::STAGE];

  const int xcd = blockIdx.x & 7, jj0 = blockIdx.x >> 3;
  const int sg = (jj0 / q_tiles) * 8 + xcd, qt = jj0 % q_tiles;
  if (sg >= n_groups) return;
  const int split = sg % n_splits, bg = sg / n_splits;
  const int gkv = bg % Hkv, b = bg / Hkv;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, g2 = lane >> 5;
  const int G = Hq / Hkv, R = G * T;

  // chunk list: lane c keeps (slot, used length) of chunk c (at most 64 chunks)
  const int32_t *trow = table + (size_t)b * tbl_stride;
  int my_slot = 0, my_used = 0;
  if (lane < (tbl_stride - kTblHeader) / 2) {
    const int2 e = *(const int2 *)(trow + kTblHeader + 2 * lane);
    my_slot = e.x;
    my_used = e.y;
  }
  const int n_chunks = trow[0];
  const int n_cached_tiles = trow[2];
  if (lane >= n_chunks) my_used = 0;
  const unsigned long long live = __ballot(my_used > 0);

  const int row_first = qt * QROWS;
  const int row_last = min(row_first + QROWS, R) - 1;
  const int i_max = (row_first / T == row_last / T) ? (row_last % T) : (T - 1);
  const int n_tiles = n_cached_tiles + i_max / TK + 1;
  const int tile_begin = (int)((long)split * n_tiles / n_splits);
  const int tile_end = (int)((long)(split + 1) * n_tiles / n_splits);
  const int n = tile_end - tile_begin;

  const int my_row = row_first + wave * 32 + l32;
  const bool row_ok = my_row < R;
  const int row_c = row_ok ? my_row : R - 1;   // (wavefronts past the last row compute on the last row and write nothing)
  const int hg = row_c / T, my_i = row_c - hg * T;
  const int head = gkv * G + hg;

  bf16x8 qf[KS];
  {
    const __bf16 *qrow = Q + (((size_t)b * Hq + head) * T + my_i) * D;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[ks] = *(const bf16x8 *)(qrow + ks * 16 + g2 * 8);
  }
  f32x16 o_acc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) o_acc[db][r] = 0.f;
  float m_ref = -INFINITY, l_run = 0.f;
  bool all_started = false;

  // ---- cursor over the tiles of this range, kept by the loading wavefronts only: pointers that move on by one tile,
  // the keys left in the chunk (or in the fresh part), and a rarely taken step to the next chunk that has keys.
  // What the computing side needs of a tile -- how many keys are valid and, for a fresh tile, its first token --
  // comes from a second, lighter cursor without pointers that every wavefront steps once per tile.
  const int ft = (T + TK - 1) / TK;
  const __bf16 *const kf_base = Kf + ((size_t)b * Hkv + gkv) * T * D;
  const __bf16 *const vf_base = Vf_blk + ((size_t)b * Hkv + gkv) * ft * (size_t)(TK * D);
  const __bf16 *c_k = kf_base, *c_v = vf_base;
  int c_chunk, c_rem, c_t0;   // c_t0 < 0: in a cached chunk; else first token of the cursor's fresh tile
  auto enter_chunk = [&](int chunk) __attribute__((always_inline)) {   // chunk == n_chunks: the fresh part
    c_chunk = chunk;
    if (chunk < n_chunks) {
      const int slot = __builtin_amdgcn_readlane(my_slot, chunk);
      const size_t cbase = ((size_t)slot * Hkv + gkv) * C * (size_t)D;
      c_k = k_store + cbase;
      c_v = v_store + cbase;
      c_rem = __builtin_amdgcn_readlane(my_used, chunk);
      c_t0 = -1;
    } else {
      c_k = kf_base;
      c_v = vf_base;
      c_rem = T;
      c_t0 = 0;
    }
  };
  {
    const int my_tiles = (my_used + TK - 1) / TK;
    int incl = my_tiles;
#pragma unroll
    for (int sh = 1; sh < 64; sh <<= 1) {
      const int up = __shfl_up(incl, sh, 64);
      if (lane >= sh) incl += up;
    }
    const int first = __popcll(__ballot(incl <= tile_begin && lane < n_chunks));   // chunks wholly before tile_begin
    const int before = __builtin_amdgcn_readlane(incl - my_tiles, min(first, 63));
    enter_chunk(first);   // (a chunk found this way has keys: its tile count is positive)
    const int off = first < n_chunks ? tile_begin - before : tile_begin - n_cached_tiles;
    c_k += (size_t)off * (TK * D);
    c_v += (size_t)off * (TK * D);
    c_rem -= off * TK;
    if (c_t0 >= 0) c_t0 = off * TK;
  }
  auto step_cursor = [&]() __attribute__((always_inline)) {
    c_k += TK * D;
    c_v += TK * D;
    c_rem -= TK;
    if (c_t0 >= 0) c_t0 += TK;
    if (__builtin_expect(c_rem <= 0 && c_t0 < 0, 0)) {
      const unsigned long long rest = c_chunk < 63 ? live >> (c_chunk + 1) : 0ull;
      enter_chunk(rest ? c_chunk + 1 + (int)__builtin_ctzll(rest) : n_chunks);
    }
  };

  int q_chunk = c_chunk, q_rem = c_rem, q_t0 = c_t0;   // the computing side's cursor: same walk, no pointers
  auto step_compute_cursor = [&]() __attribute__((always_inline)) {
    q_rem -= TK;
    if (q_t0 >= 0) q_t0 += TK;
    if (__builtin_expect(q_rem <= 0 && q_t0 < 0, 0)) {
      const unsigned long long rest = q_chunk < 63 ? live >> (q_chunk + 1) : 0ull;
      q_chunk = rest ? q_chunk + 1 + (int)__builtin_ctzll(rest) : n_chunks;
      const bool cached = q_chunk < n_chunks;
      q_rem = cached ? __builtin_amdgcn_readlane(my_used, min(q_chunk, 63)) : T;
      q_t0 = cached ? -1 : 0;
    }
  };

  // ---- requests: wavefronts 0..3 bring in a tile, 4 K instructions and 4 V instructions each
  constexpr int K_INSTR = L::K_BYTES / 1024 / NLD, V_INSTR = L::V_BYTES / 1024 / NLD;
  int k_row[K_INSTR], k_col[K_INSTR];
  unsigned k_off[K_INSTR], v_off[V_INSTR];   // byte offsets from the tile's first K row / V block
#pragma unroll
  for (int k = 0; k < K_INSTR; ++k) {
    const int byte = ((wave & (NLD - 1)) + k * NLD) * 1024 + lane * 16;
    const int row = byte / L::K_ROW, pc = (byte % L::K_ROW) / 16;
    k_row[k] = row;
    k_col[k] = (pc ^ swz<L::K_ROW>(row)) * 8;
    k_off[k] = (unsigned)(row * D + k_col[k]) * 2u;
  }
#pragma unroll
  for (int k = 0; k < V_INSTR; ++k) {
    const int byte = ((wave & (NLD - 1)) + k * NLD) * 1024 + lane * 16;
    const int d = byte / L::V_ROW, pc = (byte % L::V_ROW) / 16;
    v_off[k] = (unsigned)(d * TK + (pc ^ swz<L::V_ROW>(d)) * 8) * 2u;
  }
  int k_rd[KS], v_rd[4];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) k_rd[ks] = ((2 * ks + g2) ^ swz<L::K_ROW>(l32)) * 16;
#pragma unroll
  for (int c4 = 0; c4 < 4; ++c4) v_rd[c4] = ((2 * c4 + g2) ^ swz<L::V_ROW>(l32)) * 16;
  auto request_next = [&](int st) __attribute__((always_inline)) {   // the cursor's tile into stage st; steps the cursor
    char *kb = lds + st * L::STAGE;
    const int valid = min(TK, c_rem);
    const char *kp = (const char *)c_k, *vp = (const char *)c_v;
    if (__builtin_expect(valid < TK, 0)) {   // rows past a ragged end repeat the last valid row (masked later)
#pragma unroll
      for (int k = 0; k < K_INSTR; ++k)
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(kp + (unsigned)(min(k_row[k], valid - 1) * D + k_col[k]) * 2u),
                                         (__attribute__((address_space(3))) void *)(kb + (wave + k * NLD) * 1024), 16, 0, kKvAux);
    } else {
#pragma unroll
      for (int k = 0; k < K_INSTR; ++k)
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(kp + k_off[k]),
                                         (__attribute__((address_space(3))) void *)(kb + (wave + k * NLD) * 1024), 16, 0, kKvAux);
    }
#pragma unroll
    for (int k = 0; k < V_INSTR; ++k)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(vp + v_off[k]),
                                       (__attribute__((address_space(3))) void *)(kb + L::K_BYTES + (wave + k * NLD) * 1024), 16, 0, kKvAux);
    step_cursor();
  };

  // ---- one tile: S^T = K Q^T, softmax against the lazily refreshed reference exponent, O^T += V^T P^T
  auto tile = [&](int st) __attribute__((always_inline)) {
    const char *kb = lds + st * L::STAGE;
    const char *vb = kb + L::K_BYTES;
    f32x16 s_acc[2];
#pragma unroll
    for (int kbk = 0; kbk < 2; ++kbk)
#pragma unroll
      for (int r = 0; r < 16; ++r) s_acc[kbk][r] = 0.f;
#pragma unroll
    for (int h = 0; h < KS / 4; ++h) {
      bf16x8 kop[2][4];
#pragma unroll
      for (int k4 = 0; k4 < 4; ++k4)
#pragma unroll
        for (int kbk = 0; kbk < 2; ++kbk) kop[kbk][k4] = *(const bf16x8 *)(kb + (kbk * 32 + l32) * L::K_ROW + k_rd[4 * h + k4]);
#pragma unroll
      for (int k4 = 0; k4 < 4; ++k4)
#pragma unroll
        for (int kbk = 0; kbk < 2; ++kbk)
          s_acc[kbk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kop[kbk][k4], qf[4 * h + k4], s_acc[kbk], 0, 0, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
    }
    // V operands of the first 32-key block: their LDS latency runs under the softmax arithmetic
    bf16x8 vop0[DB][2];
#pragma unroll
    for (int c2 = 0; c2 < 2; ++c2)
#pragma unroll
      for (int db = 0; db < DB; ++db) vop0[db][c2] = *(const bf16x8 *)(vb + (db * 32 + l32) * L::V_ROW + v_rd[c2]);
    const int t_valid = min(TK, q_rem), t_t0 = q_t0;
    if (__builtin_expect(t_valid < TK || t_t0 >= 0, 0)) {
      int t_lane = g2 * 4;
      asm volatile("" : "+v"(t_lane));   // (keeps the 32 per-element key indices out of loop-invariant registers)
      const int lim_valid = t_valid - t_lane;
      const int lim_causal = t_t0 >= 0 ? my_i - t_t0 - t_lane : 0x7fffff00;
#pragma unroll
      for (int kbk = 0; kbk < 2; ++kbk)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int c = kbk * 32 + (r >> 2) * 8 + (r & 3);
          s_acc[kbk][r] = (c < lim_valid && c <= lim_causal) ? s_acc[kbk][r] : -INFINITY;
        }
    }
    bf16x8 pf[2][2];
    auto exponentials = [&](float neg_m) __attribute__((always_inline)) {
      typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
      float sum = 0.f, sum2 = 0.f;
#pragma unroll
      for (int kbk = 0; kbk < 2; ++kbk)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int e = 0; e < 8; e += 2) {
            const float p0 = fast_exp2(__builtin_fmaf(s_acc[kbk][j * 8 + e], scale_log2e, neg_m));
            const float p1 = fast_exp2(__builtin_fmaf(s_acc[kbk][j * 8 + e + 1], scale_log2e, neg_m));
            const bf16x2 pr = {(__bf16)p0, (__bf16)p1};
            pf[kbk][j][e] = pr[0];
            pf[kbk][j][e + 1] = pr[1];
            sum += p0;
            sum2 += p1;
          }
      return sum + sum2;
    };
    float psum = 0.f;
    bool refresh = !all_started;
    if (__builtin_expect(!refresh, 1)) {
      psum = exponentials(-m_ref);
      refresh = __builtin_amdgcn_ballot_w64(!(psum <= kSumLimit)) != 0;   // also catches inf / nan
    }
    if (__builtin_expect(refresh, 0)) {
      float mx = s_acc[0][0];
#pragma unroll
      for (int kbk = 0; kbk < 2; ++kbk)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s_acc[kbk][r]);
      const float mc = pair_max(mx) * scale_log2e;
      const bool upd = mc > m_ref;
      const float alpha = upd ? fast_exp2(m_ref - mc) : 1.0f;
      m_ref = upd ? mc : m_ref;
      l_run *= alpha;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o_acc[db][r] *= alpha;
      psum = exponentials((m_ref == -INFINITY) ? 0.f : -m_ref);
      all_started = __builtin_amdgcn_ballot_w64(m_ref == -INFINITY) == 0;
    }
    l_run += psum;
    bf16x8 vop1[DB][2];
#pragma unroll
    for (int c2 = 0; c2 < 2; ++c2)
#pragma unroll
      for (int db = 0; db < DB; ++db) vop1[db][c2] = *(const bf16x8 *)(vb + (db * 32 + l32) * L::V_ROW + v_rd[2 + c2]);
#pragma unroll
    for (int c2 = 0; c2 < 2; ++c2)
#pragma unroll
      for (int db = 0; db < DB; ++db)
        o_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vop0[db][c2], pf[0][c2], o_acc[db], 0, 0, 0);
#pragma unroll
    for (int c2 = 0; c2 < 2; ++c2)
#pragma unroll
      for (int db = 0; db < DB; ++db)
        o_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vop1[db][c2], pf[1][c2], o_acc[db], 0, 0, 0);
    __builtin_amdgcn_sched_group_barrier(0x100, 2 * DB, 1);
    __builtin_amdgcn_sched_group_barrier(0x008, 4 * DB, 1);
  };

  // ---- pipeline: tile t is computed from stage t % 3; tiles t+1 and t+2 are in flight or landed.  At the end of
  // iteration t wavefronts 0..3 wait for their share of tile t+1 (requested an iteration ago), request tile t+2 into
  // the stage that iteration t-1 read, and the barrier publishes tile t+1.
  if (wave < NLD) {
    if (n > 0) request_next(0);
    if (n > 1) request_next(1);
  }
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(qf[ks]));
  PC_WAIT_VMCNT(0);
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  int st = 0;
  for (int t = 0; t < n; ++t) {
    tile(st);
    step_compute_cursor();
    PC_WAIT_VMCNT(0);   // the share of tile t+1
    if (wave < NLD && t + 2 < n) request_next(st >= 1 ? st - 1 : NSTAGE - 1);
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    st = st + 1 == NSTAGE ? 0 : st + 1;
  }

  const float l_tot = pair_sum(l_run);
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
    __bf16 *po = part_o + prow * D;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        pc::bf16x4 v = {(__bf16)(o_acc[db][q4 * 4 + 0] * inv), (__bf16)(o_acc[db][q4 * 4 + 1] * inv),
                        (__bf16)(o_acc[db][q4 * 4 + 2] * inv), (__bf16)(o_acc[db][q4 * 4 + 3] * inv)};
        *(pc::bf16x4 *)(po + db * 32 + q4 * 8 + g2 * 4) = v;
      }
    if (g2 == 0) {
      part_ml[prow * 2] = m_ref;
      part_ml[prow * 2 + 1] = l_tot;
    }
  }
}

// The long-context kernel over 8-bit slots (every chunk of the launch in an 8-bit slot; head size 128; at most 32 tiles
// per chunk).  Cached tiles arrive as codes (16 KB instead of 32) in a ring of three code stages; one tile ahead of the
// arithmetic the workgroup turns a tile's codes into the bf16 tile layout of the bf16 kernel ONCE -- every thread 16 K
// codes and 16 V codes, exact (power-of-two scales) -- into one of two bf16 stages, so the tile arithmetic is that of
// the bf16 kernel and no wavefront converts what another one converts too (with every wavefront converting the whole
// tile for itself the vector port was the busiest unit: 256 conversions per tile and wavefront).  The fresh tiles are
// bf16 already and are requested straight into their bf16 stage.  The converted values are stored with ds_write
// instructions the compiler does not see as stores to the LDS array: with ordinary stores to it, it waits for every
// outstanding request before each operand read.
template <int D>
__global__ __launch_bounds__(512, 2) void reuse_attention_wide8_kernel(
    const __bf16 *__restrict__ Q, const __bf16 *__restrict__ Kf, const __bf16 *__restrict__ Vf_blk,
    const uint8_t *__restrict__ k_store, const uint8_t *__restrict__ v_store, const float *__restrict__ k_scale,
    const float *__restrict__ v_scale, int n_slots16, const int32_t *__restrict__ table,
    int tbl_stride, int T, int Hq, int Hkv, int C, int n_splits, int q_tiles, int n_groups, float scale_log2e,
    __bf16 *__restrict__ out, __bf16 *__restrict__ part_o, float *__restrict__ part_ml) {
  using L = Lds<D>;
  constexpr int NW = 8, NLD = 4, KS = D / 16, DB = D / 32, QROWS = 32 * NW;
  constexpr int K8_ROW = D, V8_ROW = TK, K8_BYTES = TK * K8_ROW, V8_BYTES = D * V8_ROW, CST = K8_BYTES + V8_BYTES, NCST = 3;
  static_assert(D == 128, "one 16-byte code chunk per thread and tile half");
  __shared__ __align__(16) char lds[2 * L::STAGE + NCST * CST];
  char *const codes = lds + 2 * L::STAGE;

  const int xcd = blockIdx.x & 7, jj0 = blockIdx.x >> 3;
  const int sg = (jj0 / q_tiles) * 8 + xcd, qt = jj0 % q_tiles;
  if (sg >= n_groups) return;
  const int split = sg % n_splits, bg = sg / n_splits;
  const int gkv = bg % Hkv, b = bg / Hkv;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, g2 = lane >> 5;
  const int G = Hq / Hkv, R = G * T;

  // chunk list: lane c keeps (slot, used length) of chunk c (at most 64 chunks)
  const int32_t *trow = table + (size_t)b * tbl_stride;
  int my_slot = 0, my_used = 0;
  if (lane < (tbl_stride - kTblHeader) / 2) {
    const int2 e = *(const int2 *)(trow + kTblHeader + 2 * lane);
    my_slot = e.x;
    my_used = e.y;
  }
  const int n_chunks = trow[0];
  const int n_cached_tiles = trow[2];
  if (lane >= n_chunks) my_used = 0;
  const unsigned long long live = __ballot(my_used > 0);

  const int row_first = qt * QROWS;
  const int row_last = min(row_first + QROWS, R) - 1;
  const int i_max = (row_first / T == row_last / T) ? (row_last % T) : (T - 1);
  const int n_tiles = n_cached_tiles + i_max / TK + 1;
  const int tile_begin = (int)((long)split * n_tiles / n_splits);
  const int tile_end = (int)((long)(split + 1) * n_tiles / n_splits);
  const int n = tile_end - tile_begin;

  const int my_row = row_first + wave * 32 + l32;
  const bool row_ok = my_row < R;
  const int row_c = row_ok ? my_row : R - 1;   // (wavefronts past the last row compute on the last row and write nothing)
  const int hg = row_c / T, my_i = row_c - hg * T;
  const int head = gkv * G + hg;

  bf16x8 qf[KS];
  {
    const __bf16 *qrow = Q + (((size_t)b * Hq + head) * T + my_i) * D;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[ks] = *(const bf16x8 *)(qrow + ks * 16 + g2 * 8);
  }
  f32x16 o_acc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) o_acc[db][r] = 0.f;
  float m_ref = -INFINITY, l_run = 0.f;
  bool all_started = false;

  const int ft = (T + TK - 1) / TK;
  const char *const kf_base = (const char *)(Kf + ((size_t)b * Hkv + gkv) * T * D);
  const char *const vf_base = (const char *)(Vf_blk + ((size_t)b * Hkv + gkv) * ft * (size_t)(TK * D));
  auto next_live = [&](int chunk) __attribute__((always_inline)) {
    const unsigned long long rest = chunk < 63 ? live >> (chunk + 1) : 0ull;
    return rest ? chunk + 1 + (int)__builtin_ctzll(rest) : n_chunks;
  };
  // where the range starts: chunk `first` (n_chunks: the fresh part), tile `off0` inside it
  int first, off0;
  {
    const int my_tiles = (my_used + TK - 1) / TK;
    int incl = my_tiles;
#pragma unroll
    for (int sh = 1; sh < 64; sh <<= 1) {
      const int up = __shfl_up(incl, sh, 64);
      if (lane >= sh) incl += up;
    }
    first = __popcll(__ballot(incl <= tile_begin && lane < n_chunks));   // chunks wholly before tile_begin
    const int before = __builtin_amdgcn_readlane(incl - my_tiles, min(first, 63));
    off0 = first < n_chunks ? tile_begin - before : tile_begin - n_cached_tiles;
  }

  // ---- the loading wavefronts' cursor over the CACHED tiles of the range (byte pointers into the 8-bit stores); it
  // stops at the fresh part, whose tiles are addressed by their index
  const char *c_k = nullptr, *c_v = nullptr;
  int c_chunk = first, c_rem = 0;   // c_chunk == n_chunks: no cached tile left
  auto enter_chunk = [&](int chunk) __attribute__((always_inline)) {
    c_chunk = chunk;
    if (chunk < n_chunks) {
      const int slot = __builtin_amdgcn_readlane(my_slot, chunk) - n_slots16;   // (every chunk of this launch sits in an 8-bit slot)
      const size_t cbase = ((size_t)slot * Hkv + gkv) * C * (size_t)D;
      c_k = (const char *)k_store + cbase;
      c_v = (const char *)v_store + cbase;
      c_rem = __builtin_amdgcn_readlane(my_used, chunk);
    }
  };
  enter_chunk(first);
  if (first < n_chunks) {
    c_k += (size_t)off0 * (TK * D);
    c_v += (size_t)off0 * (TK * D);
    c_rem -= off0 * TK;
  }
  // request instructions of this lane: code tiles (two K and two V instructions per loading wavefront) and bf16 tiles
  constexpr int K8_INSTR = K8_BYTES / 1024 / NLD, V8_INSTR = V8_BYTES / 1024 / NLD;
  constexpr int K_INSTR = L::K_BYTES / 1024 / NLD, V_INSTR = L::V_BYTES / 1024 / NLD;
  auto swz8 = [](int row_bytes, int row) { return row_bytes == 128 ? ((row >> 1) & 7) : ((row >> 2) & 3); };
  unsigned k8_off[K8_INSTR], v8_off[V8_INSTR];
#pragma unroll
  for (int k = 0; k < K8_INSTR; ++k) {
    const int byte = ((wave & (NLD - 1)) + k * NLD) * 1024 + lane * 16;
    const int row = byte / K8_ROW, pc = (byte % K8_ROW) / 16;
    k8_off[k] = (unsigned)(row * K8_ROW + (pc ^ swz8(K8_ROW, row)) * 16);
  }
#pragma unroll
  for (int k = 0; k < V8_INSTR; ++k) {
    const int byte = ((wave & (NLD - 1)) + k * NLD) * 1024 + lane * 16;
    const int d = byte / V8_ROW, pc = (byte % V8_ROW) / 16;
    v8_off[k] = (unsigned)(d * V8_ROW + (pc ^ swz8(V8_ROW, d)) * 16);
  }
  // the cursor's tile of codes into code stage cs; steps the cursor (wavefronts 0..3; call only while a cached tile is left)
  auto request_codes = [&](int cs) __attribute__((always_inline)) {
    char *dst = codes + cs * CST;
    const int valid = min(TK, c_rem);
#pragma unroll
    for (int k = 0; k < K8_INSTR; ++k) {
      unsigned o = k8_off[k];
      if (__builtin_expect(valid < TK, 0)) {   // rows past a ragged end repeat the last valid row (masked later)
        int lane_v = lane;
        asm volatile("" : "+v"(lane_v));   // (recomputed here so that nothing of it stays in registers across the loop)
        const int byte = ((wave & (NLD - 1)) + k * NLD) * 1024 + lane_v * 16;
        const int row = byte / K8_ROW, pc = (byte % K8_ROW) / 16;
        o = (unsigned)(min(row, valid - 1) * K8_ROW + (pc ^ swz8(K8_ROW, row)) * 16);
      }
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(c_k + o),
                                       (__attribute__((address_space(3))) void *)(dst + (wave + k * NLD) * 1024), 16, 0, kKvAux);
    }
#pragma unroll
    for (int k = 0; k < V8_INSTR; ++k)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(c_v + v8_off[k]),
                                       (__attribute__((address_space(3))) void *)(dst + K8_BYTES + (wave + k * NLD) * 1024), 16, 0, kKvAux);
    c_k += TK * D;
    c_v += TK * D;
    c_rem -= TK;
    if (__builtin_expect(c_rem <= 0, 0)) enter_chunk(next_live(c_chunk));
  };
  // fresh tile fi (first token fi * TK) into bf16 stage st (wavefronts 0..3)
  auto request_fresh = [&](int fi, int st) __attribute__((always_inline)) {
    char *kb = lds + st * L::STAGE;
    const int valid = min(TK, T - fi * TK);
    const char *kp = kf_base + (size_t)fi * (TK * D * 2), *vp = vf_base + (size_t)fi * (TK * D * 2);
#pragma unroll
    for (int k = 0; k < K_INSTR; ++k) {
      const int byte = ((wave & (NLD - 1)) + k * NLD) * 1024 + lane * 16;
      const int row = byte / L::K_ROW, pc = (byte % L::K_ROW) / 16;
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(kp + (unsigned)(min(row, valid - 1) * D + (pc ^ swz<L::K_ROW>(row)) * 8) * 2u),
                                       (__attribute__((address_space(3))) void *)(kb + (wave + k * NLD) * 1024), 16, 0, kKvAux);
    }
#pragma unroll
    for (int k = 0; k < V_INSTR; ++k) {
      const int byte = ((wave & (NLD - 1)) + k * NLD) * 1024 + lane * 16;
      const int d = byte / L::V_ROW, pc = (byte % L::V_ROW) / 16;
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(vp + (unsigned)(d * TK + (pc ^ swz<L::V_ROW>(d)) * 8) * 2u),
                                       (__attribute__((address_space(3))) void *)(kb + L::K_BYTES + (wave + k * NLD) * 1024), 16, 0, kKvAux);
    }
  };

  // ---- every wavefront's cursor over ALL tiles of the range, one tile ahead of the arithmetic: is the tile cached,
  // how many of its keys are valid, its place in its chunk and the chunk's scales: lane j < 32 holds the K scale of the
  // chunk's tile j, lane 32 + j its V scale; the scales of the chunk after this one are requested when this one is entered
  const int tpc = C / TK;
  auto chunk_scales = [&](int chunk) __attribute__((always_inline)) {
    float v = 1.f;
    if (chunk < n_chunks) {
      const int slot = __builtin_amdgcn_readlane(my_slot, min(chunk, 63)) - n_slots16;
      const size_t base = ((size_t)slot * Hkv + gkv) * tpc;
      if ((lane & 31) < tpc) v = (lane < 32 ? k_scale : v_scale)[base + (lane & 31)];
    }
    return v;
  };
  int r_chunk = first, r_off = off0;
  int r_rem = first < n_chunks ? __builtin_amdgcn_readlane(my_used, min(first, 63)) - off0 * TK : T - off0 * TK;
  int r_t0 = first < n_chunks ? -1 : off0 * TK;
  float sc_cur = chunk_scales(r_chunk), sc_nxt = chunk_scales(next_live(r_chunk));
  auto step_ready_cursor = [&]() __attribute__((always_inline)) {
    r_rem -= TK;
    r_off += 1;
    if (r_t0 >= 0) r_t0 += TK;
    if (__builtin_expect(r_rem <= 0 && r_t0 < 0, 0)) {
      r_chunk = next_live(r_chunk);
      const bool cached = r_chunk < n_chunks;
      r_rem = cached ? __builtin_amdgcn_readlane(my_used, min(r_chunk, 63)) : T;
      r_t0 = cached ? -1 : 0;
      r_off = 0;
      sc_cur = sc_nxt;
      sc_nxt = chunk_scales(next_live(r_chunk));
    }
  };
  // operand reads of the tile arithmetic (bf16 tile layout)
  int k_rd[KS], v_rd[4];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) k_rd[ks] = ((2 * ks + g2) ^ swz<L::K_ROW>(l32)) * 16;
#pragma unroll
  for (int c4 = 0; c4 < 4; ++c4) v_rd[c4] = ((2 * c4 + g2) ^ swz<L::V_ROW>(l32)) * 16;
  // conversion share of this thread: K row tid / 8, code chunk tid % 8 (elements 16 c .. 16 c + 15 -> bf16 chunks 2c, 2c + 1);
  // V^T row tid / 4, code chunk m = tid % 4 = 2 J + a (byte p of a row holds the key that the bf16 block holds at
  // element p with bits 3 and 4 swapped: the chunk's first 8 codes are bf16 chunk 4 J + a, its last 8 chunk 4 J + 2 + a)
  const int ck_row = tid >> 3, ck_c = tid & 7, cv_row = tid >> 2, cv_m = tid & 3;
  const int ck_src = ck_row * K8_ROW + ((ck_c ^ swz8(K8_ROW, ck_row)) * 16);
  const int cv_src = K8_BYTES + cv_row * V8_ROW + ((cv_m ^ swz8(V8_ROW, cv_row)) * 16);
  const int ck_dst0 = ck_row * L::K_ROW + (((2 * ck_c) ^ swz<L::K_ROW>(ck_row)) * 16);
  const int ck_dst1 = ck_row * L::K_ROW + (((2 * ck_c + 1) ^ swz<L::K_ROW>(ck_row)) * 16);
  const int cv_dst0 = L::K_BYTES + cv_row * L::V_ROW + (((4 * (cv_m >> 1) + (cv_m & 1)) ^ swz<L::V_ROW>(cv_row)) * 16);
  const int cv_dst1 = L::K_BYTES + cv_row * L::V_ROW + (((4 * (cv_m >> 1) + 2 + (cv_m & 1)) ^ swz<L::V_ROW>(cv_row)) * 16);
  const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) char *)lds;
  auto store16 = [&](int byte_off, bf16x8 v) __attribute__((always_inline)) {
    const unsigned addr = lds_base + (unsigned)byte_off;
    asm volatile("ds_write_b128 %0, %1" : : "v"(addr), "v"(v) : "memory");
  };
  // makes the tile the ready cursor points at ready in bf16 stage st: converts its codes (from code stage cs) or, for a
  // fresh tile, requests it; returns with the cursor's (valid keys, first fresh token or -1) in the two references
  auto make_ready = [&](int cs, int st, int &valid_out, int &t0_out) __attribute__((always_inline)) {
    valid_out = min(TK, r_rem);
    t0_out = r_t0;
    if (r_t0 < 0) {
      const float ks8 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, sc_cur), r_off));
      const float vs8 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, sc_cur), 32 + r_off));
      const char *src = codes + cs * CST;
      const pc::u32x4 kr = *(const pc::u32x4 *)(src + ck_src), vr = *(const pc::u32x4 *)(src + cv_src);
      store16(st * L::STAGE + ck_dst0, codes_to_bf16(kr[0], kr[1], ks8));
      store16(st * L::STAGE + ck_dst1, codes_to_bf16(kr[2], kr[3], ks8));
      store16(st * L::STAGE + cv_dst0, codes_to_bf16(vr[0], vr[1], vs8));
      store16(st * L::STAGE + cv_dst1, codes_to_bf16(vr[2], vr[3], vs8));
    } else if (wave < NLD) {
      request_fresh(r_t0 / TK, st);
    }
    step_ready_cursor();
  };
  int m_valid = TK, m_t0 = -1;   // of the tile the arithmetic is on

  auto tile = [&](int st) __attribute__((always_inline)) {
    const char *kb = lds + st * L::STAGE;
    const char *vb = kb + L::K_BYTES;
    f32x16 s_acc[2];
#pragma unroll
    for (int kbk = 0; kbk < 2; ++kbk)
#pragma unroll
      for (int r = 0; r < 16; ++r) s_acc[kbk][r] = 0.f;
#pragma unroll
    for (int h = 0; h < KS / 4; ++h) {
      bf16x8 kop[2][4];
#pragma unroll
      for (int k4 = 0; k4 < 4; ++k4)
#pragma unroll
        for (int kbk = 0; kbk < 2; ++kbk) kop[kbk][k4] = *(const bf16x8 *)(kb + (kbk * 32 + l32) * L::K_ROW + k_rd[4 * h + k4]);
#pragma unroll
      for (int k4 = 0; k4 < 4; ++k4)
#pragma unroll
        for (int kbk = 0; kbk < 2; ++kbk)
          s_acc[kbk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kop[kbk][k4], qf[4 * h + k4], s_acc[kbk], 0, 0, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
    }
    // V operands of the first 32-key block: their LDS latency runs under the softmax arithmetic
    bf16x8 vop0[DB][2];
#pragma unroll
    for (int c2 = 0; c2 < 2; ++c2)
#pragma unroll
      for (int db = 0; db < DB; ++db) vop0[db][c2] = *(const bf16x8 *)(vb + (db * 32 + l32) * L::V_ROW + v_rd[c2]);
    const int t_valid = m_valid, t_t0 = m_t0;
    if (__builtin_expect(t_valid < TK || t_t0 >= 0, 0)) {
      int t_lane = g2 * 4;
      asm volatile("" : "+v"(t_lane));   // (keeps the 32 per-element key indices out of loop-invariant registers)
      const int lim_valid = t_valid - t_lane;
      const int lim_causal = t_t0 >= 0 ? my_i - t_t0 - t_lane : 0x7fffff00;
#pragma unroll
      for (int kbk = 0; kbk < 2; ++kbk)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int c = kbk * 32 + (r >> 2) * 8 + (r & 3);
          s_acc[kbk][r] = (c < lim_valid && c <= lim_causal) ? s_acc[kbk][r] : -INFINITY;
        }
    }
    bf16x8 pf[2][2];
    auto exponentials = [&](float neg_m) __attribute__((always_inline)) {
      typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
      float sum = 0.f, sum2 = 0.f;
#pragma unroll
      for (int kbk = 0; kbk < 2; ++kbk)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int e = 0; e < 8; e += 2) {
            const float p0 = fast_exp2(__builtin_fmaf(s_acc[kbk][j * 8 + e], scale_log2e, neg_m));
            const float p1 = fast_exp2(__builtin_fmaf(s_acc[kbk][j * 8 + e + 1], scale_log2e, neg_m));
            const bf16x2 pr = {(__bf16)p0, (__bf16)p1};
            pf[kbk][j][e] = pr[0];
            pf[kbk][j][e + 1] = pr[1];
            sum += p0;
            sum2 += p1;
          }
      return sum + sum2;
    };
    float psum = 0.f;
    bool refresh = !all_started;
    if (__builtin_expect(!refresh, 1)) {
      psum = exponentials(-m_ref);
      refresh = __builtin_amdgcn_ballot_w64(!(psum <= kSumLimit)) != 0;   // also catches inf / nan
    }
    if (__builtin_expect(refresh, 0)) {
      float mx = s_acc[0][0];
#pragma unroll
      for (int kbk = 0; kbk < 2; ++kbk)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s_acc[kbk][r]);
      const float mc = pair_max(mx) * scale_log2e;
      const bool upd = mc > m_ref;
      const float alpha = upd ? fast_exp2(m_ref - mc) : 1.0f;
      m_ref = upd ? mc : m_ref;
      l_run *= alpha;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o_acc[db][r] *= alpha;
      psum = exponentials((m_ref == -INFINITY) ? 0.f : -m_ref);
      all_started = __builtin_amdgcn_ballot_w64(m_ref == -INFINITY) == 0;
    }
    l_run += psum;
    bf16x8 vop1[DB][2];
#pragma unroll
    for (int c2 = 0; c2 < 2; ++c2)
#pragma unroll
      for (int db = 0; db < DB; ++db) vop1[db][c2] = *(const bf16x8 *)(vb + (db * 32 + l32) * L::V_ROW + v_rd[2 + c2]);
#pragma unroll
    for (int c2 = 0; c2 < 2; ++c2)
#pragma unroll
      for (int db = 0; db < DB; ++db)
        o_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vop0[db][c2], pf[0][c2], o_acc[db], 0, 0, 0);
#pragma unroll
    for (int c2 = 0; c2 < 2; ++c2)
#pragma unroll
      for (int db = 0; db < DB; ++db)
        o_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vop1[db][c2], pf[1][c2], o_acc[db], 0, 0, 0);
    __builtin_amdgcn_sched_group_barrier(0x100, 2 * DB, 1);
    __builtin_amdgcn_sched_group_barrier(0x008, 4 * DB, 1);
  };

  // ---- pipeline.  Iteration t: make tile t+1 ready in bf16 stage (t+1) & 1 (its codes were requested two iterations
  // ago and published by the last barrier; that stage was last read in iteration t-1), run the arithmetic on tile t in
  // stage t & 1, then wait for everything this wavefront has in flight (codes of tile t+2, a fresh tile t+1, its own
  // converted stores), request the codes of tile t+3 into the code stage that iteration t-1 emptied, barrier.
  int n_cached_left = 0;   // cached tiles of the range not requested yet (loading wavefronts)
  {
    const int cached_total = first < n_chunks ? min(n, n_cached_tiles - tile_begin) : 0;
    n_cached_left = cached_total;
  }
  if (wave < NLD) {
#pragma unroll
    for (int i = 0; i < NCST; ++i)
      if (n_cached_left > 0) { request_codes(i); --n_cached_left; }
  }
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(qf[ks]));
  __builtin_amdgcn_s_waitcnt(0);
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  int nx_valid = TK, nx_t0 = -1;
  if (n > 0) make_ready(0, 0, nx_valid, nx_t0);
  __builtin_amdgcn_s_waitcnt(0);
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  int cs = 1;   // code stage of tile t+1
  for (int t = 0; t < n; ++t) {
    m_valid = nx_valid;
    m_t0 = nx_t0;
    if (t + 1 < n) make_ready(cs, (t + 1) & 1, nx_valid, nx_t0);
    tile(t & 1);
    __builtin_amdgcn_s_waitcnt(0);
    // the code stage of tile t (emptied at the top of iteration t-1, or in the prologue) takes tile t+3
    if (wave < NLD && n_cached_left > 0) { request_codes(cs >= 1 ? cs - 1 : NCST - 1); --n_cached_left; }
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    cs = cs + 1 == NCST ? 0 : cs + 1;
  }

  const float l_tot = pair_sum(l_run);
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
    __bf16 *po = part_o + prow * D;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        pc::bf16x4 v = {(__bf16)(o_acc[db][q4 * 4 + 0] * inv), (__bf16)(o_acc[db][q4 * 4 + 1] * inv),
                        (__bf16)(o_acc[db][q4 * 4 + 2] * inv), (__bf16)(o_acc[db][q4 * 4 + 3] * inv)};
        *(pc::bf16x4 *)(po + db * 32 + q4 * 8 + g2 * 4) = v;
      }
    if (g2 == 0) {
      part_ml[prow * 2] = m_ref;
      part_ml[prow * 2 + 1] = l_tot;
    }
  }
}

// Merge of the split-KV partials: m = max m_s, w_s = l_s 2^(m_s - m), o = sum w_s o_s / sum w_s.
// A row is shared by 4 * D/8 neighbouring lanes: lane (sg, dv) adds up 8 head-dim elements over the partitions
// s = sg, sg + 4, ..., and the four partial sums meet through lane shuffles.
// FEW (at most four partitions): one lane per 16 output bytes takes all of them, four independent loads in flight,
// and adds them up in the order the shuffles would, (0 + 1) + (2 + 3), so both forms give the same bits.
template <int D, bool FEW>
__global__ __launch_bounds__(256) void splitkv_combine_kernel(const __bf16 *__restrict__ part_o,
                                                              const float *__restrict__ part_ml, int n_splits, int T,
                                                              int Hq, int Hkv, long total_rows,
                                                              __bf16 *__restrict__ out) {
  constexpr int VPR = D / 8, SG = FEW ? 1 : 4, LPR = VPR * SG;  // lanes per row
  const long gid = (long)blockIdx.x * blockDim.x + threadIdx.x;
  const long prow_raw = gid / LPR;
  const int r = (int)(gid - prow_raw * LPR);
  const int sg = r / VPR, dv = r - sg * VPR;
  const bool live = prow_raw < total_rows;
  const long prow = live ? prow_raw : total_rows - 1;
  const float2 *ml = (const float2 *)part_ml + prow * n_splits;
  const __bf16 *po = part_o + prow * n_splits * D + dv * 8;
  float wsum = 0.f;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if constexpr (FEW) {
#pragma clang fp contract(off)  // products rounded before the sums, as in the other form
    float2 e[4];
    pc::bf16x8 o[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const int sc = s < n_splits ? s : 0;
      e[s] = ml[sc];
      o[s] = *(const pc::bf16x8 *)(po + (size_t)sc * D);
      if (s >= n_splits) e[s].y = 0.f;
    }
    float m = -INFINITY;
#pragma unroll
    for (int s = 0; s < 4; ++s) m = fmaxf(m, e[s].y > 0.f ? e[s].x : -INFINITY);
    float w[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) w[s] = e[s].y > 0.f ? e[s].y * exp2f(e[s].x - m) : 0.f;
    wsum = (w[0] + w[1]) + (w[2] + w[3]);
#pragma unroll
    for (int e8 = 0; e8 < 8; ++e8)
      acc[e8] = (w[0] * (float)o[0][e8] + w[1] * (float)o[1][e8]) + (w[2] * (float)o[2][e8] + w[3] * (float)o[3][e8]);
  } else {
  float m = -INFINITY;
#pragma unroll 4
  for (int s = sg; s < n_splits; s += SG) {
    const float2 e = ml[s];
    m = fmaxf(m, e.y > 0.f ? e.x : -INFINITY);
  }
  m = fmaxf(m, __shfl_xor(m, VPR, 64));
  m = fmaxf(m, __shfl_xor(m, 2 * VPR, 64));
#pragma unroll 4
  for (int s = sg; s < n_splits; s += SG) {
    const float2 e = ml[s];
    const float w = e.y > 0.f ? e.y * exp2f(e.x - m) : 0.f;  // an empty partition has weight 0 (its output row is 0)
    pc::bf16x8 o = *(const pc::bf16x8 *)(po + (size_t)s * D);
#pragma unroll
    for (int e8 = 0; e8 < 8; ++e8) acc[e8] += w * (float)o[e8];
    wsum += w;
  }
#pragma unroll
  for (int sh = VPR; sh < LPR; sh <<= 1) {
    wsum += __shfl_xor(wsum, sh, 64);
#pragma unroll
    for (int e8 = 0; e8 < 8; ++e8) acc[e8] += __shfl_xor(acc[e8], sh, 64);
  }
  }
  if (!live || sg != 0) return;
  const int G = Hq / Hkv, R = G * T;
  const long bg = prow / R;
  const int row = (int)(prow - bg * R);
  const int b = (int)(bg / Hkv), gkv = (int)(bg - (long)b * Hkv);
  const int hg = row / T, i = row - hg * T;
  const int head = gkv * G + hg;
  const float inv = wsum > 0.f ? 1.0f / wsum : 0.f;
  pc::bf16x8 v;
#pragma unroll
  for (int e8 = 0; e8 < 8; ++e8) v[e8] = (__bf16)(acc[e8] * inv);
  *(pc::bf16x8 *)(out + ((size_t)b * T + i) * ((size_t)Hq * D) + (size_t)head * D + dv * 8) = v;
}

// Fresh V [B*Hkv][T][D] -> 64-key blocks [B*Hkv][ceil(T/64)][D][64] in the key order of the store
// (see kvstore.hip: blocked_pos), zero filled past T.  One thread per 16 output bytes.
__global__ __launch_bounds__(256) void v_block_repack_kernel(const __bf16 *__restrict__ v, __bf16 *__restrict__ vb, int T,
                                                             int D, long total_vec) {
  long gid = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= total_vec) return;
  const int ft = (T + TK - 1) / TK;
  int chunk = (int)(gid & 7);
  long r = gid >> 3;
  int d = (int)(r % D);
  r /= D;
  int tile = (int)(r % ft);
  long bg = r / ft;
  pc::bf16x8 o;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    int pos = chunk * 8 + e;
    int t = tile * TK + (pos & ~15) + pc::blocked_key(pos & 15);
    o[e] = t < T ? v[((size_t)bg * T + t) * D + d] : (__bf16)0.f;
  }
  *(pc::bf16x8 *)(vb + gid * 8) = o;
}

}  // namespace

namespace pc {

int choose_splits(int slots_in, long base_wgs, int min_tiles, int cap) {
  const long slots = slots_in;  // workgroups resident at once on the whole chip
  int best = 1;
  double best_eff = 0.0;
  for (int ns = 1; ns <= cap; ++ns) {
    if (ns > 1 && min_tiles / ns < 4) break;  // keep at least 4 tiles per partition
    long w = base_wgs * ns;
    double eff = (double)w / (double)(((w + slots - 1) / slots) * slots);
    if (eff > best_eff + 0.03) { best_eff = eff; best = ns; }
  }
  return best;
}

pc_status launch_v_repack(percache_ctx *ctx, const __bf16 *vf, __bf16 *vf_blk, int batch, int t_fresh, hipStream_t stream) {
  const percache_config &c = ctx->cfg;
  const int ft = (t_fresh + TK - 1) / TK;
  long total_vec = (long)batch * c.n_kv_heads * ft * c.head_dim * (TK / 8);
  hipLaunchKernelGGL(v_block_repack_kernel, dim3((unsigned)((total_vec + 255) / 256)), dim3(256), 0, stream, vf, vf_blk,
                     t_fresh, c.head_dim, total_vec);
  PC_HIP(ctx, hipGetLastError());
  return PC_OK;
}

pc_status launch_attention(percache_ctx *ctx, int layer, const __bf16 *q, const __bf16 *kf, const __bf16 *vf_blk,
                           int batch, int t_fresh, const int32_t *table_dev, int tbl_stride, int min_tiles,
                           int n_splits, __bf16 *out, __bf16 *part_o, float *part_ml, hipStream_t stream, int formats) {
  const percache_config &c = ctx->cfg;
  const int G = c.n_q_heads / c.n_kv_heads, R = G * t_fresh;
  // the kernels that can read 8-bit tiles are taken only when the call names a chunk in an 8-bit slot, and their
  // variant that tells the formats apart tile by tile only when it names chunks of both formats
  const bool use8 = (formats & 1) && ctx->n_slots8 > 0;
  const bool mixed = use8 && (formats & 2);
  // 8 wavefronts x 32 rows (one workgroup per CU) once a kv head has more than 128 stacked rows, else 4 wavefronts
  // (two workgroups per CU); two LDS stages at D = 128, four at D = 64.
  // 256-row workgroups only when there are enough of them to go round; few, short key ranges prefer more, smaller ones
  // (8-bit slots with D = 64: a tile is too small for eight wavefronts to load)
  const bool wide = R > 128 && (long)batch * c.n_kv_heads * ((R + 255) / 256) * 4 >= ctx->n_cu && !(use8 && c.head_dim == 64);
  // at most 32 rows per kv head (decoding steps) over 8-bit slots: two wavefronts share the rows and halve every
  // tile between them.  (Over bf16 slots such a step is bound by the key stream already, and the 4-wavefront kernel
  // with its three loader wavefronts measures 3 % faster.)
  const bool few = R <= 32 && use8;
  // few workgroups for the whole chip (one or two short queries): 64-row workgroups whose wavefront pairs halve every
  // tile between them -- twice the workgroups, half the dependent chain per tile
  const bool halved = !wide && !few && !use8 && c.head_dim == 128 && R > 32 &&
                      (long)batch * c.n_kv_heads * ((R + 63) / 64) * 4 <= ctx->n_cu;
  const int qrows = few ? 32 : wide ? 256 : halved ? 64 : 128;
  const int q_tiles = (R + qrows - 1) / qrows;
  const int cap = max_splits_for(c, ctx->n_cu, batch, t_fresh);
  if (n_splits <= 0) n_splits = choose_splits(wide ? ctx->n_cu : 2 * ctx->n_cu, (long)batch * c.n_kv_heads * q_tiles, min_tiles, cap);
  if (n_splits > cap) n_splits = cap;
  const void *ks, *vs;
  const float *ksc = nullptr, *vsc = nullptr;
  const __bf16 *k16 = ctx->k_store + (size_t)layer * ctx->layer_stride, *v16 = ctx->v_store + (size_t)layer * ctx->layer_stride;
  if (use8) {
    ks = ctx->k8_store + (size_t)layer * ctx->layer_stride8;
    vs = ctx->v8_store + (size_t)layer * ctx->layer_stride8;
    const size_t sc_layer = (size_t)ctx->n_slots8 * c.n_kv_heads * (c.slot_capacity / TK);
    ksc = ctx->k_scale + (size_t)layer * sc_layer;
    vsc = ctx->v_scale + (size_t)layer * sc_layer;
  } else {
    ks = k16;
    vs = v16;
  }
  const float scale_log2e = 1.4426950408889634f / sqrtf((float)c.head_dim);
  const int n_groups = batch * c.n_kv_heads * n_splits;
  dim3 grid((unsigned)(((n_groups + 7) / 8) * 8 * q_tiles));
  prof_begin(ctx, PC_KERNEL_ATTENTION, stream);
#define PC_ATTN(DD, NWW, NS, ...)                                                                                     \
  hipLaunchKernelGGL((reuse_attention_kernel<DD, NWW, NS, ##__VA_ARGS__>), grid, dim3(64 * NWW), 0, stream, q, kf,     \
                     vf_blk, ks, vs, ksc, vsc, k16, v16, ctx->n_slots16, table_dev, tbl_stride, t_fresh, c.n_q_heads, c.n_kv_heads, \
                     c.slot_capacity, n_splits, q_tiles, n_groups, scale_log2e, out, part_o, part_ml)
  if (use8 && mixed) {
    if (c.head_dim == 128) {
      if (few) PC_ATTN(128, 2, 2, true, 2, true); else if (wide) PC_ATTN(128, 8, 2, true, 1, true); else PC_ATTN(128, 4, 2, true, 1, true);
    } else {
      if (few) PC_ATTN(64, 2, 2, true, 2, true); else PC_ATTN(64, 4, 2, true, 1, true);
    }
  } else if (use8 && c.head_dim == 128 && wide && (tbl_stride - kTblHeader) / 2 <= 64 && c.slot_capacity / TK <= 32) {
    hipLaunchKernelGGL((reuse_attention_wide8_kernel<128>), grid, dim3(512), 0, stream, q, kf, vf_blk, (const uint8_t *)ks,
                       (const uint8_t *)vs, ksc, vsc, ctx->n_slots16, table_dev, tbl_stride, t_fresh, c.n_q_heads, c.n_kv_heads,
                       c.slot_capacity, n_splits, q_tiles, n_groups, scale_log2e, out, part_o, part_ml);
  } else if (use8) {
    if (c.head_dim == 128) {
      if (few) PC_ATTN(128, 2, 2, true, 2); else if (wide) PC_ATTN(128, 8, 2, true); else PC_ATTN(128, 4, 2, true);
    } else {
      if (few) PC_ATTN(64, 2, 2, true, 2); else PC_ATTN(64, 4, 2, true);
    }
  } else if (c.head_dim == 128 && wide && (tbl_stride - kTblHeader) / 2 <= 64) {
    hipLaunchKernelGGL((reuse_attention_wide_kernel<128>), grid, dim3(512), 0, stream, q, kf, vf_blk, k16, v16, table_dev,
                       tbl_stride, t_fresh, c.n_q_heads, c.n_kv_heads, c.slot_capacity, n_splits, q_tiles, n_groups,
                       scale_log2e, out, part_o, part_ml);
  } else if (c.head_dim == 128) {
    if (wide) PC_ATTN(128, 8, 2); else if (halved) PC_ATTN(128, 4, 2, false, 2); else PC_ATTN(128, 4, 2);
  } else if (wide && (tbl_stride - kTblHeader) / 2 <= 64) {
    hipLaunchKernelGGL((reuse_attention_wide_kernel<64>), grid, dim3(512), 0, stream, q, kf, vf_blk, k16, v16, table_dev,
                       tbl_stride, t_fresh, c.n_q_heads, c.n_kv_heads, c.slot_capacity, n_splits, q_tiles, n_groups,
                       scale_log2e, out, part_o, part_ml);
  } else {
    if (wide) PC_ATTN(64, 8, 4); else PC_ATTN(64, 4, 4);
  }
#undef PC_ATTN
  prof_end(ctx, PC_KERNEL_ATTENTION, stream);
  PC_HIP(ctx, hipGetLastError());
  if (n_splits > 1) {
    long total_rows = (long)batch * c.n_kv_heads * R;
    const bool few_parts = n_splits <= 4;              // one lane per 16 output bytes, else four
    long threads = total_rows * (c.head_dim / 8) * (few_parts ? 1 : 4);
    int blocks = (int)((threads + 255) / 256);
#define PC_COMBINE(DD, FF)                                                                                          \
  hipLaunchKernelGGL((splitkv_combine_kernel<DD, FF>), dim3(blocks), dim3(256), 0, stream, part_o, part_ml, n_splits, \
                     t_fresh, c.n_q_heads, c.n_kv_heads, total_rows, out)
    if (c.head_dim == 128) { if (few_parts) PC_COMBINE(128, true); else PC_COMBINE(128, false); }
    else { if (few_parts) PC_COMBINE(64, true); else PC_COMBINE(64, false); }
#undef PC_COMBINE
    PC_HIP(ctx, hipGetLastError());
  }
  return PC_OK;
}

}  // namespace pc
