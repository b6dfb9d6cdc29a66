// Host-side state shared by the translation units of libpercache (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <string>
#include <unordered_map>
#include <vector>

#include "percache.h"

namespace pc {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(8 * sizeof(_Float16)))) _Float16 f16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
// 16-byte register staging type (a native vector: arrays of it stay in registers)
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v, size_t a = kAlign) { return (v + a - 1) / a * a; }

// Key-axis tile of the attention kernel; the chunk table counts cached tiles in this unit.
constexpr int kKvTile = 64;

// V is stored (and handed to the attention kernel for the fresh part) in blocks of kKvTile keys laid out
// [head_dim][kKvTile]; inside each group of 16 keys, position p holds key blocked_key(p) -- the order in
// which the lanes of the 32x32 score accumulators hold keys ({0-3, 8-11} then {4-7, 12-15}).  The map is
// its own inverse.
__host__ __device__ inline int blocked_key(int p) { return 8 * ((p >> 2) & 1) + 4 * (p >> 3) + (p & 3); }

// 8-bit slots: V blocks are [head_dim][kKvTile] bytes; physical byte p of a row holds key blocked_key8(p).  A lane of
// the PV product reads 16 bytes = its 8 keys of two consecutive 16-key steps: p = 32 J + 16 g2 + 8 j + e  <->
// key 32 J + 16 j + 8 (e >> 2) + 4 g2 + (e & 3)  (J: 32-key score block, j: half of it, g2: lane half).
__host__ __device__ inline int blocked_key8(int p) {
  return (p & 32) + 16 * ((p >> 3) & 1) + 8 * ((p >> 2) & 1) + 4 * ((p >> 4) & 1) + (p & 3);
}
__host__ __device__ inline int blocked_pos8(int key) {  // the inverse: the byte that holds a key
  return (key & 32) + 16 * ((key >> 2) & 1) + 8 * ((key >> 4) & 1) + 4 * ((key >> 3) & 1) + (key & 3);
}

// Device chunk table, one row per query (int32):
//   [0] n_chunks  [1] L_pre  [2] cached tiles (sum over chunks of ceil(used/kKvTile))
//   [3] formats of the chunks with keys: bit 0 = some sit in 8-bit slots, bit 1 = some in bf16 slots
//   [4 + 2c] slot id of chunk c   [5 + 2c] used length of chunk c
constexpr int kTblHeader = 4;
inline int tbl_stride(int max_chunks) { return kTblHeader + 2 * (max_chunks > 0 ? max_chunks : 0); }

constexpr int kStageRing = 16;

// Size of the file-scope scratch array behind the entry points that allocate nothing.
constexpr size_t kStaticScratchBytes = 1u << 20;

}  // namespace pc

// Host copy of a chunk list that lives on the device (percache_chunk_table_put): what the table-taking calls validate
// against the slot table without reading device memory.
struct pc_table_shadow {
  int batch = 0, max_chunks = 0;
  std::vector<int32_t> ids, used, n_chunks;  // [batch * max_chunks], [batch * max_chunks] (resolved lengths), [batch]
  std::vector<int32_t> rows;                  // the device table's contents
};

struct percache_ctx {
  percache_config cfg;
  char *arena = nullptr;
  size_t arena_bytes = 0;
  // arena sub-regions
  float *rope = nullptr;      // [max_pos][D/2] float2 (cos, sin)
  _Float16 *bank = nullptr;   // [bank_capacity][emb_dim]
  float *bank_inv = nullptr;  // [bank_capacity]
  __bf16 *k_store = nullptr;  // [n_layers][n_slots16][Hkv][C][D]   (bf16 slots)
  __bf16 *v_store = nullptr;  // same
  uint8_t *k8_store = nullptr, *v8_store = nullptr;  // 8-bit slots: [n_layers][n_slots8][Hkv][C][D] bytes
  float *k_scale = nullptr, *v_scale = nullptr;      // 8-bit slots: 2^e per [n_layers][n_slots8][Hkv][C/64]
  size_t layer_stride = 0;    // elements per layer of the bf16 store (n_slots16 slots)
  size_t layer_stride8 = 0;   // bytes per layer of the 8-bit store (n_slots8 slots)
  size_t slot_stride = 0;     // elements per slot
  int n_slots16 = 0, n_slots8 = 0;  // slots [0, n_slots16) hold bf16, slots [n_slots16, n_slots) 8-bit codes
  bool is8(int slot) const { return slot >= n_slots16; }
  int32_t bank_size = 0;
  std::vector<int32_t> slot_len;  // [n_layers * n_slots], 0 = empty
  // pinned staging ring for chunk tables (host -> workspace copies ordered on the stream)
  int32_t *stage[pc::kStageRing] = {};
  hipEvent_t stage_ev[pc::kStageRing] = {};
  bool stage_used[pc::kStageRing] = {};
  size_t stage_ints = 0;
  int stage_next = 0;
  std::unordered_map<const void *, pc_table_shadow> tables;  // device chunk tables known to this context
  int n_cu = 256;
  // this device's copy of the library's file-scope scratch array (resolved once per device at create), for the
  // entry points that must not take a workspace
  void *static_scratch = nullptr;
  // optional kernel timing (event pairs per kernel kind)
  unsigned prof_mask = 0;  // bit k: launches of kernel kind k are bracketed by events
  std::vector<hipEvent_t> prof_beg[3], prof_end[3];
  int prof_n[3] = {0, 0, 0};
  std::string err;
};

namespace pc {

pc_status fail(percache_ctx *ctx, pc_status st, const char *fmt, ...);

#define PC_HIP(ctx, call)                                                              \
  do {                                                                                 \
    hipError_t e__ = (call);                                                           \
    if (e__ != hipSuccess)                                                             \
      return pc::fail((ctx), PC_EHIP, "%s: %s", #call, hipGetErrorString(e__));        \
  } while (0)

// Validates a chunk list against the host mirror of the slot table and writes the device
// table rows into `rows` (batch * tbl_stride ints).  No device work.
pc_status build_chunk_table(percache_ctx *ctx, int32_t layer, int32_t batch, int32_t t_fresh,
                            const int32_t *slot_ids, const int32_t *used_len, const int32_t *n_chunks,
                            int32_t max_chunks, std::vector<int32_t> &rows);
// Copies table rows to device memory through the pinned ring, ordered on `stream`.
pc_status upload_table(percache_ctx *ctx, const std::vector<int32_t> &rows, int32_t *dst_dev,
                       hipStream_t stream);

// The host copy of a device chunk table for a call on `batch` queries; nullptr (with the error set) if the table is
// unknown to the context or was built for another batch size.
const pc_table_shadow *find_table(percache_ctx *ctx, const void *table_dev, int32_t batch);

// Workspace carving for the prefill calls.
struct PrefillWs {
  int32_t *table;
  __bf16 *q, *k, *v;
  __bf16 *v_blk;   // fresh V as 64-key blocks [B*Hkv][ceil(T/64)][D][64]
  float *gemm_part;  // split-k slices of the QKV projection (few token rows only), else unused
  __bf16 *part_o;  // [rows][splits][D], normalised per split
  float *part_ml;  // [rows][splits][2]
  int max_splits;  // partitions of the key axis the partial buffers can hold
  size_t total;
};
constexpr int kMaxSplits = 64;
// Largest number of key-axis partitions ever used for this shape (the library's own choice never exceeds it).
int max_splits_for(const percache_config &cfg, int n_cu, int32_t batch, int32_t t_fresh);
PrefillWs carve_prefill_ws(const percache_config &cfg, int n_cu, void *base, int32_t batch, int32_t t_fresh,
                           int32_t max_chunks);

constexpr int kProfMax = 256;
// Record the begin / end event of launch number prof_n[kind] (no-ops unless profiling is on).
void prof_begin(percache_ctx *ctx, int kind, hipStream_t stream);
void prof_end(percache_ctx *ctx, int kind, hipStream_t stream);

// kernel launchers (defined in the .hip files)
// Model-family variants of the projection: bias [(Hq+2Hkv)*D] added before everything else; RMSNorm over the head
// dimension of every q / k head with gains [D] before RoPE.  Null pointers switch a part off.
struct QkvExtras {
  const __bf16 *bias = nullptr, *q_norm = nullptr, *k_norm = nullptr;
  float eps = 1e-6f;
  bool any() const { return bias || q_norm || k_norm; }
};
// gemm_part: workspace for the split-k path (nullptr: always the single-pass kernel)
// v_blk / v_blk_done: if given, the launch may also write V as the 64-key blocks of launch_v_repack and says so
pc_status launch_qkv_rope(percache_ctx *ctx, const __bf16 *x, const __bf16 *w, int batch, int t_fresh,
                          const int32_t *table_dev, int tbl_stride, __bf16 *q, __bf16 *k, __bf16 *v,
                          hipStream_t stream, float *gemm_part = nullptr, const QkvExtras &extras = QkvExtras(),
                          __bf16 *v_blk = nullptr, bool *v_blk_done = nullptr);

// Split-k projections for few token rows (see block.hip).  P[s][m][n] = sum over slice s of A[m][k] W[n][k];
// weight rows >= n_split come from w1.  Returns the number of slices written (chosen by choose_split_k).
constexpr int kMaxSplitK = 16;
inline bool splitk_applies(long M) { return M <= 192; }
int choose_split_k(int n_cu, int n_tiles, int k_steps);
pc_status launch_splitk_partial(percache_ctx *ctx, const __bf16 *a, int lda, const __bf16 *w0, const __bf16 *w1, int n_split,
                                int ldw, float *part, int M, int N, int K, int n_k, hipStream_t stream);
pc_status launch_v_repack(percache_ctx *ctx, const __bf16 *vf, __bf16 *vf_blk, int batch, int t_fresh, hipStream_t stream);
// formats: which slot formats the call's chunks sit in (see table_formats): bit 0 = 8-bit, bit 1 = bf16
pc_status launch_attention(percache_ctx *ctx, int layer, const __bf16 *q, const __bf16 *kf, const __bf16 *vf_blk,
                           int batch, int t_fresh, const int32_t *table_dev, int tbl_stride, int max_tiles,
                           int n_splits, __bf16 *out, __bf16 *part_o, float *part_ml, hipStream_t stream, int formats);
inline int table_formats(const std::vector<int32_t> &rows, int stride, int batch) {
  int f = 0;
  for (int b = 0; b < batch; ++b) f |= rows[(size_t)b * stride + 3];
  return f;
}

// Copies n_tokens tokens of a dense [Hkv][.][D] tensor whose heads are dense_head_stride elements apart into a
// slot (no validation, no slot-table update).
pc_status launch_kv_store(percache_ctx *ctx, int layer, int slot, const __bf16 *k, const __bf16 *v, int n_tokens,
                          long dense_head_stride, hipStream_t stream);

// Appends n_tokens tokens behind the `off` tokens a slot holds (no validation, no slot-table update).
pc_status launch_kv_append(percache_ctx *ctx, int layer, int slot, const __bf16 *k, const __bf16 *v, int off, int n_tokens,
                           long new_head_stride, hipStream_t stream);

}  // namespace pc
