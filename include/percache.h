/*
 * percache.h -- C ABI of the MI355X (gfx950) cache-reusing prefill and query-level match.
 *
 * The calls follow the online path of PerCache (arXiv 2601.11553, Sec. 3 "System Overview",
 * Sec. 4.2 "Cache Reuse", App. B.1): a query embedding is first matched against the QA bank
 * (percache_lookup); on a miss the K/V tensors of the retrieved chunks are taken from the
 * cache (a slot-indexed, per-layer, device-resident store filled by percache_kv_put) and only
 * the fresh suffix of the prompt is projected and attended (percache_prefill_reuse).
 *
 * Conventions
 *   - "dev" pointers are device (HBM) pointers owned by the caller; "host" pointers are
 *     ordinary host memory read before the call returns.  The library allocates no device
 *     memory: the caller hands over one arena at create time and a workspace per call.
 *   - Storage dtypes are fixed: hidden states, weights, Q/K/V and attention output are bf16;
 *     query embeddings are fp16; similarities and softmax state are fp32.
 *   - Every call validates its arguments (pointers, shapes, sizes, slot occupancy, lengths) on the host
 *     BEFORE enqueuing anything, so a call that returns any status but PC_EHIP has had no effect.
 *     PC_EHIP reports a failure of the HIP runtime itself (a launch or copy that was refused); work
 *     enqueued before it, and slot lengths already recorded for it, stay as they are.
 *   - Work is enqueued on the caller's stream (a hipStream_t passed as void*; NULL = the default
 *     stream) and is complete once the caller synchronises that stream.  Only percache_create
 *     synchronises the device.  Calls that take a chunk list as HOST arrays copy a small table to the
 *     device through a ring of 16 pinned staging buffers: the 17th such call in flight waits on the host
 *     for the oldest copy (hipEventSynchronize), a longer list than any before re-allocates the ring
 *     (hipHostMalloc), and such a call cannot be captured into a HIP graph with live contents.  The calls
 *     that take a device-resident chunk table (percache_chunk_table_put once, then *_table calls) do
 *     none of this: they enqueue kernels only, wait for nothing, allocate nothing, and can be captured.
 *   - One context serves one stream at a time; concurrent calls on one context are not safe, with one
 *     exception: percache_lookup / _topk / _refresh_scan touch only the bank and their own workspace and
 *     may run on a second stream beside a prefill or stack call (not beside percache_bank_put).
 *   - All functions return PC_OK (0) or a negative pc_status; percache_last_error gives text.
 */
#ifndef PERCACHE_H
#define PERCACHE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct percache_ctx percache_ctx;

typedef enum {
  PC_OK = 0,
  PC_EINVAL = -1, /* null pointer, negative count, bad alignment */
  PC_ESHAPE = -2, /* a dimension the kernels do not support, or out of configured range */
  PC_ESLOT = -3,  /* slot / layer index out of range, or slot empty */
  PC_ELEN = -4,   /* used length exceeds stored length, capacity or max_pos */
  PC_ENOMEM = -5, /* arena or workspace too small */
  PC_EHIP = -6    /* HIP runtime error; text in percache_last_error */
} pc_status;

/* Immutable shape of one context.  Supported: head_dim 64 or 128; hidden a multiple of 64;
 * n_q_heads a multiple of n_kv_heads; slot_capacity a multiple of 64; emb_dim a multiple of 64, at most 2048. */
typedef struct {
  int32_t n_layers;      /* layers of K/V store */
  int32_t hidden;        /* model width H */
  int32_t n_q_heads;     /* Hq */
  int32_t n_kv_heads;    /* Hkv */
  int32_t head_dim;      /* D */
  int32_t n_slots;       /* S: chunk slots per layer */
  int32_t slot_capacity; /* C: tokens per slot */
  int32_t max_pos;       /* RoPE table length; L_pre + T_f must not exceed it */
  float rope_theta;      /* RoPE base */
  int32_t bank_capacity; /* N_max: rows of the query-embedding bank (0 = no bank) */
  int32_t emb_dim;       /* d: embedding width */
  int32_t kv_fp8;        /* 0: slots hold bf16.  1: slots hold 8-bit codes, half the bytes (see "8-bit slots" below) */
  int32_t n_slots_8bit;  /* with kv_fp8 = 0: the LAST n_slots_8bit of the n_slots slots hold 8-bit codes, the others bf16
                            (a store of two organisations: which chunk goes where is the caller's choice by slot id);
                            must be 0 with kv_fp8 = 1 */
} percache_config;

/* Bytes of device memory the caller must provide for a context of this shape (0 on a bad
 * config).  Holds the RoPE table, the embedding bank with its inverse norms, and the K and V
 * stores of every layer. */
size_t percache_arena_bytes(const percache_config *cfg);

/* Builds a context over the caller's arena (256-byte aligned device memory of at least
 * percache_arena_bytes).  Computes the RoPE table on the host in double precision and copies it
 * in (this call synchronises).  All slots start empty and the bank starts with zero rows.
 * The arena must outlive the context; percache_destroy frees host state only. */
pc_status percache_create(const percache_config *cfg, void *arena_dev, size_t arena_bytes,
                          percache_ctx **out);
void percache_destroy(percache_ctx *ctx);
/* Text of the last error on this context (never NULL; "" if none).  With ctx == NULL: the last
 * error of percache_create on this thread. */
const char *percache_last_error(const percache_ctx *ctx);

/* ---------------------------------------------------------------- front tier (Sec. 4.2.1)
 * The QA bank's embedding matrix E[N, d] (fp16, row-major).  percache_bank_put writes rows
 * [index, index + n) from emb_dev ([n, d] fp16) and computes their inverse L2 norms; the bank
 * size becomes max(size, index + n).  index must not exceed the current size (no holes). */
pc_status percache_bank_put(percache_ctx *ctx, int32_t index, const void *emb_dev, int32_t n,
                            void *stream);
int32_t percache_bank_size(const percache_ctx *ctx);

/* Cosine top-1 of each probe against every bank row, and the hit flag of Sec. 4.2.1:
 *   sim[p] = max_j <probe_p, e_j> / (|probe_p| |e_j|),  idx[p] = the lowest j attaining it,
 *   hit[p] = sim[p] > tau   (strict: the similarity must EXCEED the threshold).
 * A zero-norm probe or row has similarity 0.  Empty bank: idx -1, sim -inf, hit 0.
 *   probes_dev [n_probes, d] fp16;  idx_out_dev int32[n_probes];  sim_out_dev float[n_probes];
 *   hit_out_dev uint8[n_probes];  workspace_dev >= percache_lookup_workspace_bytes. */
size_t percache_lookup_workspace_bytes(const percache_ctx *ctx, int32_t n_probes);
pc_status percache_lookup(percache_ctx *ctx, const void *probes_dev, int32_t n_probes, float tau,
                          int32_t *idx_out_dev, float *sim_out_dev, uint8_t *hit_out_dev,
                          void *workspace_dev, size_t workspace_bytes, void *stream);

/* percache_lookup for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same result as percache_lookup.  The per-workgroup
 * partial results go to a file-scope device array of the library (1 MiB, held by every GPU the library has created
 * a context on until the process ends) instead of a caller workspace; the call allocates and frees nothing.
 *   limits: n_probes <= 32 (one streaming pass of the bank) and a bank whose percache_lookup_workspace_bytes(ctx, 32)
 *           fits the array (bank_capacity up to about one million rows); beyond them PC_ESHAPE, nothing enqueued.
 *   sharing: every call on one GPU, from any context, uses that GPU's one array, and the array keeps the last call's
 *           contents (nothing in it needs clearing: a pass writes every entry it later reads).  Calls that can
 *           overlap on one GPU (different streams, different contexts) race on it; serialise them. */
pc_status percache_lookup_noalloc(percache_ctx *ctx, const void *probes_dev, int32_t n_probes, float tau,
                                  int32_t *idx_out_dev, float *sim_out_dev, uint8_t *hit_out_dev, void *stream);

/* The k best rows per probe instead of the best one (1 <= k <= 8): the ranking that cache refresh (Sec. 4.1.3,
 * "top-k_refresh") and dense retrieval over chunk embeddings need.  Same similarity, same tie rule (equal
 * similarities: lower row first), sorted best first.
 *   idx_out_dev int32[n_probes * k], sim_out_dev float[n_probes * k]; entries beyond the bank size: idx -1, sim -inf.
 * Same workspace as percache_lookup. */
pc_status percache_lookup_topk(percache_ctx *ctx, const void *probes_dev, int32_t n_probes, int32_t k,
                               int32_t *idx_out_dev, float *sim_out_dev, void *workspace_dev,
                               size_t workspace_bytes, void *stream);

/* Cache refresh scan (Sec. 4.1.3): new chunks have been added to the knowledge bank; a stored query's answer is
 * outdated if one of them ranks in that query's top-k_refresh.  With the bank holding the STORED QUERY embeddings
 * and kth_sim_dev[j] the similarity of query j's current k-th ranked chunk (percache_lookup_topk over the chunk
 * embeddings gives it), one pass over the bank per 32 new chunks computes for every bank row j
 *   best_sim[j] = max over new chunks c of cos(e_j, c),  best_new[j] = the lowest c attaining it,
 *   stale[j]    = best_sim[j] > kth_sim[j].
 *   new_emb_dev [n_new, d] fp16;  kth_sim_dev, best_sim_out_dev float[bank size];  best_new_out_dev int32[bank size];
 *   stale_out_dev uint8[bank size];  workspace as for percache_lookup (it also bounds n_new: 4 bytes per new row). */
pc_status percache_bank_refresh_scan(percache_ctx *ctx, const void *new_emb_dev, int32_t n_new,
                                     const float *kth_sim_dev, float *best_sim_out_dev, int32_t *best_new_out_dev,
                                     uint8_t *stale_out_dev, void *workspace_dev, size_t workspace_bytes,
                                     void *stream);

/* ---------------------------------------------------------------- 8-bit slots (kv_fp8 = 1, or the last n_slots_8bit slots)
 * The paper keeps the chunks' complete tensors (Sec. 4.1.1) and leaves other cache organisations to future work
 * (Sec. 7); this is a smaller slot for the same tensors.  An element is stored as an E4M3 code of the OCP 8-bit
 * floating point specification (1 sign, 4 exponent bits with bias 7, 3 mantissa bits, largest magnitude 448, no
 * infinities), with one power-of-two scale 2^e per (slot, kv head, block of 64 tokens), separately for K and V:
 * e is the smallest integer with max|x| <= 448 * 2^e over the block's stored tokens (0 for an all-zero block), kept in
 * [-110, 127]; code = E4M3(x * 2^-e), round to nearest, ties to even; the value read back is code * 2^e, exactly
 * representable in bf16.  percache_kv_put / _put_batch / _slice and the save slots of percache_stack_reuse quantise;
 * percache_kv_get returns the values read back; the attention calls read them on the fly (fresh K/V stay bf16).
 * percache_kv_append (and the decoding steps that use it): everything from the block that holds the first new token
 * on is quantised afresh from the values the slot reads back plus the new tokens; full blocks before it stay.
 * A store of both organisations (n_slots_8bit > 0 with kv_fp8 = 0; Sec. 7 looks ahead to chunks that are not all kept in the
 * same form): slot ids below n_slots - n_slots_8bit are bf16 slots, the others 8-bit
 * slots.  Every call treats each slot by its own format; one chunk list, one batched put or one list of save slots may
 * name slots of both kinds. */

/* ---------------------------------------------------------------- K/V store (Sec. 4.1.1)
 * One slot holds one knowledge chunk's K and V for one layer, as collected from the attention
 * module during a prefill (K already rotated at the positions it had then).
 *   k_dev, v_dev: [n_kv_heads, n_tokens, head_dim] bf16, 1 <= n_tokens <= slot_capacity.
 * percache_kv_put overwrites the slot and records n_tokens; percache_kv_get copies the stored
 * tokens back out in the same layout and reports the count (known on the host: no sync).
 * percache_kv_evict marks a slot empty (no device work). */
pc_status percache_kv_put(percache_ctx *ctx, int32_t layer, int32_t slot, const void *k_dev,
                          const void *v_dev, int32_t n_tokens, void *stream);
pc_status percache_kv_get(percache_ctx *ctx, int32_t layer, int32_t slot, void *k_out_dev,
                          void *v_out_dev, int32_t *n_tokens_out_host, void *stream);
pc_status percache_kv_evict(percache_ctx *ctx, int32_t layer, int32_t slot);
/* percache_kv_put for n chunks in one launch: tensors [n, n_kv_heads, n_tokens, head_dim] (the layout of
 * percache_prefill_reuse's k_fresh_out / v_fresh_out, so the fresh part of every query of a batch can be
 * saved at once); chunk i goes to slot slots_host[i].  Slots must be distinct. */
pc_status percache_kv_put_batch(percache_ctx *ctx, int32_t layer, const int32_t *slots_host, int32_t n,
                                const void *k_dev, const void *v_dev, int32_t n_tokens, void *stream);
/* percache_kv_get for n chunks in one launch: the first n_tokens tokens of slot slots_host[i] go to chunk i of the
 * output tensors [n, n_kv_heads, n_tokens, head_dim]; every slot named must hold at least n_tokens tokens (PC_ELEN
 * otherwise) and may appear more than once. */
pc_status percache_kv_get_batch(percache_ctx *ctx, int32_t layer, const int32_t *slots_host, int32_t n, void *k_out_dev,
                                void *v_out_dev, int32_t n_tokens, void *stream);
/* Appends n_tokens tokens ([n_kv_heads, n_tokens, head_dim] bf16 each) behind the tokens a slot already holds (an
 * empty slot is allowed): the decoding stage grows a sequence's own K/V token by token (Sec. 2.1). */
pc_status percache_kv_append(percache_ctx *ctx, int32_t layer, int32_t slot, const void *k_dev, const void *v_dev,
                             int32_t n_tokens, void *stream);
/* Cache slicer (Sec. 4.1.1, App. B.2): cuts the K/V of one prefilled sequence at chunk boundaries and stores
 * each piece in a slot of its own.  k_dev, v_dev: [n_kv_heads, seq_len, head_dim] bf16 (post-RoPE K); piece j is
 * the token range [bounds_host[j], bounds_host[j+1]) (n + 1 bounds; at most slot_capacity tokens per piece) and
 * goes to slot slots_host[j]; a negative slot id skips the piece.  Slots must be distinct. */
pc_status percache_kv_slice(percache_ctx *ctx, int32_t layer, const void *k_dev, const void *v_dev, int32_t seq_len,
                            const int32_t *bounds_host, const int32_t *slots_host, int32_t n, void *stream);
/* Stored token count of a slot, 0 if empty, negative pc_status on a bad index. */
int32_t percache_kv_len(const percache_ctx *ctx, int32_t layer, int32_t slot);

/* ---------------------------------------------------------------- cache-reusing prefill
 * (Sec. 4.2.2, App. B.1) for the attention module of one layer, `batch` independent queries.
 *
 * Chunk list, on the host: query b uses chunks slot_ids_host[b*max_chunks + c], c <
 * n_chunks_host[b], in prompt order, taking the first used_len_host[b*max_chunks + c] tokens of
 * each (used_len_host == NULL: the stored length; a shorter length drops the chunk's last tokens,
 * App. B.2).  L_pre[b] is the sum of the used lengths.  n_chunks_host[b] == 0 is an ordinary
 * causal prefill (full recomputation).
 *
 * Steps, all on device:
 *   1. [Q|K|V] = x_fresh Wqkv^T on the fresh rows only (Wqkv rows: Q heads, K heads, V heads);
 *   2. RoPE (pairs (m, m + D/2), angle pos * theta^(-2m/D)) on q and k of fresh token i at
 *      position L_pre[b] + i;
 *   3. fresh row i of head h attends over [cached chunk tokens ; fresh tokens t <= i] of kv
 *      head h / (Hq/Hkv): softmax(q.k / sqrt(D)) weighted sum of values.
 *
 *   x_fresh_dev      [batch, t_fresh, hidden] bf16
 *   wqkv_dev         [(Hq + 2 Hkv) * D, hidden] bf16
 *   attn_out_dev     [batch, t_fresh, Hq * D] bf16
 *   k_fresh_out_dev, v_fresh_out_dev  [batch, Hkv, t_fresh, D] bf16 (post-RoPE K), the layout
 *                    percache_kv_put takes per query; either may be NULL (kept in workspace).
 *   workspace_dev    >= percache_prefill_workspace_bytes(ctx, batch, t_fresh, max_chunks)
 */
size_t percache_prefill_workspace_bytes(const percache_ctx *ctx, int32_t batch, int32_t t_fresh,
                                        int32_t max_chunks);
pc_status percache_prefill_reuse(percache_ctx *ctx, int32_t layer, const void *x_fresh_dev,
                                 const void *wqkv_dev, int32_t batch, int32_t t_fresh,
                                 const int32_t *slot_ids_host, const int32_t *used_len_host,
                                 const int32_t *n_chunks_host, int32_t max_chunks,
                                 void *attn_out_dev, void *k_fresh_out_dev, void *v_fresh_out_dev,
                                 void *workspace_dev, size_t workspace_bytes, void *stream);

/* Device-resident chunk lists.  percache_chunk_table_put validates a chunk list exactly as percache_prefill_reuse
 * does (against layer `layer` of the slot table; used_len_host == NULL takes that layer's stored lengths), writes it
 * as a table into caller-owned device memory (table_dev, 16-byte aligned, at least percache_chunk_table_bytes) on the
 * stream, and keeps a host copy in the context.  The *_table calls then take the table in place of the three host
 * arrays: they check the host copy against the slot table as it is NOW (occupancy, lengths and slot formats of the
 * layers they touch, L_pre + t_fresh <= max_pos; PC_ELEN / PC_ESLOT if a slot has changed since the put), enqueue
 * kernels only, and are safe to capture into a HIP graph.  Writing another list of the same batch and max_chunks into
 * the same table_dev (ordered on the stream, outside the graph) changes what the next replay of a captured call reads;
 * the captured launch shapes stay those of the list at capture time, which is correct for any list and best for
 * lists of similar length.  percache_chunk_table_drop forgets the host copy (the memory stays the caller's).
 * Workspace of the *_table calls: as for the host-list calls with the table's max_chunks. */
size_t percache_chunk_table_bytes(const percache_ctx *ctx, int32_t batch, int32_t max_chunks);
pc_status percache_chunk_table_put(percache_ctx *ctx, void *table_dev, size_t table_bytes, int32_t layer, int32_t batch,
                                   const int32_t *slot_ids_host, const int32_t *used_len_host,
                                   const int32_t *n_chunks_host, int32_t max_chunks, void *stream);
pc_status percache_chunk_table_drop(percache_ctx *ctx, const void *table_dev);
pc_status percache_prefill_reuse_table(percache_ctx *ctx, int32_t layer, const void *x_fresh_dev, const void *wqkv_dev,
                                       int32_t batch, int32_t t_fresh, const void *table_dev, void *attn_out_dev,
                                       void *k_fresh_out_dev, void *v_fresh_out_dev, void *workspace_dev,
                                       size_t workspace_bytes, void *stream);

/* The two halves of percache_prefill_reuse as separate calls (same arguments and checks), so
 * that each can be measured and tested on its own.
 *   percache_qkv_rope: steps 1-2; q_out_dev [batch, Hq, t_fresh, D] bf16.
 *   percache_attention_reuse: step 3 from given q / fresh k / fresh v.  n_splits > 0 forces the
 *   number of partitions of the key axis that are processed by separate workgroups and merged
 *   afterwards (0 = chosen by the library); results do not depend on it beyond fp32 rounding. */
pc_status percache_qkv_rope(percache_ctx *ctx, const void *x_fresh_dev, const void *wqkv_dev,
                            int32_t batch, int32_t t_fresh, const int32_t *slot_ids_host,
                            const int32_t *used_len_host, const int32_t *n_chunks_host,
                            int32_t max_chunks, int32_t layer, void *q_out_dev, void *k_fresh_out_dev,
                            void *v_fresh_out_dev, void *workspace_dev, size_t workspace_bytes,
                            void *stream);
pc_status percache_attention_reuse(percache_ctx *ctx, int32_t layer, const void *q_dev,
                                   const void *k_fresh_dev, const void *v_fresh_dev, int32_t batch,
                                   int32_t t_fresh, const int32_t *slot_ids_host,
                                   const int32_t *used_len_host, const int32_t *n_chunks_host,
                                   int32_t max_chunks, int32_t n_splits, void *attn_out_dev,
                                   void *workspace_dev, size_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------- cache index (Sec. 4.1.1, Sec. 4.2.2, App. B.2)
 * Host-side prefix tree over knowledge chunks that hands out slot ids of the K/V store; no device work.  A node is
 * one chunk (keyed by its text), a path from the root the chunk list of one query.  The same slot id is meant to
 * be used in every layer of the store.
 *   create: n_slots slots; the stored chunks may take at most byte_limit bytes at bytes_per_token bytes per token
 *           (all layers together); a matched chain is used without the last tail_discard_tokens tokens of its final
 *           chunk (App. B.2).  NULL on a bad argument.
 *   match:  longest chain root -> chunk 0 -> chunk 1 ... present in the tree; returns its length m (0..n), writes
 *           slots_out[0..m) and used_len_out[0..m) (the stored token counts, the last one shortened by the tail
 *           discard) and counts one retrieval on each matched node.
 *   insert: stores the chain of n chunks (chunk_tokens[i] tokens each).  Returns the number s of leading chunks
 *           shared with the tree (their slots are in slots_out, is_new_out = 0: nothing to fill); chunks s..n-1 get
 *           fresh slots (is_new_out = 1) that the caller must fill, e.g. with percache_kv_slice.  Sharing stops one
 *           node before the end of the common prefix (App. B.2), unless the whole chain is already stored.  When
 *           the byte limit or the slot count requires it, least-frequently-retrieved leaves are evicted first
 *           (ties: least recently used); their slots are listed in evicted_out[0..*n_evicted_out) -- the caller
 *           clears them with percache_kv_evict in every layer -- and this list is final even when the call then
 *           fails with PC_ENOMEM (chain larger than the limits allow).  evicted_cap must be at least n_slots. */
typedef struct percache_tree percache_tree;
percache_tree *percache_tree_create(int32_t n_slots, int64_t byte_limit, int64_t bytes_per_token,
                                    int32_t tail_discard_tokens);
void percache_tree_destroy(percache_tree *tree);
int32_t percache_tree_match(percache_tree *tree, const char *const *chunk_texts, int32_t n, int32_t *slots_out,
                            int32_t *used_len_out);
int32_t percache_tree_insert(percache_tree *tree, const char *const *chunk_texts, const int32_t *chunk_tokens,
                             int32_t n, int32_t *slots_out, uint8_t *is_new_out, int32_t *evicted_out,
                             int32_t evicted_cap, int32_t *n_evicted_out);
int32_t percache_tree_nodes(const percache_tree *tree);
int64_t percache_tree_bytes(const percache_tree *tree);

/* ---------------------------------------------------------------- a stack of layers on the retained rows
 * (App. B.1).  After the attention module a block goes on as usual, and the next layer crops the cached rows
 * again, so only the retained (fresh) rows of every layer are ever computed:
 *   n  = RMSNorm(h; gain1, eps)                    y = x / sqrt(mean(x^2) + eps) * gain
 *   a  = cache-reusing attention of layer l on n   (percache_prefill_reuse with that layer's wqkv and store)
 *   h' = h + a wo^T
 *   h''= h' + (silu(m w_gate^T) * (m w_up^T)) w_down^T,   m = RMSNorm(h'; gain2, eps)
 * All weights bf16 device pointers, 16-byte aligned; the struct array itself is host memory. */
typedef struct {
  const void *gain1;  /* [hidden] */
  const void *wqkv;   /* [(Hq + 2 Hkv) * D, hidden] */
  const void *wo;     /* [hidden, Hq * D] */
  const void *gain2;  /* [hidden] */
  const void *w_gate; /* [ffn, hidden] */
  const void *w_up;   /* [ffn, hidden] */
  const void *w_down; /* [hidden, ffn] */
  /* model-family variants of the projection (the paper runs Llama and Qwen models, Sec. 5.1); NULL = absent */
  const void *qkv_bias; /* [(Hq + 2 Hkv) * D]: added to the projection before anything else (Qwen2 style) */
  const void *q_norm;   /* [D]: gain of an RMSNorm (same eps) over the head dimension of every q head, before RoPE */
  const void *k_norm;   /* [D]: the same for every k head (Qwen3 style) */
} percache_block_weights;

/* Runs layers 0 .. n_layers-1 (layer l reads store layer l; the chunk list is the same for every layer and the
 * chunks' stored lengths must agree across layers).  hidden must be a multiple of 128, ffn of 64.
 *   h_in_dev, h_out_dev  [batch, t_fresh, hidden] bf16 (may be the same buffer)
 *   save_*: optional cache slicer on the way (n_save == 0: off).  The fresh K/V of every layer are cut at
 *           save_bounds_host[0 .. n_save] (token indices inside the fresh part, the same for every query) and piece
 *           j of query b is stored in slot save_slots_host[b * n_save + j] of that layer (negative: skipped).
 *           Save slots must be distinct and must not be read by this call.  With n_chunks == 0 this is the
 *           population pass: an ordinary prefill that fills the cache.
 *   workspace_dev        >= percache_stack_workspace_bytes(ctx, batch, t_fresh, max_chunks, ffn), 256-byte aligned */
size_t percache_stack_workspace_bytes(const percache_ctx *ctx, int32_t batch, int32_t t_fresh, int32_t max_chunks,
                                      int32_t ffn);
pc_status percache_stack_reuse(percache_ctx *ctx, const percache_block_weights *layers_host, int32_t n_layers,
                               int32_t ffn, float eps, const void *h_in_dev, int32_t batch, int32_t t_fresh,
                               const int32_t *slot_ids_host, const int32_t *used_len_host,
                               const int32_t *n_chunks_host, int32_t max_chunks, const int32_t *save_bounds_host,
                               const int32_t *save_slots_host, int32_t n_save, void *h_out_dev, void *workspace_dev,
                               size_t workspace_bytes, void *stream);

/* percache_stack_reuse with the chunk list in a device-resident table (see percache_chunk_table_put; no save slots):
 * kernels only, so the whole stack can be captured into a HIP graph and replayed (App. B.1: the same per-block
 * sequence runs for every layer and every query with the same shapes). */
pc_status percache_stack_reuse_table(percache_ctx *ctx, const percache_block_weights *layers_host, int32_t n_layers,
                                     int32_t ffn, float eps, const void *h_in_dev, int32_t batch, int32_t t_fresh,
                                     const void *table_dev, void *h_out_dev, void *workspace_dev, size_t workspace_bytes,
                                     void *stream);

/* Decoding step (Sec. 2.1: after prefill the model emits one token at a time, each attending to everything before
 * it): percache_stack_reuse for n_new >= 1 new tokens per query (h_in_dev [batch, n_new, hidden]) whose chunk
 * list names everything already stored -- the reused knowledge chunks, then the slots that hold the prompt's own
 * K/V and the tokens generated so far -- and whose new K/V are APPENDED, layer by layer, to slot
 * append_slots_host[b] (negative: not stored).  That slot may be (and usually is) the last one of the query's own
 * chunk list: it is read with its old length and grows afterwards.  Same workspace as percache_stack_reuse. */
pc_status percache_stack_decode(percache_ctx *ctx, const percache_block_weights *layers_host, int32_t n_layers,
                                int32_t ffn, float eps, const void *h_in_dev, int32_t batch, int32_t n_new,
                                const int32_t *slot_ids_host, const int32_t *used_len_host,
                                const int32_t *n_chunks_host, int32_t max_chunks, const int32_t *append_slots_host,
                                void *h_out_dev, void *workspace_dev, size_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------- kernel timing
 * With profiling on, the launches of the three main kernels are bracketed by HIP events on the caller's
 * stream (the paper reports per-stage latency breakdowns, Sec. 5.3 and Table "System Overhead"; this is
 * the device-side counterpart).  percache_profile_read waits for the recorded events, returns the summed
 * duration in milliseconds and the number of launches since the last read or enable, and clears the record
 * (at most 256 launches per kernel are kept).  kernel: 0 lookup stream pass, 1 QKV projection + RoPE,
 * 2 reuse attention (main kernel, without the split merge).
 * on: 0 switches the events off, 1 brackets all three kinds, any other value is a mask in which bit (kernel + 1)
 * selects a kind (4 = the projection only, 8 = attention only, ...): an event pair costs a few microseconds on the
 * stream, so a caller that times a whole step asks only for the kernel it needs. */
typedef enum { PC_KERNEL_LOOKUP = 0, PC_KERNEL_QKV_ROPE = 1, PC_KERNEL_ATTENTION = 2 } pc_kernel;
pc_status percache_profile_enable(percache_ctx *ctx, int32_t on);
pc_status percache_profile_read(percache_ctx *ctx, int32_t kernel, float *sum_ms_host, int32_t *count_host);

/* ---------------------------------------------------------------- achievable peaks (measurement aids)
 * The paper reports where its time goes (Sec. 5.3 breakdowns); here every kernel of the path is priced against a
 * roofline, and these calls measure what the device sustains on each resource with a kernel that does nothing
 * else, so that a fraction can be quoted against the published peak and against the achievable one.  The caller times
 * them with events on the stream.
 *   percache_peak_mfma_bf16: every compute unit runs `iters` x 64 register-resident 32x32x16 bf16 matrix instructions
 *     per wavefront (two wavefronts per SIMD), on constant operands (random_operands = 0) or on random ones (the
 *     sustained clock depends on the data's bit activity); *flops_out_host receives the flop count of the launch.
 *   percache_peak_stream_read: reads `bytes` bytes of buf_dev once, every workgroup one contiguous range.
 *   percache_peak_attention_tile_loop: a model of the reuse-attention kernel's inner loop (Sec. 4.2.2: the attention
 *     over [loaded ; fresh] keys) with the bookkeeping taken away -- per 64-key tile and wavefront the same operand
 *     reads, matrix instructions, exponentials, global->LDS requests (three LDS stages), wait and barrier, but no chunk list, mask or
 *     running maximum, all tiles from the first 8 MiB of kv_dev (bf16 values, e.g. N(0,1)), which stay in L2.  `tiles`
 *     tiles per workgroup, one workgroup of eight wavefronts per compute unit.  What it sustains is what this loop
 *     structure allows on the device; the kernel of the path is reported against it.
 *   scratch_dev: at least percache_peak_scratch_bytes(ctx) bytes, written by all three (contents meaningless). */
size_t percache_peak_scratch_bytes(const percache_ctx *ctx);
pc_status percache_peak_mfma_bf16(percache_ctx *ctx, int32_t iters, int32_t random_operands, void *scratch_dev,
                                  size_t scratch_bytes, double *flops_out_host, void *stream);
pc_status percache_peak_stream_read(percache_ctx *ctx, const void *buf_dev, size_t bytes, void *scratch_dev,
                                    size_t scratch_bytes, void *stream);
pc_status percache_peak_attention_tile_loop(percache_ctx *ctx, const void *kv_dev, size_t kv_bytes, int32_t tiles,
                                            void *scratch_dev, size_t scratch_bytes, double *flops_out_host, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* PERCACHE_H */
