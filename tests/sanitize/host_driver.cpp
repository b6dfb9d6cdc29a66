// Sanitizer driver for the host side of the C ABI (built with -fsanitize=address,undefined, see
// tests/test_sanitizers.py): the cache index (Sec. 4.1.1, App. B.2: csrc/cache_tree.cpp, pointer-heavy host code) under
// random streams of insert / match with tight slot and byte limits, every output array sized exactly as the header
// says, plus the argument checks of the context calls that return before any device work.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <string>
#include <vector>

#include "percache.h"

static uint32_t state = 2463534242u;
static uint32_t rnd() { state ^= state << 13; state ^= state >> 17; state ^= state << 5; return state; }

static int tree_stream(int n_slots, int64_t byte_limit, int tail, int steps) {
  percache_tree *t = percache_tree_create(n_slots, byte_limit, 2, tail);
  if (!t) return 1;
  int bad = 0;
  std::vector<int32_t> slots(8), used(8), evicted(n_slots);
  std::vector<uint8_t> is_new(8);
  for (int s = 0; s < steps; ++s) {
    const int n = 1 + rnd() % 6;
    std::vector<std::string> texts(n);
    std::vector<const char *> ptrs(n);
    std::vector<int32_t> tok(n);
    for (int i = 0; i < n; ++i) {
      texts[i] = "chunk-" + std::to_string(rnd() % (i == 0 ? 3 : 9));   // few distinct first chunks: shared prefixes
      ptrs[i] = texts[i].c_str();
      tok[i] = 1 + rnd() % 40;
    }
    slots.assign(n, -7);
    used.assign(n, -7);
    is_new.assign(n, 9);
    const int m = percache_tree_match(t, ptrs.data(), n, slots.data(), used.data());
    if (m < 0 || m > n) ++bad;
    for (int i = 0; i < m; ++i)
      if (slots[i] < 0 || slots[i] >= n_slots || used[i] < 0) ++bad;
    if (rnd() % 3) {
      int32_t n_ev = -1;
      const int sh = percache_tree_insert(t, ptrs.data(), tok.data(), n, slots.data(), is_new.data(), evicted.data(), n_slots, &n_ev);
      if (n_ev < 0 || n_ev > n_slots) ++bad;
      if (sh >= 0) {
        if (sh > n) ++bad;
        for (int i = 0; i < n; ++i)
          if (slots[i] < 0 || slots[i] >= n_slots || is_new[i] != (i >= sh ? 1 : 0)) ++bad;
      } else if (sh != PC_ENOMEM) {
        ++bad;
      }
    }
    if (percache_tree_nodes(t) < 0 || percache_tree_nodes(t) > n_slots || percache_tree_bytes(t) < 0 || percache_tree_bytes(t) > byte_limit) ++bad;
  }
  percache_tree_destroy(t);
  return bad;
}

int main() {
  int bad = 0;
  bad += tree_stream(4, 1 << 20, 0, 400);      // slot-bound
  bad += tree_stream(16, 300, 0, 400);         // byte-bound
  bad += tree_stream(7, 200, 5, 400);          // both, with a tail discard
  bad += tree_stream(1, 1 << 20, 0, 100);      // a single slot
  // bad arguments
  if (percache_tree_create(0, 1, 1, 0) || percache_tree_create(1, 0, 1, 0) || percache_tree_create(1, 1, 1, -1)) ++bad;
  percache_tree_destroy(nullptr);
  const char *one[1] = {"x"};
  int32_t s1[1], u1[1];
  if (percache_tree_match(nullptr, one, 1, s1, u1) >= 0) ++bad;
#ifdef WITH_CONTEXT
  // context calls that must return before touching a device
  percache_config c = {1, 1024, 16, 8, 128, 16, 512, 4096, 10000.0f, 1000, 1024, 0, 0};
  if (percache_arena_bytes(&c) == 0 || percache_arena_bytes(nullptr) != 0) ++bad;
  percache_config bads[6] = {c, c, c, c, c, c};
  bads[0].head_dim = 96; bads[1].hidden = 1000; bads[2].n_kv_heads = 3; bads[3].slot_capacity = 100; bads[4].emb_dim = 96; bads[5].kv_fp8 = 2;
  for (const percache_config &b : bads)
    if (percache_arena_bytes(&b) != 0) ++bad;
  percache_ctx *ctx = nullptr;
  if (percache_create(&bads[0], nullptr, 0, &ctx) != PC_ESHAPE || ctx) ++bad;
  if (percache_create(&c, nullptr, 0, &ctx) != PC_EINVAL || percache_create(&c, (void *)0x1001, (size_t)1 << 40, &ctx) != PC_EINVAL) ++bad;
  if (percache_create(&c, (void *)0x1000, 16, &ctx) != PC_ENOMEM || ctx) ++bad;
  if (percache_create(&c, (void *)0x1000, 16, nullptr) != PC_EINVAL) ++bad;
  if (!percache_last_error(nullptr) || percache_bank_size(nullptr) != PC_EINVAL || percache_kv_len(nullptr, 0, 0) != PC_EINVAL) ++bad;
  if (percache_chunk_table_bytes(nullptr, 1, 1) != 0 || percache_prefill_workspace_bytes(nullptr, 1, 1, 1) != 0) ++bad;
  percache_destroy(nullptr);
#endif
  std::printf(bad ? "host driver: %d FAILED checks\n" : "host driver: ok\n", bad);
  return bad ? 1 : 0;
}
