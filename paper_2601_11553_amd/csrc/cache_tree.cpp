// Host-side index of the K/V cache: the prefix tree of knowledge chunks of Sec. 4.1.1 with the LFU eviction of
// the same section and the two boundary rules of App. B.2.  No device work: the tree hands out slot ids of the
// device-resident store; the caller fills them (cache slicer) and clears the ones the tree evicts.
//
//  - a node is one knowledge chunk (its text is the key: prefix matching is done on strings, App. B.2), a path
//    from the root is the chunk list one query retrieved; a node's tensors are only valid behind its own path
//    (they were computed at those positions, after those tokens);
//  - match: first chunk, then the second among the immediate children, ... until a mismatch (Sec. 4.2.2).
//    Several children may carry the same text (see insert), so the walk keeps the longest chain;
//  - insert: the new chain shares the common prefix with the tree only up to its second-to-last node; the last
//    node of the common prefix is stored again under the new path, because its final tokens were tokenized next
//    to a different successor (App. B.2, measure 1);
//  - a matched chain is used without the last few tokens of its final node (App. B.2, measure 2): match reports
//    used lengths accordingly;
//  - every node counts its retrievals; when the byte limit or the number of slots is exceeded, the leaf with the
//    lowest count goes first (ties: the one used longest ago).  Only leaves are evicted: an inner node's children
//    depend on it.
#include <algorithm>
#include <cstdint>
#include <cstring>
#include <map>
#include <memory>
#include <string>
#include <vector>

#include "percache.h"

struct percache_tree {
  struct Node {
    std::string text;
    Node *parent = nullptr;
    std::vector<std::unique_ptr<Node>> children;
    int32_t slot = -1;
    int32_t tokens = 0;
    int64_t count = 0;     // retrievals (LFU key)
    int64_t last_use = 0;  // logical clock of the last retrieval or insertion (tie break)
    bool pinned = false;   // part of the path being inserted: not evictable
  };
  Node root;
  int32_t n_slots = 0;
  int64_t byte_limit = 0, bytes_per_token = 0;
  int32_t tail_discard = 0;
  int64_t bytes_used = 0, clock = 0;
  std::vector<int32_t> free_slots;  // stack, lowest id on top
  int32_t n_nodes = 0;
};

namespace {
using Node = percache_tree::Node;

// longest chain of children matching keys[pos..n): returns its length and writes the nodes
int longest_chain(Node *at, const char *const *keys, int pos, int n, std::vector<Node *> &best) {
  best.clear();
  if (pos >= n) return 0;
  int best_len = 0;
  std::vector<Node *> sub;
  for (auto &ch : at->children) {
    if (ch->text != keys[pos]) continue;
    int len = 1 + longest_chain(ch.get(), keys, pos + 1, n, sub);
    // ties: the more often retrieved node, then the more recent one
    bool better = len > best_len || (len == best_len && !best.empty() &&
                                     (ch->count > best[0]->count || (ch->count == best[0]->count && ch->last_use > best[0]->last_use)));
    if (better) {
      best_len = len;
      best.assign(1, ch.get());
      best.insert(best.end(), sub.begin(), sub.end());
    }
  }
  return best_len;
}

void collect_leaves(Node *at, std::vector<Node *> &out) {
  for (auto &ch : at->children) {
    if (ch->children.empty()) out.push_back(ch.get());
    else collect_leaves(ch.get(), out);
  }
}

// evicts one leaf (lowest count, then oldest); returns its slot or -1 when nothing is evictable
int32_t evict_one(percache_tree *t) {
  std::vector<Node *> leaves;
  collect_leaves(&t->root, leaves);
  Node *victim = nullptr;
  for (Node *l : leaves) {
    if (l->pinned) continue;
    if (!victim || l->count < victim->count || (l->count == victim->count && l->last_use < victim->last_use)) victim = l;
  }
  if (!victim) return -1;
  const int32_t slot = victim->slot;
  t->bytes_used -= (int64_t)victim->tokens * t->bytes_per_token;
  t->free_slots.push_back(slot);
  std::sort(t->free_slots.begin(), t->free_slots.end(), [](int a, int b) { return a > b; });
  Node *p = victim->parent;
  auto &v = p->children;
  v.erase(std::find_if(v.begin(), v.end(), [&](const std::unique_ptr<Node> &u) { return u.get() == victim; }));
  --t->n_nodes;
  return slot;
}
}  // namespace

extern "C" {

percache_tree *percache_tree_create(int32_t n_slots, int64_t byte_limit, int64_t bytes_per_token, int32_t tail_discard_tokens) {
  if (n_slots < 1 || byte_limit < 1 || bytes_per_token < 1 || tail_discard_tokens < 0) return nullptr;
  percache_tree *t = new percache_tree;
  t->n_slots = n_slots;
  t->byte_limit = byte_limit;
  t->bytes_per_token = bytes_per_token;
  t->tail_discard = tail_discard_tokens;
  for (int32_t s = n_slots - 1; s >= 0; --s) t->free_slots.push_back(s);
  return t;
}

void percache_tree_destroy(percache_tree *t) { delete t; }

int32_t percache_tree_match(percache_tree *t, const char *const *chunk_texts, int32_t n, int32_t *slots_out,
                            int32_t *used_len_out) {
  if (!t || n < 0 || (n > 0 && (!chunk_texts || !slots_out || !used_len_out))) return PC_EINVAL;
  for (int i = 0; i < n; ++i)
    if (!chunk_texts[i]) return PC_EINVAL;
  std::vector<Node *> chain;
  const int len = longest_chain(&t->root, chunk_texts, 0, n, chain);
  ++t->clock;
  for (int i = 0; i < len; ++i) {
    Node *nd = chain[i];
    ++nd->count;
    nd->last_use = t->clock;
    slots_out[i] = nd->slot;
    used_len_out[i] = nd->tokens;
  }
  if (len > 0) used_len_out[len - 1] = std::max(0, chain[len - 1]->tokens - t->tail_discard);
  return len;
}

int32_t percache_tree_insert(percache_tree *t, const char *const *chunk_texts, const int32_t *chunk_tokens, int32_t n,
                             int32_t *slots_out, uint8_t *is_new_out, int32_t *evicted_out, int32_t evicted_cap,
                             int32_t *n_evicted_out) {
  if (!t || n < 1 || !chunk_texts || !chunk_tokens || !slots_out || !is_new_out || !n_evicted_out || evicted_cap < 0 ||
      !evicted_out || evicted_cap < t->n_slots)
    return PC_EINVAL;
  for (int i = 0; i < n; ++i)
    if (!chunk_texts[i] || chunk_tokens[i] < 1) return PC_EINVAL;
  *n_evicted_out = 0;
  std::vector<Node *> chain;
  int common = longest_chain(&t->root, chunk_texts, 0, n, chain);
  // the chain is shared only where the stored chunk has the same length, and the last node the two chains have in
  // common is not shared but stored again; a chain that is already there in full is shared in full (nothing new)
  for (int i = 0; i < common; ++i)
    if (chain[i]->tokens != chunk_tokens[i]) { common = i; break; }
  const int shared = common == n ? n : std::max(0, common - 1);
  int64_t need_bytes = 0;
  for (int i = shared; i < n; ++i) need_bytes += (int64_t)chunk_tokens[i] * t->bytes_per_token;
  if (need_bytes > t->byte_limit || n - shared > t->n_slots) return PC_ENOMEM;
  ++t->clock;
  Node *at = &t->root;
  for (int i = 0; i < shared; ++i) {
    at = chain[i];
    at->pinned = true;
    at->last_use = t->clock;
    slots_out[i] = at->slot;
    is_new_out[i] = 0;
  }
  // make room: bytes and slots
  const int n_new = n - shared;
  bool failed = false;
  while (!failed && (t->bytes_used + need_bytes > t->byte_limit || (int)t->free_slots.size() < n_new)) {
    int32_t s = evict_one(t);
    if (s < 0) { failed = true; break; }
    if (*n_evicted_out < evicted_cap) evicted_out[*n_evicted_out] = s;
    ++*n_evicted_out;
  }
  if (!failed) {
    for (int i = shared; i < n; ++i) {
      std::unique_ptr<Node> nd(new Node);
      nd->text = chunk_texts[i];
      nd->parent = at;
      nd->slot = t->free_slots.back();
      t->free_slots.pop_back();
      nd->tokens = chunk_tokens[i];
      nd->last_use = t->clock;
      nd->pinned = true;
      t->bytes_used += (int64_t)nd->tokens * t->bytes_per_token;
      ++t->n_nodes;
      slots_out[i] = nd->slot;
      is_new_out[i] = 1;
      Node *raw = nd.get();
      at->children.push_back(std::move(nd));
      at = raw;
    }
  }
  for (Node *p = at; p && p != &t->root; p = p->parent) p->pinned = false;
  for (int i = 0; i < shared; ++i) chain[i]->pinned = false;
  return failed ? PC_ENOMEM : shared;
}

int32_t percache_tree_nodes(const percache_tree *t) { return t ? t->n_nodes : PC_EINVAL; }
int64_t percache_tree_bytes(const percache_tree *t) { return t ? t->bytes_used : PC_EINVAL; }

}  // extern "C"
