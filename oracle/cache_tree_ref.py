"""Plain reference of the chunk prefix tree with LFU eviction (test infrastructure only; nothing here is used
by the product path).

Rules, from the paper:
  * Sec. 4.1.1: cached tensors are organised as a tree, one node per knowledge chunk, one path per retrieved chunk
    list; a retrieval counter per node, least-frequently-used eviction under a storage limit.
  * Sec. 4.2.2: matching goes chunk by chunk, the next chunk being looked for among the immediate children of the
    last matched node, until a mismatch.
  * App. B.2: matching is on the chunks' strings; when a new chain is merged, only the common prefix up to its
    second-to-last node is shared and the last common node is stored again; a matched chain loses the last few
    tokens of its final node.
Readings where the paper is silent (the same as the C library documents): only leaves are evicted (a node's
children were computed behind it), ties in the counter go to the least recently used, slot ids are handed out
lowest-first, among equal-length candidate chains the more retrieved (then more recent) first node wins, and a
stored chunk is only shared if its token count agrees.
"""
from __future__ import annotations


class _N:
    def __init__(self, text, parent, slot, tokens, now):
        self.text, self.parent, self.slot, self.tokens = text, parent, slot, tokens
        self.kids = []
        self.count = 0
        self.last = now


class TreeRef:
    def __init__(self, n_slots, byte_limit, bytes_per_token, tail_discard=0):
        self.root = _N(None, None, -1, 0, 0)
        self.free = list(range(n_slots))
        self.n_slots, self.limit, self.bpt, self.tail = n_slots, byte_limit, bytes_per_token, tail_discard
        self.now = 0
        self.bytes = 0

    # all maximal chains that follow `texts` from `node`
    def _chains(self, node, texts):
        if not texts:
            return [[]]
        out = [[]]
        for k in node.kids:
            if k.text == texts[0]:
                out += [[k] + rest for rest in self._chains(k, texts[1:])]
        return out

    def _best(self, texts):
        best = []
        for ch in self._chains(self.root, list(texts)):
            if not ch:
                continue
            if len(ch) > len(best):
                best = ch
            elif len(ch) == len(best) and ch[0] is not best[0]:
                # decided level by level from the top: more retrievals, then more recent
                for a, b in zip(ch, best):
                    if a is b:
                        continue
                    if (a.count, a.last) > (b.count, b.last):
                        best = ch
                    break
        return best

    def match(self, texts):
        ch = self._best(texts)
        self.now += 1
        for nd in ch:
            nd.count += 1
            nd.last = self.now
        slots = [nd.slot for nd in ch]
        used = [nd.tokens for nd in ch]
        if used:
            used[-1] = max(0, used[-1] - self.tail)
        return slots, used

    def _leaves(self, node, acc):
        for k in node.kids:
            if k.kids:
                self._leaves(k, acc)
            else:
                acc.append(k)
        return acc

    def insert(self, texts, tokens):
        n = len(texts)
        ch = self._best(texts)
        common = len(ch)
        for i, nd in enumerate(ch):
            if nd.tokens != tokens[i]:
                common = i
                break
        shared = n if common == n else max(0, common - 1)
        need = sum(tokens[shared:]) * self.bpt
        if need > self.limit or n - shared > self.n_slots:
            raise MemoryError
        self.now += 1
        keep = ch[:shared]
        for nd in keep:
            nd.last = self.now
        evicted = []
        while self.bytes + need > self.limit or len(self.free) < n - shared:
            cands = [l for l in self._leaves(self.root, []) if all(l is not k for k in keep)]
            if not cands:
                raise MemoryError(evicted)
            v = min(cands, key=lambda l: (l.count, l.last))
            v.parent.kids.remove(v)
            self.bytes -= v.tokens * self.bpt
            self.free.append(v.slot)
            evicted.append(v.slot)
        at = keep[-1] if keep else self.root
        slots = [nd.slot for nd in keep]
        new = [False] * shared
        for i in range(shared, n):
            s = min(self.free)
            self.free.remove(s)
            nd = _N(texts[i], at, s, tokens[i], self.now)
            at.kids.append(nd)
            at = nd
            self.bytes += tokens[i] * self.bpt
            slots.append(s)
            new.append(True)
        return shared, slots, new, evicted

    def n_nodes(self):
        def cnt(n):
            return sum(1 + cnt(k) for k in n.kids)
        return cnt(self.root)
