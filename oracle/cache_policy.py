"""Reference model of the expert cache (integer bookkeeping only).  TEST INFRASTRUCTURE ONLY.

The paper evaluates expert caching on top of Pre-gated MoE with three replacement policies
(Sec. VI, caching discussion: last-in-first-out, least-frequently-used, least-recently-used) and
gives no further detail, so the rules are fixed here and in include/pgmoe.h:

  * one cache of C slots per MoE block; a fetch presents the ascending list of distinct experts;
  * an expert found in a slot is a hit (its last-use time is set to this fetch, its use count
    goes up by one) and that slot cannot be evicted by this fetch;
  * every missing expert, in ascending order, takes a slot not used by this fetch: an empty one
    first (lowest index), else the victim of the policy - LRU: oldest last use; LFU: smallest use
    count, then oldest last use; LIFO: most recently inserted; remaining ties to the lowest slot;
  * a missing expert for which no such slot is left is not cached (it goes to the ordinary
    per-block slots);
  * every missing expert is copied; hits are not.
"""
from __future__ import annotations

LRU, LFU, LIFO = 0, 1, 2


class ExpertCache:
    def __init__(self, slots: int, policy: int):
        self.C, self.policy = slots, policy
        self.exp = [-1] * slots
        self.use = [-1] * slots
        self.cnt = [-1] * slots
        self.ins = [-1] * slots
        self.tick = -1
        self.seq = -1

    def _key(self, c):
        if self.exp[c] < 0:
            return (0, 0, 0)
        if self.policy == LRU:
            return (1, self.use[c], 0)
        if self.policy == LFU:
            return (1, self.cnt[c], self.use[c])
        return (1, -self.ins[c], 0)

    def fetch(self, selected):
        """selected: iterable of distinct expert ids.  -> dict(hits, copies=[(expert, 'cache'|'gen', slot)])."""
        sel = sorted(set(int(e) for e in selected))
        self.tick += 1
        pinned = set()
        hits = 0
        for c in range(self.C):
            if self.exp[c] >= 0 and self.exp[c] in sel:
                hits += 1
                self.use[c] = self.tick
                self.cnt[c] += 1
                pinned.add(c)
        cached_now = {self.exp[c] for c in pinned}
        copies, gen = [], 0
        for e in sel:
            if e in cached_now:
                continue
            cand = [c for c in range(self.C) if c not in pinned]
            if cand:
                v = min(cand, key=lambda c: (self._key(c), c))
                self.seq += 1
                self.exp[v], self.use[v], self.cnt[v], self.ins[v] = e, self.tick, 1, self.seq
                pinned.add(v)
                copies.append((e, "cache", v))
            else:
                copies.append((e, "gen", gen))
                gen += 1
        return dict(hits=hits, copies=copies, unique=len(sel))
