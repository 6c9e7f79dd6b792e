"""Oracle of the cache bookkeeping around the hot path - TEST INFRASTRUCTURE, not product code.

Plain, slow and per token: a trie with ONE token per node, so that nothing here depends on how a radix tree happens
to cut its edges.  It states what Sec. 3.3 of the paper describes for the local scheduler - match a new request to the
prefix tree and update the tree; keep, per tree node, the number of active requests sharing it; when memory is short
evict by the access time of the requests (LRU), a whole node or the part of one that is enough - under the readings the
library documents: whole pages for the new part of a prompt, token t of it in slot page[t // p] * p + t % p; page 0
handed out first, freed pages reused last-freed-first; admission times strictly increase.

Eviction, per token: while fewer than `need` slots have become free, drop the token that (a) has no child, (b) lies on
no admitted request's path, (c) has the smallest access time among those.  (Admission times are distinct and one
admission touches one root-to-leaf path, so (c) never ties between two leaves.)

For the eviction term of the load cost (Sec. 3.2, second cost: the nodes that would be evicted to run a request, each
weighted by the share of the recent requests that used it) every token also keeps the times of the admissions that
ran through it, and `evict_plan` says which tokens an eviction would drop, without dropping them.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Tuple


class _Tok:
    __slots__ = ("token", "slot", "parent", "child", "ref", "last", "hits")

    def __init__(self, token: int, slot: int, parent: Optional["_Tok"]):
        self.token, self.slot, self.parent = token, slot, parent
        self.child: Dict[int, _Tok] = {}
        self.ref = 0
        self.last = 0
        self.hits: List[int] = []


class CacheOracle:
    def __init__(self, num_slots: int, page_size: int):
        assert page_size >= 1 and num_slots % page_size == 0
        self.p = page_size
        self.n_pages = num_slots // page_size
        self.free_pages: List[int] = list(range(self.n_pages - 1, -1, -1))  # the back is handed out next
        self.page_live = [0] * self.n_pages
        self.root = _Tok(-1, -1, None)
        self.clock: Optional[int] = None
        self.admissions: List[int] = []  # times of all admissions

    # -- queries -------------------------------------------------------------------------------------------------
    def free_slots(self) -> int:
        return len(self.free_pages) * self.p

    def match(self, tokens) -> Tuple[int, List[int]]:
        node, slots = self.root, []
        for t in tokens:
            nxt = node.child.get(int(t))
            if nxt is None:
                break
            node = nxt
            slots.append(node.slot)
        return len(slots), slots

    def tokens_cached(self) -> int:
        n, stack = 0, [self.root]
        while stack:
            x = stack.pop()
            n += len(x.child)
            stack.extend(x.child.values())
        return n

    # -- updates -------------------------------------------------------------------------------------------------
    def admit(self, tokens, now: int):
        """-> (n_cached, slots of the new tokens, handle) or None if the free pages do not suffice (nothing changes)."""
        assert len(tokens) >= 1 and (self.clock is None or now > self.clock)
        n_cached, _ = self.match(tokens)
        rem = len(tokens) - n_cached
        need = (rem + self.p - 1) // self.p
        if need > len(self.free_pages):
            return None
        node = self.root
        for t in tokens[:n_cached]:
            node = node.child[int(t)]
        new_slots, page = [], -1
        for i, t in enumerate(tokens[n_cached:]):
            if i % self.p == 0:
                page = self.free_pages.pop()
            slot = page * self.p + i % self.p
            self.page_live[page] += 1
            nxt = _Tok(int(t), slot, node)
            node.child[int(t)] = nxt
            node = nxt
            new_slots.append(slot)
        x = node
        while x is not self.root:
            x.ref += 1
            x.last = now
            x.hits.append(now)
            x = x.parent
        self.clock = now
        self.admissions.append(now)
        return n_cached, new_slots, node

    def release(self, handle: _Tok) -> None:
        x = handle
        while x is not self.root:
            assert x.ref > 0
            x.ref -= 1
            x = x.parent

    def need_for(self, tokens) -> int:
        """Slots that admitting this prompt still lacks: the whole pages of its part that is not cached, less the
        free pages."""
        rem = len(tokens) - self.match(tokens)[0]
        return max(0, ((rem + self.p - 1) // self.p) * self.p - self.free_slots())

    def _cached_part(self, tokens) -> set:
        node, keep = self.root, set()
        for t in tokens:
            node = node.child.get(int(t))
            if node is None:
                break
            keep.add(id(node))
        return keep

    def evict_for(self, tokens) -> Tuple[int, int]:
        """Make room for a prompt about to be admitted, never dropping a token of its cached part."""
        return self.evict(self.need_for(tokens), keep=self._cached_part(tokens))

    def evict_plan_for(self, tokens, since: int):
        return self.evict_plan(self.need_for(tokens), since, keep=self._cached_part(tokens))

    def evict_plan(self, need_slots: int, since: int, keep: Optional[set] = None):
        """What evict(need_slots) would drop: -> (per dropped token, in order: the number of admissions after time
        `since` that ran through it; per dropped token: whether it is the parent of the token dropped just before;
        the number of admissions after `since` in all).  Nothing changes."""
        pages_before, live_before = list(self.free_pages), list(self.page_live)
        victims: List[_Tok] = []
        self.evict(need_slots, victims, keep)
        for v in reversed(victims):
            v.parent.child[v.token] = v
        self.free_pages, self.page_live = pages_before, live_before
        sharers = [sum(1 for t in v.hits if t > since) for v in victims]
        linked = [k > 0 and victims[k - 1].parent is v for k, v in enumerate(victims)]
        return sharers, linked, sum(1 for t in self.admissions if t > since)

    def evict(self, need_slots: int, victims_out: Optional[List[_Tok]] = None, keep: Optional[set] = None) -> Tuple[int, int]:
        """-> (slots of the pages that became free, tokens dropped)."""
        freed = gone = 0
        while freed < need_slots:
            victim, stack = None, [self.root]
            while stack:  # every leaf token, from scratch each time: slow and plain
                x = stack.pop()
                if x.child:
                    stack.extend(x.child.values())
                elif x is not self.root and x.ref == 0 and (keep is None or id(x) not in keep) and \
                        (victim is None or x.last < victim.last):
                    victim = x
            if victim is None:
                break
            del victim.parent.child[victim.token]
            if victims_out is not None:
                victims_out.append(victim)
            gone += 1
            page = victim.slot // self.p
            self.page_live[page] -= 1
            if self.page_live[page] == 0:
                self.free_pages.append(page)
                freed += self.p
        return freed, gone
