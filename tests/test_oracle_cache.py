"""Pins for the oracle of the cache bookkeeping (CPU only), and the library's host code against it.

The per-token oracle is checked against things that are not itself: a hand-worked example
(tests/golden/cache_hand_example.txt), and properties that Sec. 3.3 and the documented readings fix for ANY
sequence of operations, each evaluated from the raw history or from the state before and after a call:
no slot is handed out twice while its token is cached; pages are whole; eviction never touches a token that an
admitted request runs through, takes the least recently used of the evictable leaves first, and stops as soon as
enough pages are free.  Then the library's radix-tree implementation (pa_tree_attach_pool / admit / release /
evict) has to agree with the oracle call by call on random operation sequences.
"""
import os

import numpy as np
import pytest

from oracle.cache_oracle import CacheOracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "cache_hand_example.txt")


@pytest.fixture(scope="module")
def pa():
    from paper_2407_00023_amd import binding
    return binding


class LibSide:
    """The library behind the same small interface as the oracle."""

    def __init__(self, pa, num_slots, page_size):
        self.pa, self.t = pa, pa.Tree()
        self.t.attach_pool(num_slots, page_size)

    def admit(self, tokens, now):
        try:
            c, s, h = self.t.admit(np.asarray(tokens, np.int32), now)
        except self.pa.PrefixAttnError as e:
            assert e.code == -2, e
            return None
        return c, s.tolist(), h

    def release(self, h):
        self.t.release(h)

    def evict(self, need):
        return self.t.evict(need)

    def free_slots(self):
        return self.t.free_slots()

    def tokens_cached(self):
        return self.t.stats()[1]


def run_golden(make):
    side, handles = None, {}
    for raw in open(GOLDEN):
        line = raw.split("#")[0].strip()
        if not line:
            continue
        op, _, rest = line.partition(" ")
        f = [x.strip() for x in rest.split("|")]
        if op == "pool":
            ns, ps = map(int, f[0].split())
            side = make(ns, ps)
        elif op == "admit":
            name, now, *toks = f[0].split()
            got = side.admit([int(x) for x in toks], int(now))
            assert got is not None, line
            assert got[0] == int(f[1]) and list(got[1]) == [int(x) for x in f[2].split()], (line, got)
            handles[name] = got[2]
        elif op == "release":
            side.release(handles.pop(f[0]))
        elif op == "evict":
            assert tuple(side.evict(int(f[0]))) == (int(f[1]), int(f[2])), line
        elif op == "free":
            assert side.free_slots() == int(f[0]), line
        elif op == "query":
            if hasattr(side, "root"):  # only the oracle answers queries on the host
                n, slots = side.match([int(x) for x in f[0].split()])
                assert n == int(f[1]) and slots == [int(x) for x in f[2].split()], (line, n, slots)
        else:
            raise AssertionError(line)


def test_oracle_hand_worked_example():
    run_golden(CacheOracle)


def test_library_hand_worked_example(pa):
    run_golden(lambda ns, ps: LibSide(pa, ns, ps))


def random_ops(rng, n_ops, vocab, ns):
    """(op, payload) stream; prompts reuse earlier prompts' prefixes so that the tree branches and shares."""
    seqs, now = [], 0
    for _ in range(n_ops):
        x = rng.random()
        if x < 0.55:
            if seqs and rng.random() < 0.6:
                base = seqs[int(rng.integers(len(seqs)))]
                toks = list(base[:int(rng.integers(0, len(base) + 1))]) + [int(t) for t in rng.integers(0, vocab, int(rng.integers(0, 12)))]
            else:
                toks = [int(t) for t in rng.integers(0, vocab, int(rng.integers(1, 14)))]
            toks = toks or [1]
            now += int(rng.integers(1, 5))
            seqs.append(toks)
            yield "admit", (toks, now)
        elif x < 0.8:
            yield "release", rng.random()
        else:
            yield "evict", int(rng.integers(1, ns // 2 + 2))


def snapshot(o):
    """token path -> (slot, ref, last) of every cached token."""
    out, stack = {}, [((), o.root)]
    while stack:
        path, x = stack.pop()
        for t, c in x.child.items():
            out[path + (t,)] = (c.slot, c.ref, c.last)
            stack.append((path + (t,), c))
    return out


@pytest.mark.parametrize("seed", range(12))
def test_oracle_properties_on_random_histories(seed):
    rng = np.random.default_rng(seed)
    ps = int(rng.choice([1, 2, 4, 16]))
    ns = ps * int(rng.integers(4, 40))
    o = CacheOracle(ns, ps)
    live = []       # (handle, prompt) of admitted, unreleased requests
    touched = {}    # token path -> time of the last admission through it, from the raw history
    for op, arg in random_ops(rng, 150, 4, ns):
        before = snapshot(o)
        if op == "admit":
            toks, now = arg
            got = o.admit(toks, now)
            cached_before = 0
            while cached_before < len(toks) and tuple(toks[:cached_before + 1]) in before:
                cached_before += 1
            if got is None:
                need_pages = (len(toks) - cached_before + ps - 1) // ps
                assert need_pages * ps > o.free_slots() and snapshot(o) == before
                continue
            n_cached, new_slots, h = got
            assert n_cached == cached_before and len(new_slots) == len(toks) - n_cached
            # whole pages, consecutive inside a page, never a slot that some cached token already has
            in_use = {v[0] for v in before.values()}
            assert not (set(new_slots) & in_use) and len(set(new_slots)) == len(new_slots)
            for i, s in enumerate(new_slots):
                assert s % ps == i % ps and (i % ps == 0 or s == new_slots[i - 1] + 1)
            live.append((h, tuple(toks)))
            for j in range(1, len(toks) + 1):
                touched[tuple(toks[:j])] = now
        elif op == "release":
            if live:
                h, _ = live.pop(int(arg * len(live)))
                o.release(h)
        else:
            free0 = o.free_slots()
            freed, gone = o.evict(arg)
            after = snapshot(o)
            dropped = set(before) - set(after)
            assert len(dropped) == gone and set(after) <= set(before) and o.free_slots() == free0 + freed
            pinned = {p[:j] for _, p in live for j in range(1, len(p) + 1)}
            assert not (dropped & pinned)
            # what is left is still a tree, and the tokens that went were leaves when they went: no survivor below them
            assert all(path[:-1] in after for path in after if len(path) > 1)
            # LRU: every token that could still go is at least as recent as everything that went
            could_go = [p for p in after if p not in pinned and not any(q[:len(p)] == p and len(q) > len(p) for q in after)]
            if dropped and could_go:
                assert max(touched[p] for p in dropped) <= min(touched[p] for p in could_go)
            # only as far as needed: either the request is met and the last page freed was needed, or nothing could go
            if freed >= arg:
                assert freed - ps < arg or ps > arg
            else:
                assert not could_go
        # bookkeeping that holds at every step
        snap = snapshot(o)
        assert all(v[2] == touched[p] for p, v in snap.items())
        assert all(v[1] == sum(1 for _, q in live if q[:len(p)] == p) for p, v in snap.items())
        used_pages = {v[0] // ps for v in snap.values()}
        assert o.free_slots() == ns - ps * len(used_pages)


@pytest.mark.parametrize("seed", range(40))
def test_library_agrees_with_oracle_call_by_call(pa, seed):
    rng = np.random.default_rng(1000 + seed)
    ps = int(rng.choice([1, 2, 4, 16]))
    ns = ps * int(rng.integers(4, 40))
    o, lib = CacheOracle(ns, ps), LibSide(pa, ns, ps)
    live = []
    for op, arg in random_ops(rng, 120, int(rng.choice([2, 4, 50])), ns):
        if op == "admit":
            ro, rl = o.admit(*arg), lib.admit(*arg)
            assert (ro is None) == (rl is None)
            if ro is not None:
                assert ro[0] == rl[0] and ro[1] == rl[1]
                live.append((ro[2], rl[2]))
        elif op == "release":
            if live:
                ho, hl = live.pop(int(arg * len(live)))
                o.release(ho)
                lib.release(hl)
        else:
            assert tuple(o.evict(arg)) == tuple(lib.evict(arg))
        assert o.free_slots() == lib.free_slots() and o.tokens_cached() == lib.tokens_cached()


def test_library_error_paths(pa):
    t = pa.Tree()
    with pytest.raises(pa.PrefixAttnError):
        t.admit([1, 2], 1)                      # no pool attached
    t.attach_pool(8, 2)
    with pytest.raises(pa.PrefixAttnError):
        t.insert(np.array([1], np.int32), np.array([0], np.int32))   # slots come from admit now
    with pytest.raises(pa.PrefixAttnError):
        t.attach_pool(8, 2)                     # only once
    c, s, h = t.admit([1, 2, 3], 5)
    with pytest.raises(pa.PrefixAttnError):
        t.admit([1, 2, 3], 5)                   # time must increase
    with pytest.raises(pa.PrefixAttnError):
        t.admit(list(range(100, 120)), 6)       # 10 pages wanted, 2 free
    assert t.free_slots() == 4 and t.stats()[1] == 3
    with pytest.raises(pa.PrefixAttnError):
        t.release(12345)
    t.release(h)
    with pytest.raises(pa.PrefixAttnError):
        t.release(h)                            # not admitted any more
    assert t.evict(100) == (4, 3) and t.free_slots() == 8
