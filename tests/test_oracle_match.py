"""Pins for the oracle's trie matcher (CPU only).

The trie is checked against things that are not the trie: the definition "longest
common prefix with any cached sequence" evaluated by brute force over the raw list
(Sec. 3.2: match from the beginning until no match exists; Algorithm 1: cached_len =
sum of matched length), a hand-worked example, and the prefix lengths the workload
generators construct on purpose.
"""
import os

import numpy as np
import pytest

import oracle
from paper_2407_00023_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "radix_hand_example.txt")


def lcp(a, b):
    n = min(len(a), len(b))
    k = 0
    while k < n and a[k] == b[k]:
        k += 1
    return k


def brute_force(cached, prompt):
    """(matched length, slots): longest common prefix with any cached sequence; the slot of
    position j is the one carried by the FIRST inserted sequence sharing the first j+1 tokens."""
    lens = [lcp(prompt, tok) for tok, _ in cached]
    best = max(lens) if lens else 0
    slots = []
    for j in range(best):
        first = next(i for i, L in enumerate(lens) if L > j)
        slots.append(int(cached[first][1][j]))
    return best, slots


def run_oracle(cached, prompts):
    toks = np.concatenate([np.asarray(p, np.int32) for p in prompts]) if prompts else np.zeros(0, np.int32)
    off = np.zeros(len(prompts) + 1, np.int32)
    off[1:] = np.cumsum([len(p) for p in prompts])
    pl, si = oracle.match_prefixes(cached, toks, off)
    return pl, si, off


def test_hand_worked_example():
    cached, queries = [], []
    for line in open(GOLDEN):
        line = line.strip()
        if line.startswith("insert"):
            pairs = [x.split(":") for x in line.split()[1:]]
            cached.append((np.array([int(a) for a, _ in pairs], np.int32), np.array([int(b) for _, b in pairs], np.int32)))
        elif line.startswith("query"):
            a, b, c = line[len("query"):].split("|")
            queries.append(([int(x) for x in a.split()], int(b), [int(x) for x in c.split()]))
    assert len(cached) == 4 and len(queries) == 8
    pl, si, off = run_oracle(cached, [q[0] for q in queries])
    for r, (prompt, want_len, want_slots) in enumerate(queries):
        assert pl[r] == want_len, (prompt, pl[r])
        assert list(si[off[r]:off[r] + pl[r]]) == want_slots
        assert all(si[off[r] + pl[r]:off[r + 1]] == -1)


@pytest.mark.parametrize("vocab,seed", [(2, 0), (3, 1), (4, 2), (3, 3), (2, 4)])
def test_brute_force_tiny_vocab(vocab, seed):
    rng = np.random.default_rng(seed)
    for _ in range(60):
        nseq = int(rng.integers(0, 9))
        cached, next_slot = [], 0
        for _ in range(nseq):
            n = int(rng.integers(1, 13))
            cached.append((rng.integers(0, vocab, n).astype(np.int32),
                           np.arange(next_slot, next_slot + n, dtype=np.int32)))
            next_slot += n
        prompts = [rng.integers(0, vocab, int(rng.integers(0, 15))).astype(np.int32) for _ in range(12)]
        # also: prompts that are exact cached sequences, proper prefixes, and extensions of them
        for tok, _ in cached[:3]:
            prompts += [tok.copy(), tok[:len(tok) // 2].copy(), np.concatenate([tok, tok[:2]])]
        pl, si, off = run_oracle(cached, prompts)
        for r, p in enumerate(prompts):
            L, slots = brute_force(cached, p)
            assert pl[r] == L
            assert list(si[off[r]:off[r] + L]) == slots


def test_exhaustive_all_prompts_small():
    """Every prompt of length <= 6 over a 2-symbol vocabulary against a fixed cache."""
    rng = np.random.default_rng(7)
    cached = [(rng.integers(0, 2, n).astype(np.int32), (100 * k + np.arange(n)).astype(np.int32))
              for k, n in enumerate([5, 7, 3, 6, 1])]
    prompts = [[(x >> b) & 1 for b in range(n)] for n in range(0, 7) for x in range(1 << n)]
    pl, si, off = run_oracle(cached, prompts)
    for r, p in enumerate(prompts):
        L, slots = brute_force(cached, p)
        assert pl[r] == L and list(si[off[r]:off[r] + L]) == slots


def test_insert_reports_already_cached_prefix():
    tr = oracle.Trie()
    a = np.array([4, 5, 6, 7], np.int32)
    assert tr.insert(a, np.arange(4)) == 0
    assert tr.insert(a, np.arange(10, 14)) == 4          # fully present: nothing new
    assert tr.insert(np.array([4, 5, 9], np.int32), np.arange(20, 23)) == 2
    assert tr.num_nodes == 1 + 4 + 1
    pl, si = tr.match(np.array([4, 5, 9, 1], np.int32), np.array([0, 4], np.int32))
    assert pl[0] == 3 and list(si[:3]) == [0, 1, 22]


def test_empty_tree_and_empty_prompts():
    pl, si, off = run_oracle([], [[1, 2, 3], []])
    assert list(pl) == [0, 0] and all(si == -1)


@pytest.mark.parametrize("name", ["tiny_fp32", "tool_use", "long_doc_qa", "agent_tree", "video_qa", "programming", "tool_use_zipf", "decode"])
def test_designed_prefix_small_variants(name):
    """Generators build prompts whose cached prefix is known by construction; the trie must
    find exactly that, and brute force over the raw cached list must agree."""
    wl = W.small_variant(name, seed=3)
    cached = [wl.cached_seq(i) for i in range(wl.n_cached)]
    pl, si = oracle.match_prefixes(cached, wl.tokens, wl.offsets)
    assert np.array_equal(pl, wl.designed_prefix_len)
    for r in range(wl.B):
        lo, P = int(wl.offsets[r]), int(pl[r])
        assert np.array_equal(si[lo:lo + P], wl.designed_slots[lo:lo + P])
        L, slots = brute_force(cached, wl.prompt(r))
        assert L == P and slots == list(si[lo:lo + P])
        assert len(set(slots)) == len(slots)            # slots of one request are pairwise distinct
    assert int((wl.ext_len == (wl.offsets[1:] - wl.offsets[:-1]) - pl).all())


@pytest.mark.parametrize("name", ["tool_use", "long_doc_qa", "agent_tree", "video_qa", "programming", "tool_use_zipf", "decode"])
def test_designed_prefix_full_configs(name):
    wl = W.CONFIGS[name]()
    tr = oracle.Trie()
    for i in range(wl.n_cached):
        tr.insert(*wl.cached_seq(i))
    pl, si = tr.match(wl.tokens, wl.offsets)
    assert np.array_equal(pl, wl.designed_prefix_len)
    valid = wl.designed_slots >= 0
    assert np.array_equal(si[valid], wl.designed_slots[valid])
    assert (si[~valid] == -1).all()
    # every slot a request reaches is a real (backed) pool slot
    assert si[valid].max() < wl.num_slots
    assert np.isin(si[valid], wl.pool_slots).all()
    # sampled brute force on the raw list (vectorised compare against every cached sequence)
    rng = np.random.default_rng(0)
    for r in rng.choice(wl.B, size=min(3, wl.B), replace=False):
        p = wl.prompt(int(r))
        best = 0
        for i in range(wl.n_cached):
            tok, _ = wl.cached_seq(i)
            n = min(len(tok), len(p))
            neq = np.nonzero(tok[:n] != p[:n])[0]
            best = max(best, int(neq[0]) if len(neq) else n)
        assert best == pl[r]
