"""Seeded synthetic workloads for the prefix-cached extend-prefill path.

This module only *draws inputs*: token ids, the list of cached sequences with the
KV slot of every token, request prompts, and Q/K/V values.  It holds none of the
method's arithmetic (no prefix matching, no attention) and imports neither the HIP
binding nor the CPU oracle; both sides consume exactly the arrays produced here.

Shapes follow the workload study of the paper (Table 1 and Appendix A: tool use,
embodied agents, long-document QA, video QA; 85-97 % of prompt tokens shared).  The
datasets themselves are not used; every array is random with the given seed.

Slot assignment.  The pool has ``num_slots // page_size`` pages.  Pages are handed
out from one seeded random permutation.  Every *segment* (a run of tokens that the
construction below makes new to the cache) receives ceil(len / page_size) whole
pages; token t of the segment sits in slot ``page[t // p] * p + t % p`` and the tail
of the last page stays unused.  Sequences that share a segment by construction carry
identical slots for it.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

_CHUNK = 1 << 22  # elements per independently seeded chunk (fixed: results do not depend on thread count)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to fp32 exactly."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _normal(seed_seq: np.random.SeedSequence, n: int, dtype: str) -> np.ndarray:
    """n i.i.d. N(0,1) values: fp32 array for 'f32', bf16 bit patterns (uint16) for 'bf16'."""
    n = int(n)
    out = np.empty(n, dtype=np.float32 if dtype == "f32" else np.uint16)
    nchunks = (n + _CHUNK - 1) // _CHUNK
    children = seed_seq.spawn(max(nchunks, 1))

    def fill(c):
        lo, hi = c * _CHUNK, min(n, (c + 1) * _CHUNK)
        x = np.random.default_rng(children[c]).standard_normal(hi - lo, dtype=np.float32)
        out[lo:hi] = x if dtype == "f32" else f32_to_bf16_bits(x)

    if nchunks <= 1:
        if n:
            fill(0)
    else:
        with ThreadPoolExecutor(max_workers=8) as ex:
            list(ex.map(fill, range(nchunks)))
    return out


class _Pages:
    """Hands out whole pages from a seeded random permutation."""

    def __init__(self, rng, num_slots: int, page_size: int):
        assert num_slots % page_size == 0
        self.p = page_size
        self.perm = rng.permutation(num_slots // page_size).astype(np.int64)
        self.cur = 0

    def take(self, ntok: int) -> np.ndarray:
        """Slots for a new segment of ntok tokens."""
        npg = (ntok + self.p - 1) // self.p
        if self.cur + npg > len(self.perm):
            raise ValueError("pool too small for workload")
        pg = self.perm[self.cur:self.cur + npg]
        self.cur += npg
        t = np.arange(ntok, dtype=np.int64)
        return (pg[t // self.p] * self.p + t % self.p).astype(np.int32)


class _Virtual:
    """Slot ids >= num_slots for cached tokens that no request can reach (never dereferenced)."""

    def __init__(self, num_slots: int, page_size: int):
        self.p = page_size
        self.next = num_slots

    def take(self, ntok: int) -> np.ndarray:
        npg = (ntok + self.p - 1) // self.p
        s = np.arange(self.next, self.next + ntok, dtype=np.int64).astype(np.int32)
        self.next += npg * self.p
        return s


@dataclass
class Workload:
    name: str
    dtype: str                 # 'f32' or 'bf16' (bf16 arrays are uint16 bit patterns)
    Hq: int
    Hkv: int
    D: int
    page_size: int
    num_slots: int
    vocab: int
    scale: float
    # cached sequences in insertion order (packed)
    cached_tokens: np.ndarray  # int32 [sum len]
    cached_slots: np.ndarray   # int32 [sum len]
    cached_offsets: np.ndarray  # int64 [nseq+1]
    # requests
    tokens: np.ndarray         # int32 [sum N_r]
    offsets: np.ndarray        # int32 [B+1]
    designed_prefix_len: np.ndarray  # int32 [B]
    designed_slots: np.ndarray  # int32 [sum N_r]: slot of each prompt position < designed prefix, else -1
    ext_len: np.ndarray        # int32 [B]
    ext_offsets: np.ndarray    # int32 [B+1]
    q_ext: np.ndarray          # [T, Hq, D]
    k_ext: np.ndarray          # [T, Hkv, D]
    v_ext: np.ndarray          # [T, Hkv, D]
    # KV already in the pool (rows for the slots a request can reach)
    pool_slots: np.ndarray     # int32 [n_backed]
    pool_k: np.ndarray         # [n_backed, Hkv, D]
    pool_v: np.ndarray         # [n_backed, Hkv, D]
    new_slots: np.ndarray      # int32 [T]: where append_kv puts the extend tokens' KV
    notes: dict = field(default_factory=dict)

    @property
    def B(self) -> int:
        return len(self.offsets) - 1

    @property
    def T(self) -> int:
        return int(self.ext_offsets[-1])

    def cached_seq(self, i: int):
        lo, hi = int(self.cached_offsets[i]), int(self.cached_offsets[i + 1])
        return self.cached_tokens[lo:hi], self.cached_slots[lo:hi]

    @property
    def n_cached(self) -> int:
        return len(self.cached_offsets) - 1

    def prompt(self, r: int) -> np.ndarray:
        return self.tokens[int(self.offsets[r]):int(self.offsets[r + 1])]


def _pack(seqs: List[np.ndarray], dtype):
    off = np.zeros(len(seqs) + 1, dtype=np.int64)
    for i, s in enumerate(seqs):
        off[i + 1] = off[i] + len(s)
    out = np.empty(int(off[-1]), dtype=dtype)
    for i, s in enumerate(seqs):
        out[off[i]:off[i + 1]] = s
    return out, off


def _finish(name, dtype, Hq, Hkv, D, page_size, num_slots, vocab, rng, seed,
            cached, req_prefix, ext_lens, forbidden_first, pages, backed_slots, notes=None) -> Workload:
    """Common tail: draw extend tokens, pack everything, draw Q/K/V.

    cached          list of (tokens, slots) in insertion order
    req_prefix      list of (tokens, slots): designed cached prefix of each request
    ext_lens        extend length of each request (>= 1)
    forbidden_first per request: token values the first extend token must avoid (the
                    tokens that, by construction, follow the designed prefix in some
                    cached sequence), so the designed prefix is also the longest match
    backed_slots    int32 array of slots whose KV rows are generated
    """
    B = len(req_prefix)
    prompts, dslots = [], []
    for r in range(B):
        ptok, pslot = req_prefix[r]
        e = rng.integers(0, vocab, size=int(ext_lens[r])).astype(np.int32)
        while int(e[0]) in forbidden_first[r]:
            e[0] = rng.integers(0, vocab)
        prompts.append(np.concatenate([ptok, e]).astype(np.int32))
        dslots.append(np.concatenate([pslot, np.full(len(e), -1, np.int32)]).astype(np.int32))
    tokens, off64 = _pack(prompts, np.int32)
    designed_slots, _ = _pack(dslots, np.int32)
    offsets = off64.astype(np.int32)
    ext_len = np.asarray(ext_lens, dtype=np.int32)
    ext_offsets = np.zeros(B + 1, dtype=np.int32)
    ext_offsets[1:] = np.cumsum(ext_len)
    T = int(ext_offsets[-1])
    new_slots = np.concatenate([pages.take(int(e)) for e in ext_len]) if B else np.zeros(0, np.int32)

    ctok, coff = _pack([c[0] for c in cached], np.int32)
    cslot, _ = _pack([c[1] for c in cached], np.int32)

    ss = np.random.SeedSequence([int(seed), 0x5EED])
    s_q, s_k, s_v, s_pk, s_pv = ss.spawn(5)
    nb = len(backed_slots)
    wl = Workload(
        name=name, dtype=dtype, Hq=Hq, Hkv=Hkv, D=D, page_size=page_size, num_slots=num_slots,
        vocab=vocab, scale=float(1.0 / np.sqrt(D)),
        cached_tokens=ctok, cached_slots=cslot, cached_offsets=coff,
        tokens=tokens, offsets=offsets,
        designed_prefix_len=np.asarray([len(p[0]) for p in req_prefix], dtype=np.int32),
        designed_slots=designed_slots,
        ext_len=ext_len, ext_offsets=ext_offsets,
        q_ext=_normal(s_q, T * Hq * D, dtype).reshape(T, Hq, D),
        k_ext=_normal(s_k, T * Hkv * D, dtype).reshape(T, Hkv, D),
        v_ext=_normal(s_v, T * Hkv * D, dtype).reshape(T, Hkv, D),
        pool_slots=np.asarray(backed_slots, dtype=np.int32),
        pool_k=_normal(s_pk, nb * Hkv * D, dtype).reshape(nb, Hkv, D),
        pool_v=_normal(s_pv, nb * Hkv * D, dtype).reshape(nb, Hkv, D),
        new_slots=new_slots.astype(np.int32),
        notes=notes or {},
    )
    return wl


def _unique_slots(parts: List[np.ndarray]) -> np.ndarray:
    if not parts:
        return np.zeros(0, np.int32)
    return np.unique(np.concatenate(parts)).astype(np.int32)


# --------------------------------------------------------------------------------------
# config 1: tiny fp32
# --------------------------------------------------------------------------------------
def tiny_fp32(seed=0, B=4, prefix=96, ext_lo=16, ext_hi=32, n_distract=8, dist_lo=64, dist_hi=128,
              Hq=4, Hkv=2, D=64, num_slots=512, page_size=1, vocab=32000, dtype="f32") -> Workload:
    """B requests sharing one cached prefix, each with its own new tokens; the tree also
    holds random distractor sequences.  Page size 1: slots fully shuffled.  The distractors
    (about 770 tokens) do not fit the 512-slot pool next to the prefix and the new tokens,
    so they carry slot ids >= num_slots that no request can reach."""
    rng = np.random.default_rng(seed)
    pages = _Pages(rng, num_slots, page_size)
    virt = _Virtual(num_slots, page_size)
    ptok = rng.integers(0, vocab, size=prefix).astype(np.int32)
    pslot = pages.take(prefix)
    cached = [(ptok, pslot)]
    for _ in range(n_distract):
        n = int(rng.integers(dist_lo, dist_hi + 1))
        cached.append((rng.integers(0, vocab, size=n).astype(np.int32), virt.take(n)))
    ext = rng.integers(ext_lo, ext_hi + 1, size=B)
    return _finish("tiny_fp32", dtype, Hq, Hkv, D, page_size, num_slots, vocab, rng, seed,
                   cached, [(ptok, pslot)] * B, ext, [set()] * B, pages, pslot)


# --------------------------------------------------------------------------------------
# config 2: tool-use shaped
# --------------------------------------------------------------------------------------
def tool_use(seed=0, B=64, sys_len=1800, n_tools=16, tool_lo=200, tool_hi=600, ext_lo=50, ext_hi=150,
             Hq=32, Hkv=8, D=128, num_slots=262144, page_size=16, vocab=128256, dtype="bf16", zipf=0.0,
             name="tool_use") -> Workload:
    """Every prompt = system prefix + one of n_tools tool-demonstration prefixes (all
    cached) + new tokens.  Stand-in for the tool-use workload (Table 1, first row).  With zipf > 0 the
    tool of a request is drawn with probability proportional to rank**-zipf instead of uniformly (the
    skewed tool popularity of the ablation study, which uses 1.1)."""
    rng = np.random.default_rng(seed)
    pages = _Pages(rng, num_slots, page_size)
    stok = rng.integers(0, vocab, size=sys_len).astype(np.int32)
    sslot = pages.take(sys_len)
    tools = []
    for _ in range(n_tools):
        n = int(rng.integers(tool_lo, tool_hi + 1))
        tools.append((rng.integers(0, vocab, size=n).astype(np.int32), pages.take(n)))
    cached = [(np.concatenate([stok, t]), np.concatenate([sslot, s])) for t, s in tools]
    if zipf > 0:
        weight = np.arange(1, n_tools + 1, dtype=np.float64) ** -float(zipf)
        which = rng.choice(n_tools, size=B, p=weight / weight.sum())
    else:
        which = rng.integers(0, n_tools, size=B)
    ext = rng.integers(ext_lo, ext_hi + 1, size=B)
    backed = _unique_slots([c[1] for c in cached])
    return _finish(name, dtype, Hq, Hkv, D, page_size, num_slots, vocab, rng, seed,
                   cached, [cached[int(w)] for w in which], ext, [set()] * B, pages, backed,
                   notes={"tool_of_request": which})


# --------------------------------------------------------------------------------------
# config 3: long-document QA shaped
# --------------------------------------------------------------------------------------
def long_doc_qa(seed=0, n_docs=4, per_doc=4, doc_len=16384, n_distract=12, ext_lo=20, ext_hi=80,
                Hq=32, Hkv=8, D=128, num_slots=524288, page_size=16, vocab=128256, dtype="bf16") -> Workload:
    """Groups of requests each sharing one cached document; distractor documents copy a
    real one up to a random position and then diverge.  Stand-in for long-document QA."""
    rng = np.random.default_rng(seed)
    pages = _Pages(rng, num_slots, page_size)
    docs = []
    for _ in range(n_docs):
        docs.append((rng.integers(0, vocab, size=doc_len).astype(np.int32), pages.take(doc_len)))
    cached = list(docs)
    for _ in range(n_distract):
        src = int(rng.integers(0, n_docs))
        cut = int(rng.integers(0, doc_len))
        tail = rng.integers(0, vocab, size=doc_len - cut).astype(np.int32)
        while cut < doc_len and tail[0] == docs[src][0][cut]:
            tail[0] = rng.integers(0, vocab)
        cached.append((np.concatenate([docs[src][0][:cut], tail]),
                       np.concatenate([docs[src][1][:cut], pages.take(doc_len - cut)])))
    B = n_docs * per_doc
    ext = rng.integers(ext_lo, ext_hi + 1, size=B)
    backed = _unique_slots([d[1] for d in docs])
    return _finish("long_doc_qa", dtype, Hq, Hkv, D, page_size, num_slots, vocab, rng, seed,
                   cached, [docs[r // per_doc] for r in range(B)], ext, [set()] * B, pages, backed)


# --------------------------------------------------------------------------------------
# config 4: agent / multi-turn shaped
# --------------------------------------------------------------------------------------
def agent_tree(seed=0, B=128, depth=4, branch=4, seg_len=512, ext_lo=200, ext_hi=1000,
               Hq=32, Hkv=8, D=128, num_slots=262144, page_size=16, vocab=128256, dtype="bf16") -> Workload:
    """Requests sit at leaves of a cached prefix tree (depth x branch, seg_len tokens per
    level); long extends put attention in the compute-bound regime."""
    rng = np.random.default_rng(seed)
    pages = _Pages(rng, num_slots, page_size)
    # level l holds branch**(l+1) segments; segment j at level l has parent j // branch at level l-1
    levels = []
    for l in range(depth):
        segs = []
        for j in range(branch ** (l + 1)):
            tok = rng.integers(0, vocab, size=seg_len).astype(np.int32)
            if j % branch:
                # siblings must start with different tokens so that they stay distinct children
                while any(tok[0] == s[0][0] for s in segs[j - j % branch:j]):
                    tok[0] = rng.integers(0, vocab)
            segs.append((tok, pages.take(seg_len)))
        levels.append(segs)
    n_leaves = branch ** depth

    def path(leaf):
        toks, slots = [], []
        for l in range(depth):
            j = leaf // (branch ** (depth - 1 - l))
            toks.append(levels[l][j][0])
            slots.append(levels[l][j][1])
        return np.concatenate(toks), np.concatenate(slots)

    cached = [path(leaf) for leaf in range(n_leaves)]
    leaf_of = rng.integers(0, n_leaves, size=B)
    ext = rng.integers(ext_lo, ext_hi + 1, size=B)
    backed = _unique_slots([s[1] for segs in levels for s in segs])
    return _finish("agent_tree", dtype, Hq, Hkv, D, page_size, num_slots, vocab, rng, seed,
                   cached, [cached[int(l)] for l in leaf_of], ext, [set()] * B, pages, backed,
                   notes={"leaf_of_request": leaf_of})


# --------------------------------------------------------------------------------------
# config 5: video-QA shaped, 70B attention shape
# --------------------------------------------------------------------------------------
def video_qa(seed=0, B=32, vis_len=8192, n_templates=8, tmpl_len=256, ext_lo=32, ext_hi=64,
             n_cached=4096, len_lo=1000, len_hi=9000,
             Hq=64, Hkv=8, D=128, num_slots=262144, page_size=16, vocab=128256, dtype="bf16") -> Workload:
    """All requests share one long cached prefix (stand-in visual tokens) followed by one
    of n_templates cached question templates.  The tree holds n_cached sequences: the
    template paths first, then sequences that copy a uniformly chosen earlier sequence up
    to a uniform cut and continue with random tokens.  Only template-path tokens own real
    slots; all other cached tokens get slot ids >= num_slots that are never dereferenced."""
    rng = np.random.default_rng(seed)
    pages = _Pages(rng, num_slots, page_size)
    virt = _Virtual(num_slots, page_size)
    vtok = rng.integers(0, vocab, size=vis_len).astype(np.int32)
    vslot = pages.take(vis_len)
    cached = []
    for t in range(n_templates):
        tok = rng.integers(0, vocab, size=tmpl_len).astype(np.int32)
        while any(tok[0] == c[0][vis_len] for c in cached):
            tok[0] = rng.integers(0, vocab)
        cached.append((np.concatenate([vtok, tok]), np.concatenate([vslot, pages.take(tmpl_len)])))
    path_len = vis_len + tmpl_len
    # continuation[t]: tokens that follow template path t in some later cached sequence
    continuation = [set() for _ in range(n_templates)]
    holds_template = list(range(n_templates))  # per cached sequence: template index it fully contains, or -1
    for k in range(n_templates, n_cached):
        n = int(rng.integers(len_lo, len_hi + 1))
        src = int(rng.integers(0, k))
        cut = int(rng.integers(0, min(n, len(cached[src][0])) + 1))
        tail = rng.integers(0, vocab, size=n - cut).astype(np.int32)
        cached.append((np.concatenate([cached[src][0][:cut], tail]),
                       np.concatenate([cached[src][1][:cut], virt.take(n - cut)])))
        ht = holds_template[src] if cut >= path_len else -1
        holds_template.append(ht)
        if ht >= 0 and n > path_len:
            continuation[ht].add(int(cached[-1][0][path_len]))
    which = rng.integers(0, n_templates, size=B)
    ext = rng.integers(ext_lo, ext_hi + 1, size=B)
    backed = _unique_slots([c[1] for c in cached[:n_templates]])
    return _finish("video_qa", dtype, Hq, Hkv, D, page_size, num_slots, vocab, rng, seed,
                   cached, [cached[int(w)] for w in which], ext, [continuation[int(w)] for w in which],
                   pages, backed, notes={"template_of_request": which})


# --------------------------------------------------------------------------------------
# config 6: program-generation shaped
# --------------------------------------------------------------------------------------
def programming(seed=0, B=64, sys_len=1500, n_problems=6, n_new=3, prob_mean=2371, prob_sd=1656, prob_lo=200,
                prob_hi=7000, gen_lo=1, gen_hi=8, Hq=32, Hkv=8, D=128, num_slots=262144, page_size=16,
                vocab=128256, dtype="bf16") -> Workload:
    """Every prompt = one system prompt of code demonstrations + a problem description.  n_problems
    problems are cached with it; most requests are further generations for a cached problem (everything
    but their last gen_lo..gen_hi tokens is cached), n_new requests bring a problem that is not cached yet
    and prefill all of it behind the cached system prompt.  Stand-in for the programming workload
    (Table 1, third row: prompts of 3,871 +- 1,656 tokens, 97 % shared)."""
    rng = np.random.default_rng(seed)
    pages = _Pages(rng, num_slots, page_size)
    stok = rng.integers(0, vocab, size=sys_len).astype(np.int32)
    sslot = pages.take(sys_len)

    def problem_len():
        return int(np.clip(rng.normal(prob_mean, prob_sd), prob_lo, prob_hi))

    cached, firsts = [], set()
    for _ in range(n_problems):
        n = problem_len()
        t = rng.integers(0, vocab, size=n).astype(np.int32)
        while int(t[0]) in firsts:
            t[0] = rng.integers(0, vocab)
        firsts.add(int(t[0]))
        cached.append((np.concatenate([stok, t]), np.concatenate([sslot, pages.take(n)])))
    is_new = np.zeros(B, dtype=bool)
    is_new[rng.choice(B, size=min(n_new, B), replace=False)] = True
    which = rng.integers(0, n_problems, size=B)
    req_prefix, ext, forbidden = [], [], []
    for r in range(B):
        if is_new[r]:
            req_prefix.append((stok, sslot))
            ext.append(problem_len())
            forbidden.append(firsts)
        else:
            req_prefix.append(cached[int(which[r])])
            ext.append(int(rng.integers(gen_lo, gen_hi + 1)))
            forbidden.append(set())
    backed = _unique_slots([c[1] for c in cached])
    return _finish("programming", dtype, Hq, Hkv, D, page_size, num_slots, vocab, rng, seed,
                   cached, req_prefix, ext, forbidden, pages, backed,
                   notes={"new_problem": is_new, "problem_of_request": which})


# --------------------------------------------------------------------------------------
# decode-phase batch of the tool-use shape
# --------------------------------------------------------------------------------------
def decode(seed=0, B=256, sys_len=1800, n_tools=16, tool_lo=200, tool_hi=600, own_lo=51, own_hi=350, ext=1,
           Hq=32, Hkv=8, D=128, num_slots=262144, page_size=16, vocab=128256, dtype="bf16") -> Workload:
    """A batch in the decoding phase: every request's prompt and the tokens it has generated so far are
    cached (system prefix + one of n_tools tool prefixes, shared; then own_lo..own_hi tokens of its own: its
    question and its output so far) and it brings `ext` new tokens (one).  The tool-use shape (Table 1, first row:
    43-token outputs behind 1,835-token prompts) in the phase the paper calls the decoding-phase unit
    (Sec. 3.3)."""
    rng = np.random.default_rng(seed)
    pages = _Pages(rng, num_slots, page_size)
    stok = rng.integers(0, vocab, size=sys_len).astype(np.int32)
    sslot = pages.take(sys_len)
    tools = []
    for _ in range(n_tools):
        n = int(rng.integers(tool_lo, tool_hi + 1))
        tools.append((rng.integers(0, vocab, size=n).astype(np.int32), pages.take(n)))
    which = rng.integers(0, n_tools, size=B)
    cached, firsts = [], [set() for _ in range(n_tools)]
    for r in range(B):
        w = int(which[r])
        n = int(rng.integers(own_lo, own_hi + 1))
        own = rng.integers(0, vocab, size=n).astype(np.int32)
        while int(own[0]) in firsts[w]:     # requests on one tool part ways at their first own token
            own[0] = rng.integers(0, vocab)
        firsts[w].add(int(own[0]))
        cached.append((np.concatenate([stok, tools[w][0], own]), np.concatenate([sslot, tools[w][1], pages.take(n)])))
    backed = _unique_slots([c[1] for c in cached])
    # (a pair (lo, hi) draws the number of new tokens per request; the default draws nothing, so the default batch
    # stays what it was)
    ext_lens = rng.integers(ext[0], ext[1] + 1, size=B) if isinstance(ext, tuple) else np.full(B, int(ext), dtype=np.int64)
    return _finish("decode", dtype, Hq, Hkv, D, page_size, num_slots, vocab, rng, seed,
                   cached, list(cached), ext_lens, [set()] * B, pages, backed,
                   notes={"tool_of_request": which})


CONFIGS = {
    "tiny_fp32": tiny_fp32,
    "tool_use": tool_use,
    "long_doc_qa": long_doc_qa,
    "agent_tree": agent_tree,
    "video_qa": video_qa,
    "programming": programming,
    "tool_use_zipf": lambda seed=0: tool_use(seed, zipf=1.1, name="tool_use_zipf"),
    "decode": decode,
}


def small_variant(name: str, seed: int = 0) -> Workload:
    """Reduced versions of the bf16 configs: same structure, sizes an fp64 CPU oracle
    finishes in seconds, still several tiles plus ragged tails."""
    if name == "tool_use":
        return tool_use(seed, B=6, sys_len=333, n_tools=3, tool_lo=40, tool_hi=130, ext_lo=5, ext_hi=70,
                        Hq=8, Hkv=2, num_slots=4096)
    if name == "tool_use_zipf":
        return tool_use(seed, B=9, sys_len=333, n_tools=4, tool_lo=40, tool_hi=130, ext_lo=5, ext_hi=70,
                        Hq=8, Hkv=2, num_slots=4096, zipf=1.1, name="tool_use_zipf")
    if name == "decode":
        return decode(seed, B=11, sys_len=333, n_tools=3, tool_lo=40, tool_hi=130, own_lo=3, own_hi=90,
                      Hq=8, Hkv=2, num_slots=8192)
    if name == "long_doc_qa":
        return long_doc_qa(seed, n_docs=2, per_doc=2, doc_len=1500, n_distract=3, ext_lo=3, ext_hi=40,
                           Hq=8, Hkv=2, num_slots=16384)
    if name == "agent_tree":
        return agent_tree(seed, B=5, depth=2, branch=2, seg_len=100, ext_lo=60, ext_hi=300,
                          Hq=8, Hkv=2, num_slots=4096)
    if name == "video_qa":
        return video_qa(seed, B=4, vis_len=700, n_templates=2, tmpl_len=50, ext_lo=8, ext_hi=33,
                        n_cached=40, len_lo=100, len_hi=900, Hq=16, Hkv=2, num_slots=4096)
    if name == "programming":
        return programming(seed, B=7, sys_len=300, n_problems=2, n_new=2, prob_mean=400, prob_sd=250, prob_lo=60,
                           prob_hi=900, gen_lo=1, gen_hi=5, Hq=8, Hkv=2, num_slots=8192)
    if name == "tiny_fp32":
        return tiny_fp32(seed)
    raise KeyError(name)
