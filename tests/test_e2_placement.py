"""Request placement over several simulated instances: Algorithms 1 and 2 of the paper driven step by step.

Each instance is a cache of its own (prefix tree + page pool, as one GPU's local scheduler holds, Sec. 3.3).  For
every request of a stream the loop below asks each instance how much of the prompt it caches, what running the
request there would evict, and what its recent load is; it forms the load cost L + M + P of Algorithm 2 per
instance and lets Algorithm 1 choose.  The loop is run twice - on the library's host functions and on the oracle -
and the two must take the same decision at every step.  On the CPU the library side receives the cached lengths as
inputs (they are the matcher's output, and the matcher runs on the GPU); the GPU test takes them from
pa_match_prefixes on each instance's tree.

The paper's "GPUs with the longest node in the matched path" needs the nodes of a global tree, which is not built
here: the matched path is cut where the instances' cached lengths differ, the longest piece stands for the longest
node, and the instances that cache it are flagged (pa_e2_longest_piece, and its twin in the oracle).

Streams: prompts of the synthetic tool_use and agent_tree generators under several seeds (each seed is one
application with its own shared context), shuffled together.
"""
from collections import deque

import numpy as np
import pytest

from oracle import sched_oracle as so
from oracle.cache_oracle import CacheOracle
from paper_2407_00023_amd import workloads as W

COEF = (0.05, 2.0, 0.8, 1.0, 40.0)   # made-up regression: prefill 0.05/token + 2, decode 0.8/token + 1
WINDOW, IMBAL_R, LAG = 40, 0.97, 3


def stream(kind, seeds, rng):
    prompts = []
    for s in seeds:
        wl = W.small_variant(kind, seed=s)
        prompts += [wl.prompt(r).astype(np.int32) for r in range(wl.B)]
    order = rng.permutation(len(prompts))
    return [prompts[i] for i in order], rng.integers(5, 80, len(prompts)).tolist()


class OracleSide:
    def __init__(self, n_gpus, slots, page):
        self.caches = [CacheOracle(slots, page) for _ in range(n_gpus)]
        self.model = so.CostModel(*COEF)
        self.hist = so.ClusterHistory(n_gpus, WINDOW, self.model)

    def cached_len(self, g, toks):
        return self.caches[g].match(toks.tolist())[0]

    def free_slots(self, g):
        return self.caches[g].free_slots()

    def evict_plan_for(self, g, prompt, since):
        """-> (tokens per evicted run, sharers per run, admissions in the window); a run = consecutive dropped
        tokens, each the parent of the one before, with the same count: how a node shows in a per-token view."""
        per_token, linked, nreq = self.caches[g].evict_plan_for(prompt.tolist(), since)
        toks, shr = [], []
        for x, l in zip(per_token, linked):
            if shr and l and shr[-1] == x:
                toks[-1] += 1
            else:
                toks.append(1), shr.append(x)
        return toks, shr, nreq

    def load_cost(self, avg, et, es, nreq, missed):
        return so.load_cost(self.model, [], avg, et, es, nreq, missed)

    def schedule(self, *a):
        return so.e2_schedule(*a)

    def longest_piece(self, c):
        return [1 if x else 0 for x in so.longest_piece(c)]

    def evict_for(self, g, prompt):
        return self.caches[g].evict_for(prompt.tolist())

    def admit(self, g, toks, now):
        return self.caches[g].admit(toks.tolist(), now)

    def release(self, g, h):
        self.caches[g].release(h)


class LibSide:
    def __init__(self, pa, n_gpus, slots, page, cached_len):
        self.pa = pa
        self.trees = [pa.Tree() for _ in range(n_gpus)]
        for t in self.trees:
            t.attach_pool(slots, page)
            t.set_hit_window(WINDOW)
        self.model = pa.CostModel(*COEF)
        self.hist = pa.History(n_gpus, WINDOW, self.model)
        self.cached_len = cached_len   # (gpu, tokens) -> cached leading tokens on that instance

    def free_slots(self, g):
        return self.trees[g].free_slots()

    def evict_plan_for(self, g, prompt, since):
        toks, shr, nreq = self.trees[g].evict_plan_for(prompt, since)
        return toks.tolist(), shr.tolist(), nreq

    def load_cost(self, avg, et, es, nreq, missed):
        return self.pa.e2_load_cost(self.model, [], avg, et, es, nreq, missed)

    def schedule(self, *a):
        return self.pa.e2_schedule(*a)

    def longest_piece(self, c):
        return self.pa.e2_longest_piece(c).tolist()

    def evict_for(self, g, prompt):
        return self.trees[g].evict_for(prompt)

    def admit(self, g, toks, now):
        try:
            c, s, h = self.trees[g].admit(toks, now)
        except self.pa.PrefixAttnError as e:
            assert e.code == -2, e
            return None
        return c, s.tolist(), h

    def release(self, g, h):
        self.trees[g].release(h)




def run_cluster(side, prompts, out_lens, n_gpus, page, policy="e2"):
    """-> per request (gpu, mode, cached there, costs of all instances); total missed tokens."""
    log, live, now, missed_total = [], deque(), 0, 0
    for r, toks in enumerate(prompts):
        now += 1
        n = len(toks)
        c = [side.cached_len(g, toks) for g in range(n_gpus)]
        costs, ratios = [], []
        for g in range(n_gpus):
            L, ratio, _, avg = side.hist.gpu_load(g, now)
            missed = n - c[g]
            et, es, nreq = side.evict_plan_for(g, toks, now - WINDOW)
            _, M, P = side.load_cost(avg, et, es, nreq, missed)
            costs.append(L + M + P)
            ratios.append(ratio)
        if policy == "e2":
            gpu, mode = side.schedule(n, max(c), side.longest_piece(c), costs, ratios, IMBAL_R)
        else:
            gpu, mode = r % n_gpus, -1
        missed = n - c[gpu]
        side.evict_for(gpu, toks)
        res = side.admit(gpu, toks, now)
        if res is None:   # too much is pinned: the running requests finish first
            while live:
                g, h, o = live.popleft()
                side.release(g, h)
                side.hist.complete(g, now, o)
            side.evict_for(gpu, toks)
            res = side.admit(gpu, toks, now)
        assert res is not None and res[0] == c[gpu]
        side.hist.assign(gpu, now, missed)
        missed_total += missed
        live.append((gpu, res[2], out_lens[r]))
        if len(live) > LAG:
            g, h, o = live.popleft()
            side.release(g, h)
            side.hist.complete(g, now, o)
        log.append((gpu, mode, c[gpu], costs))
    return log, missed_total


def same_decisions(a, b):
    assert len(a) == len(b)
    for k, (x, y) in enumerate(zip(a, b)):
        assert x[:3] == y[:3], (k, x, y)
        assert y[3] == pytest.approx(x[3], rel=1e-9), (k, x, y)


@pytest.fixture(scope="module")
def pa():
    from paper_2407_00023_amd import binding
    return binding


class MirroredLibSide(LibSide):
    """The library side on a machine without a GPU: per-token caches kept in step with the library's trees stand in
    for the matcher and say how much of a prompt each instance caches.  Everything else is the library's."""

    def __init__(self, pa, n_gpus, slots, page):
        self.mirror = [CacheOracle(slots, page) for _ in range(n_gpus)]
        self.handles = []   # (gpu, library handle, mirror handle) of the running requests
        super().__init__(pa, n_gpus, slots, page, lambda g, toks: self.mirror[g].match(toks.tolist())[0])

    def evict_for(self, g, prompt):
        self.mirror[g].evict_for(prompt.tolist())
        return super().evict_for(g, prompt)

    def admit(self, g, toks, now):
        res = super().admit(g, toks, now)
        res_m = self.mirror[g].admit(toks.tolist(), now)
        assert (res is None) == (res_m is None)
        if res is not None:
            self.handles.append((g, res[2], res_m[2]))
        return res

    def release(self, g, h):
        k = next(k for k, (gg, hh, _) in enumerate(self.handles) if (gg, hh) == (g, h))
        self.mirror[g].release(self.handles.pop(k)[2])
        super().release(g, h)


@pytest.mark.parametrize("kind,slots", [("tool_use", 1024), ("agent_tree", 3072)])
def test_library_places_requests_as_the_oracle_does(pa, kind, slots):
    rng = np.random.default_rng(5)
    prompts, out_lens = stream(kind, range(8), rng)
    n_gpus, page = 4, 16
    evictions = []

    class Counting(OracleSide):
        def evict_for(self, g, prompt):
            res = super().evict_for(g, prompt)
            if res[1]:
                evictions.append(res)
            return res

    log_o, missed_o = run_cluster(Counting(n_gpus, slots, page), prompts, out_lens, n_gpus, page)
    log_l, missed_l = run_cluster(MirroredLibSide(pa, n_gpus, slots, page), prompts, out_lens, n_gpus, page)
    same_decisions(log_o, log_l)
    assert missed_o == missed_l
    modes = [m for _, m, _, _ in log_o]
    assert so.EXPLOIT in modes and so.EXPLORE_COST in modes          # both branches of Algorithm 1 were taken
    assert len(evictions) >= 3                                       # and the eviction term of the cost was live
    assert len(set(g for g, _, _, _ in log_o)) == n_gpus


@pytest.mark.parametrize("kind,slots", [("tool_use", 1024), ("agent_tree", 3072)])
def test_e2_recomputes_less_than_round_robin(kind, slots):
    """Not a number from the paper: the direction of its claim (prefix-aware placement saves recomputation) on
    these streams, evaluated with the oracle only."""
    rng = np.random.default_rng(5)
    prompts, out_lens = stream(kind, range(8), rng)
    _, missed_e2 = run_cluster(OracleSide(4, slots, 16), prompts, out_lens, 4, 16)
    _, missed_rr = run_cluster(OracleSide(4, slots, 16), prompts, out_lens, 4, 16, policy="rr")
    assert missed_e2 < missed_rr, (missed_e2, missed_rr)


@pytest.mark.gpu
@pytest.mark.parametrize("kind,slots", [("tool_use", 1024), ("agent_tree", 3072)])
def test_placement_driven_by_the_gpu_matcher(pa, gpu_device, kind, slots):
    import torch
    rng = np.random.default_rng(5)
    prompts, out_lens = stream(kind, range(4), rng)
    n_gpus, page = 4, 16
    orc = OracleSide(n_gpus, slots, page)
    log_o, missed_o = run_cluster(orc, prompts, out_lens, n_gpus, page)

    def cached_len(g, toks):
        t = lib.trees[g]
        t.upload()
        d_tok = torch.from_numpy(toks).to(gpu_device)
        d_off = torch.tensor([0, len(toks)], dtype=torch.int32, device=gpu_device)
        pl, _ = pa.match_prefixes(t, d_tok, d_off)
        return int(pl.cpu()[0])

    lib = LibSide(pa, n_gpus, slots, page, cached_len)
    log_l, missed_l = run_cluster(lib, prompts, out_lens, n_gpus, page)
    same_decisions(log_o, log_l)
    assert missed_o == missed_l
