"""Pins for the oracle of the scheduling rules (CPU only), and the library's host functions against it.

Pins that are not the oracle itself: the worked example the paper prints in Sec. 3.3 (63 of 100 tokens cached with
P = 10 is group 6; 55 picks take 10, 9, ..., 1 from groups 10..1), hand-worked cases of the documented readings
(tests/golden/priority_worked_example.txt), the inequality that defines a group (g / P <= cached / prompt <
(g + 1) / P), the quota property of a proportional share, closed forms of the load cost with unit coefficients, the
strict inequality of the exploit test of Algorithm 1, and window edges of the history.  Every test runs on the oracle
and on the library; then the two are compared on random inputs.
"""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import sched_oracle as so
from oracle.cache_oracle import CacheOracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "priority_worked_example.txt")


@pytest.fixture(scope="module")
def pa():
    from paper_2407_00023_amd import binding
    return binding


class OracleImpl:
    name = "oracle"

    def group(self, c, n, P):
        return so.priority_group(c, n, P)

    def select(self, c, n, P, k):
        return list(so.priority_select(c, n, P, k))

    def model(self, a, b, c, d, e):
        return so.CostModel(a, b, c, d, e)

    def load_cost(self, m, hist, avg, et, es, nreq, missed):
        return so.load_cost(m, hist, avg, et, es, nreq, missed)

    def schedule(self, n, c, flags, cost, ratio, imbal):
        return so.e2_schedule(n, c, flags, cost, ratio, imbal)

    def history(self, n_gpus, window, m):
        return so.ClusterHistory(n_gpus, window, m)


class LibImpl:
    name = "library"

    def __init__(self, pa):
        self.pa = pa

    def group(self, c, n, P):
        return self.pa.priority_group(c, n, P)

    def select(self, c, n, P, k):
        return self.pa.priority_select(c, n, P, k).tolist()

    def model(self, a, b, c, d, e):
        return self.pa.CostModel(a, b, c, d, e)

    def load_cost(self, m, hist, avg, et, es, nreq, missed):
        return self.pa.e2_load_cost(m, hist, avg, et, es, nreq, missed)

    def schedule(self, n, c, flags, cost, ratio, imbal):
        return self.pa.e2_schedule(n, c, flags, cost, ratio, imbal)

    def history(self, n_gpus, window, m):
        return self.pa.History(n_gpus, window, m)


@pytest.fixture(params=["oracle", "library"])
def impl(request, pa):
    return OracleImpl() if request.param == "oracle" else LibImpl(pa)


def golden_lines(kind):
    for raw in open(GOLDEN):
        line = raw.split("#")[0].strip()
        if line.startswith(kind + " "):
            yield line[len(kind):].strip()


def queue_with(waiting_per_group, P, rng=None):
    """A waiting queue with the given number of requests in each group 0..P, in a shuffled arrival order."""
    cached, prompt = [], []
    for g, w in enumerate(waiting_per_group):
        for _ in range(w):
            prompt.append(10 * P)
            cached.append(10 * g)  # exactly g P-ths cached
    order = np.arange(len(cached)) if rng is None else rng.permutation(len(cached))
    return [cached[i] for i in order], [prompt[i] for i in order]


# ---- the paper's worked example and the hand-worked readings ------------------------------------------------------
def test_group_of_the_worked_example(impl):
    for line in golden_lines("group"):
        lhs, rhs = line.split("->")
        c, n, P = map(int, lhs.split())
        assert impl.group(c, n, P) == int(rhs)


def test_selection_of_the_worked_example(impl):
    for line in golden_lines("select"):
        lhs, rhs = line.split("->")
        picks, P = map(int, lhs.split())
        want = list(map(int, rhs.split()))  # groups P .. 1
        cached, prompt = queue_with([picks] * (P + 1), P, np.random.default_rng(1))
        batch = impl.select(cached, prompt, P, picks)
        per_group = np.bincount([cached[i] // 10 for i in batch], minlength=P + 1)
        assert per_group[1:][::-1].tolist() == want and per_group[0] == 0


def test_hand_worked_selections(impl):
    n = 0
    for line in golden_lines("hand"):
        head, rest = line.split("|")
        P, picks = map(int, head.split())
        waiting, taken = (list(map(int, x.split())) for x in rest.split("->"))
        assert len(waiting) == P + 1 == len(taken)
        cached, prompt = queue_with(waiting, P, np.random.default_rng(7))
        batch = impl.select(cached, prompt, P, picks)
        assert np.bincount([cached[i] // 10 for i in batch], minlength=P + 1).tolist() == taken, line
        n += 1
    assert n >= 4


# ---- what defines a group ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("P", [1, 2, 3, 10, 16])
def test_group_is_the_whole_number_of_pths_cached(impl, P):
    for n in range(1, 41):
        for c in range(0, n + 1):
            g = impl.group(c, n, P)
            assert 0 <= g <= P
            assert g * n <= P * c, (c, n, P, g)            # g / P <= c / n
            if c < n:
                assert P * c < (g + 1) * n, (c, n, P, g)   # c / n < (g + 1) / P
            else:
                assert g == P                              # only a fully cached prompt is in the top group
    assert impl.group(0, 0, P) == 0


# ---- properties of a batch -----------------------------------------------------------------------------------------
def check_batch(cached, prompt, P, n_pick, batch, group_of):
    groups = [group_of(c, n, P) for c, n in zip(cached, prompt)]
    assert len(batch) == min(n_pick, len(cached))
    assert len(set(batch)) == len(batch)
    got = [groups[i] for i in batch]
    assert got == sorted(got, reverse=True)                       # higher groups first
    for g in range(P + 1):
        members = [i for i, x in enumerate(groups) if x == g]
        mine = [i for i in batch if groups[i] == g]
        assert mine == members[:len(mine)]                        # arrival order inside a group
    left_waiting = [sum(1 for i, x in enumerate(groups) if x == g and i not in set(batch)) for g in range(P + 1)]
    taken = np.bincount(got, minlength=P + 1)
    if taken[0] > 0:                                              # group 0 only fills what the others cannot
        assert all(left_waiting[g] == 0 for g in range(1, P + 1))
    return taken


@pytest.mark.parametrize("seed", range(12))
def test_batch_properties_on_random_queues(impl, seed):
    rng = np.random.default_rng(seed)
    P = int(rng.choice([1, 2, 4, 10]))
    n_wait = int(rng.integers(0, 120))
    prompt = rng.integers(1, 400, n_wait)
    cached = np.minimum(prompt, (prompt * rng.random(n_wait) * rng.choice([0, 1, 1.3], n_wait)).astype(np.int64))
    for n_pick in [0, 1, 7, 55, 200]:
        batch = impl.select(cached.tolist(), prompt.tolist(), P, n_pick)
        check_batch(cached.tolist(), prompt.tolist(), P, n_pick, batch, so.priority_group)


@pytest.mark.parametrize("P,n_pick", [(10, 55), (10, 7), (10, 100), (4, 9), (3, 50), (16, 31)])
def test_share_is_proportional_when_no_group_is_short(impl, P, n_pick):
    cached, prompt = queue_with([n_pick] * (P + 1), P, np.random.default_rng(P))
    batch = impl.select(cached, prompt, P, n_pick)
    taken = check_batch(cached, prompt, P, n_pick, batch, so.priority_group)
    W = P * (P + 1) // 2
    for g in range(P + 1):
        quota = Fraction(n_pick * g, W)
        assert abs(taken[g] - quota) < 1, (g, taken[g], quota)   # the quota property of largest remainders
    assert all(taken[g] <= taken[g + 1] for g in range(P))       # a higher group never gets fewer
    assert taken[0] == 0


# ---- load cost -----------------------------------------------------------------------------------------------------
def test_load_cost_closed_forms(impl):
    m = impl.model(1.0, 0.0, 1.0, 0.0, 5.0)  # one time unit per token, no constant
    hist, et, es = [100, 0, 30], [40, 8], [3, 1]
    L, M, P = impl.load_cost(m, hist, 20.0, et, es, 4, 77)
    assert L == 130 + 3 * 20          # missed tokens of the window + one average decode per request
    assert M == 40 * 3 / 4 + 8 * 1 / 4
    assert P == 77
    m2 = impl.model(0.5, 10.0, 0.25, 2.0, 5.0)
    L, M, P = impl.load_cost(m2, hist, 20.0, et, es, 4, 0)
    assert L == pytest.approx((0.5 * 100 + 10) + 0 + (0.5 * 30 + 10) + 3 * (0.25 * 20 + 2))  # no constant for 0 tokens
    assert M == pytest.approx((0.5 * 40 + 10) * 0.75 + (0.5 * 8 + 10) * 0.25)
    assert P == 0.0
    assert impl.load_cost(m2, [], 20.0, [], [], 0, 10) == (0.0, 0.0, 15.0)
    assert impl.load_cost(m2, [], 20.0, [40], [0], 9, 0)[1] == 0.0     # evicting what nobody used costs nothing
    assert impl.load_cost(m2, [], 20.0, [40], [3], 0, 0)[1] == 0.0     # empty window


def test_load_cost_grows_with_each_term(impl):
    m = impl.model(0.3, 4.0, 0.1, 1.0, 50.0)
    base = sum(impl.load_cost(m, [10, 20], 30.0, [5], [1], 2, 40))
    assert sum(impl.load_cost(m, [10, 20, 1], 30.0, [5], [1], 2, 40)) > base
    assert sum(impl.load_cost(m, [10, 20], 31.0, [5], [1], 2, 40)) > base
    assert sum(impl.load_cost(m, [10, 20], 30.0, [5, 5], [1, 1], 2, 40)) > base
    assert sum(impl.load_cost(m, [10, 20], 30.0, [5], [2], 2, 40)) > base
    assert sum(impl.load_cost(m, [10, 20], 30.0, [5], [1], 2, 41)) > base


# ---- Algorithm 1 ---------------------------------------------------------------------------------------------------
def test_exploit_needs_strictly_more_cached_than_missed(impl):
    flags, cost, ratio = [0, 1, 1, 0], [1.0, 9.0, 8.0, 0.5], [0.1, 0.1, 0.1, 0.1]
    assert impl.schedule(100, 51, flags, cost, ratio, 0.9) == (2, so.EXPLOIT)        # cheapest of the flagged GPUs
    assert impl.schedule(100, 50, flags, cost, ratio, 0.9) == (3, so.EXPLORE_COST)   # 50 missed is not < 50 cached
    assert impl.schedule(100, 49, flags, cost, ratio, 0.9) == (3, so.EXPLORE_COST)
    assert impl.schedule(100, 100, flags, cost, ratio, 0.9) == (2, so.EXPLOIT)
    assert impl.schedule(100, 0, flags, cost, ratio, 0.9) == (3, so.EXPLORE_COST)


def test_explore_prefers_a_gpu_heavy_with_decoding(impl):
    flags, cost = [0, 0, 0], [3.0, 1.0, 2.0]
    assert impl.schedule(100, 10, flags, cost, [0.2, 0.3, 0.95], 0.9) == (2, so.EXPLORE_DECODE)
    assert impl.schedule(100, 10, flags, cost, [0.2, 0.3, 0.9], 0.9) == (1, so.EXPLORE_COST)  # not above the limit
    assert impl.schedule(100, 90, [0, 0, 1], cost, [0.99, 0.3, 0.1], 0.9) == (2, so.EXPLOIT)   # exploit comes first


def test_ties_go_to_the_lowest_index_and_no_flag_means_explore(impl):
    assert impl.schedule(10, 9, [1, 1, 1], [2.0, 1.0, 1.0], [0, 0, 0], 0.5) == (1, so.EXPLOIT)
    assert impl.schedule(10, 1, [0, 0, 0], [2.0, 1.0, 1.0], [0, 0, 0], 0.5) == (1, so.EXPLORE_COST)
    assert impl.schedule(10, 1, [0, 0, 0], [2.0, 1.0, 1.0], [0.7, 0.8, 0.8], 0.5) == (1, so.EXPLORE_DECODE)
    assert impl.schedule(10, 9, [0, 0, 0], [2.0, 1.0, 3.0], [0, 0, 0], 0.5) == (1, so.EXPLORE_COST)


def test_longest_piece_of_the_matched_path(pa):
    for impl in (so.longest_piece, lambda c: [bool(x) for x in pa.e2_longest_piece(c).tolist()]):
        assert impl([0, 0, 0]) == [False, False, False]
        assert impl([1800, 2200, 0, 1800]) == [True, True, False, True]      # pieces 1800 and 400: the first
        assert impl([100, 900, 0, 900]) == [False, True, False, True]        # pieces 100 and 800: the second
        assert impl([500, 1000]) == [True, True]                             # equal pieces: the earlier one
        assert impl([7]) == [True]
    rng = np.random.default_rng(5)
    for _ in range(200):
        c = rng.integers(0, 6, int(rng.integers(1, 9))) * int(rng.integers(1, 50))
        assert [bool(x) for x in pa.e2_longest_piece(c).tolist()] == so.longest_piece(c.tolist())


# ---- history window ------------------------------------------------------------------------------------------------
def test_history_window_edges_and_ratio(impl):
    m = impl.model(1.0, 0.0, 2.0, 0.0, 7.0)
    h = impl.history(2, 10, m)
    h.assign(0, 1, 100)
    h.assign(0, 5, 50)
    h.assign(1, 5, 9)
    L, ratio, n, avg = h.gpu_load(0, 5)
    assert (n, avg) == (2, 7.0) and L == 150 + 2 * 14 and ratio == pytest.approx(28 / 178)  # default output length
    h.complete(0, 6, 10)
    h.complete(0, 7, 30)
    L, ratio, n, avg = h.gpu_load(0, 10)
    assert (n, avg) == (2, 20.0) and L == 150 + 2 * 40
    L, ratio, n, avg = h.gpu_load(0, 11)      # the request of time 1 is exactly one window old: out
    assert n == 1 and L == 50 + 40
    L, ratio, n, avg = h.gpu_load(0, 16)      # the output seen at time 6 is out, the one of time 7 still in
    assert n == 0 and L == 0 and ratio == 0 and avg == 30.0
    assert h.gpu_load(1, 14)[2] == 1 and h.gpu_load(1, 15)[2] == 0
    assert h.gpu_load(0, 40) == (0.0, 0.0, 0, 7.0)


# ---- library against oracle on random inputs ----------------------------------------------------------------------
@pytest.mark.parametrize("seed", range(40))
def test_library_selects_what_the_oracle_selects(pa, seed):
    rng = np.random.default_rng(1000 + seed)
    P = int(rng.integers(1, 13))
    n_wait = int(rng.integers(0, 300))
    prompt = rng.integers(0, 500, n_wait)
    cached = (prompt * rng.random(n_wait) * rng.choice([0, 1, 1, 1.2], n_wait)).astype(np.int64)
    cached = np.minimum(cached, prompt)
    for n_pick in [0, 1, int(rng.integers(0, 400)), int(rng.integers(0, 60)), n_wait]:
        a = so.priority_select(cached.tolist(), prompt.tolist(), P, n_pick)
        b = pa.priority_select(cached, prompt, P, n_pick).tolist()
        assert a == b
    for c, n in zip(cached[:50].tolist(), prompt[:50].tolist()):
        assert so.priority_group(c, n, P) == pa.priority_group(c, n, P)


@pytest.mark.parametrize("seed", range(20))
def test_library_costs_and_decisions_match_the_oracle(pa, seed):
    rng = np.random.default_rng(2000 + seed)
    coef = [float(x) for x in rng.random(5) * [1, 20, 1, 5, 100]]
    mo, ml = so.CostModel(*coef), pa.CostModel(*coef)
    for _ in range(20):
        hist = rng.integers(0, 4000, int(rng.integers(0, 50))).tolist()
        ne = int(rng.integers(0, 8))
        et, es = rng.integers(1, 900, ne).tolist(), rng.integers(0, 12, ne).tolist()
        nreq, missed, avg = int(rng.integers(0, 40)), int(rng.integers(0, 3000)), float(rng.random() * 300)
        a = so.load_cost(mo, hist, avg, et, es, nreq, missed)
        b = pa.e2_load_cost(ml, hist, avg, et, es, nreq, missed)
        assert b == pytest.approx(a, rel=1e-13, abs=0)
        n_gpus = int(rng.integers(1, 9))
        cost = np.round(rng.random(n_gpus) * 4, 1)      # coarse values: ties happen
        ratio = np.round(rng.random(n_gpus), 1)
        flags = rng.integers(0, 2, n_gpus)
        n = int(rng.integers(1, 200))
        c = int(rng.integers(0, n + 1))
        imbal = float(rng.choice([0.3, 0.8, 2.0]))
        assert pa.e2_schedule(n, c, flags, cost, ratio, imbal) == so.e2_schedule(n, c, flags.tolist(), cost.tolist(), ratio.tolist(), imbal)


@pytest.mark.parametrize("seed", range(10))
def test_library_history_matches_the_oracle(pa, seed):
    rng = np.random.default_rng(3000 + seed)
    coef = [float(x) for x in rng.random(5) * [1, 20, 1, 5, 100]]
    n_gpus, window = 3, int(rng.integers(1, 30))
    ho, hl = so.ClusterHistory(n_gpus, window, so.CostModel(*coef)), pa.History(n_gpus, window, pa.CostModel(*coef))
    now = 0
    for _ in range(300):
        now += int(rng.integers(0, 4))
        g = int(rng.integers(0, n_gpus))
        op = rng.random()
        if op < 0.5:
            x = int(rng.integers(0, 2000))
            ho.assign(g, now, x), hl.assign(g, now, x)
        elif op < 0.75:
            x = int(rng.integers(0, 300))
            ho.complete(g, now, x), hl.complete(g, now, x)
        else:
            a, b = ho.gpu_load(g, now), hl.gpu_load(g, now)
            assert b[2] == a[2] and b == pytest.approx(a, rel=1e-12, abs=0)


def test_error_paths(pa):
    with pytest.raises(pa.PrefixAttnError):
        pa.priority_group(1, 2, 0)
    with pytest.raises(pa.PrefixAttnError):
        pa.priority_select([-1], [5], 4, 1)
    with pytest.raises(pa.PrefixAttnError):
        pa.e2_schedule(10, 11, [0], [1.0], [0.0], 0.5)
    h = pa.History(2, 5, pa.CostModel(1, 0, 1, 0, 1))
    with pytest.raises(pa.PrefixAttnError):
        h.assign(2, 1, 5)
    h.assign(0, 5, 5)
    with pytest.raises(pa.PrefixAttnError):
        h.assign(0, 4, 5)


# ---- what an eviction would drop (the E of Algorithm 2) -----------------------------------------------------------
def runs_of(per_token, linked):
    """Dropped tokens grouped into runs: consecutive, each the parent of the one before, same count."""
    runs = []
    for x, l in zip(per_token, linked):
        if runs and l and runs[-1][1] == x:
            runs[-1][0] += 1
        else:
            runs.append([1, x])
    return [(n, x) for n, x in runs]


def random_cache_history(rng, lib_tree, orc, steps, now=0, vocab=6, max_len=40, release_all=False):
    """The same random admissions, releases and evictions on both sides; returns the time reached."""
    held = []
    stems = [rng.integers(0, vocab, int(rng.integers(4, max_len))) for _ in range(6)]
    for _ in range(steps):
        op = rng.random()
        if op < 0.6:
            stem = stems[int(rng.integers(0, len(stems)))]
            cut = int(rng.integers(1, len(stem) + 1))
            toks = np.concatenate([stem[:cut], rng.integers(0, vocab, int(rng.integers(0, 12)))]).astype(np.int32)
            now += int(rng.integers(1, 4))
            a = orc.admit(toks.tolist(), now)
            if a is None:
                need = len(toks)
                assert lib_tree.evict(need) == orc.evict(need)
                now += 1
                a = orc.admit(toks.tolist(), now)
                if a is None:
                    continue
            c, s, h = lib_tree.admit(toks, now)
            assert c == a[0] and s.tolist() == a[1]
            held.append((h, a[2]))
        elif op < 0.9 and held:
            h, ho = held.pop(int(rng.integers(0, len(held))))
            lib_tree.release(h), orc.release(ho)
    while release_all and held:
        h, ho = held.pop()
        lib_tree.release(h), orc.release(ho)
    return now


@pytest.mark.parametrize("seed", range(25))
def test_eviction_plan_names_what_eviction_then_drops(pa, seed):
    rng = np.random.default_rng(4000 + seed)
    page = int(rng.choice([1, 2, 4, 8]))
    slots = page * int(rng.integers(40, 120))
    window = int(rng.integers(5, 60))
    t, orc = pa.Tree(), CacheOracle(slots, page)
    t.attach_pool(slots, page)
    if seed % 2:
        t.set_hit_window(window)   # forgetting old admissions must not change what is counted inside the window
    now = random_cache_history(rng, t, orc, 150)
    for _ in range(6):
        need = int(rng.integers(0, slots // 2))
        since = now - int(rng.integers(0, window + 1))
        toks, shr, nreq = t.evict_plan(need, since)
        per_token, linked, nreq_o = orc.evict_plan(need, since)
        assert nreq == nreq_o
        assert np.repeat(shr.numpy(), toks.numpy()).tolist() == per_token   # same tokens, same order, same counts
        assert toks.tolist() == [n for n, _ in runs_of(per_token, linked)]  # cut where the path or the count changes
        assert (toks.numpy() > 0).all()
        before = (t.free_slots(), t.stats())
        assert before[0] == orc.free_slots() and before[1][1] == orc.tokens_cached()   # a plan changes nothing
        # and the eviction itself then drops exactly the planned number of tokens
        if rng.random() < 0.5:
            freed, gone = t.evict(need)
            assert (freed, gone) == orc.evict(need) and gone == int(toks.sum())
            now = random_cache_history(rng, t, orc, 10, now)


@pytest.mark.parametrize("seed", range(25))
def test_making_room_for_a_prompt_spares_its_cached_part(pa, seed):
    rng = np.random.default_rng(5000 + seed)
    page = int(rng.choice([1, 2, 4, 8]))
    slots = max(64, page * int(rng.integers(12, 30)))   # tight: most prompts below need room made
    t, orc = pa.Tree(), CacheOracle(slots, page)
    t.attach_pool(slots, page)
    now = random_cache_history(rng, t, orc, 120, release_all=True)
    made_room = 0
    for _ in range(8):
        # a prompt that continues something cached (often ending inside a node), then new tokens
        path, node = [], orc.root
        while node.child and rng.random() < 0.93:
            tok = list(node.child)[int(rng.integers(0, len(node.child)))]
            path.append(tok)
            node = node.child[tok]
        prompt = np.array(path + rng.integers(100, 200, int(rng.integers(1, slots // 2))).tolist(), np.int32)
        cached_before = orc.match(prompt.tolist())[0]
        assert cached_before >= len(path)
        since = now - int(rng.integers(0, 40))
        toks, shr, nreq = t.evict_plan_for(prompt, since)
        per_token, linked, nreq_o = orc.evict_plan_for(prompt.tolist(), since)
        assert nreq == nreq_o and np.repeat(shr.numpy(), toks.numpy()).tolist() == per_token
        assert toks.tolist() == [n for n, _ in runs_of(per_token, linked)]
        res = t.evict_for(prompt)
        assert res == orc.evict_for(prompt.tolist())
        made_room += res[1] > 0 and cached_before > 0
        assert orc.match(prompt.tolist())[0] == cached_before               # nothing of the cached part went
        assert t.free_slots() == orc.free_slots() and t.stats()[1] == orc.tokens_cached()
        now += 1
        a = orc.admit(prompt.tolist(), now)
        if a is None:                                                        # pinned tokens stand in the way
            with pytest.raises(pa.PrefixAttnError):
                t.admit(prompt, now)
            now -= 1
            continue
        c, s, h = t.admit(prompt, now)
        assert c == a[0] == cached_before and s.tolist() == a[1]
        if rng.random() < 0.7:
            t.release(h), orc.release(a[2])
    assert made_room >= 1


def test_eviction_plan_capacity_and_state_errors(pa):
    t = pa.Tree()
    with pytest.raises(pa.PrefixAttnError):
        t.evict_plan(1, 0)                       # no pool attached
    t.attach_pool(64, 1)
    now = 0
    for k in range(5):
        now += 1
        _, _, h = t.admit(np.array([k, 1, 2, 3], np.int32), now)
        t.release(h)
    toks, shr, nreq = t.evict_plan(8, 0)
    assert toks.tolist() == [4, 4] and shr.tolist() == [1, 1] and nreq == 5
    with pytest.raises(pa.PrefixAttnError) as e:
        t.evict_plan(8, 0, cap=1)
    assert e.value.code == -2
    assert t.evict_plan(8, 3)[1].tolist() == [0, 0] and t.evict_plan(8, 3)[2] == 2


def test_eviction_plan_joins_a_path_cut_between_the_same_requests(pa):
    t = pa.Tree()
    t.attach_pool(64, 1)
    for now, toks in [(1, [1, 2, 3, 4]), (2, [1, 2])]:   # the second prompt cuts the first one's node after 2 tokens
        t.release(t.admit(np.array(toks, np.int32), now)[2])
    toks, shr, nreq = t.evict_plan(4, 0)
    assert (toks.tolist(), shr.tolist(), nreq) == ([2, 2], [1, 2], 2)    # tail used by one request, head by both
    toks, shr, nreq = t.evict_plan(4, 2)
    assert (toks.tolist(), shr.tolist(), nreq) == ([4], [0], 0)          # nobody in the window: one run
    toks, shr, nreq = t.evict_plan(3, 2)
    assert toks.tolist() == [3]
