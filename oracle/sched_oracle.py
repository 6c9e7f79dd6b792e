"""Scheduling decisions of the paper, written out plainly.  TEST INFRASTRUCTURE ONLY: nothing in the
product may import this module; the tests compare the library's host functions with it.

What is here, and the passage each part follows:

* ``priority_group`` / ``priority_select``: Sec. 3.3, "waiting queue request ordering", and Algorithm 3.
  A request's group is the whole number of P-ths of its prompt that are cached (63 of 100 tokens, P = 10:
  group 6).  A batch takes requests from the groups in proportion to the group numbers (55 picks with every
  group full: 10 from group 10, 9 from group 9, ... 1 from group 1).
* ``load_cost``: Algorithm 2 (L + M + P) with the text of Sec. 3.2 for the three terms.
* ``e2_schedule``: Algorithm 1 (exploit if the missed part is shorter than the cached part, else explore:
  first the decode-ratio shortcut, then the lowest load cost).
* ``ClusterHistory``: the per-GPU request history over the window H that L and the decode ratio are
  computed from (Sec. 3.2, first cost).

Readings where the paper is silent (the same list is in the design document):

* Groups are numbered 0..P; group P holds only fully cached prompts.  Group p has weight p, so group 0 has
  weight 0: it is served only from capacity the other groups leave unused.
* "Proportionally": the picks are apportioned to the groups that have waiting requests by largest remainder
  (exact rational arithmetic; ties go to the higher group).  A group with fewer waiting requests than its
  share takes what it has; what is left over is apportioned again among the groups that still have requests
  ("round-robin with limits" in Algorithm 3), until the batch is full or only group 0 is left, which then
  fills the rest.  Inside a group requests leave in arrival order.  The batch lists higher groups first.
* PrefillTime(n) = prefill_per_token * n + prefill_base for n > 0 and 0 for n = 0; DecodeTime likewise.
  The coefficients come from profiling (not printed in the paper) and are parameters here.
* The average output length on a GPU with no finished request in the window is a parameter.
* DecodeRatio of a GPU = decode time / (prefill time + decode time) over its window (0 if the window is
  empty).  ImbalR is a parameter.
* Ties between GPUs (equal cost, equal ratio) go to the lowest GPU index.
* ``longest_piece``: Algorithm 1 sends an exploited request to the GPUs that cache the longest node of the matched
  path, which presupposes the global tree.  With one tree per GPU only the cached lengths are known: the path is cut
  where they differ and the longest piece stands for the longest node.
"""
from fractions import Fraction
from typing import List, Optional, Sequence, Tuple

EXPLOIT, EXPLORE_DECODE, EXPLORE_COST = 0, 1, 2


def priority_group(cached_len: int, prompt_len: int, P: int) -> int:
    if prompt_len <= 0 or cached_len <= 0:
        return 0
    return min(P, (P * min(cached_len, prompt_len)) // prompt_len)


def _apportion(total: int, weights: Sequence[int]) -> List[int]:
    """Largest-remainder apportionment of `total` to integer weights; ties go to the later index."""
    W = sum(weights)
    if W == 0 or total == 0:
        return [0] * len(weights)
    exact = [Fraction(total * w, W) for w in weights]
    out = [int(e) for e in exact]  # floor: all values are non-negative
    left = total - sum(out)
    order = sorted(range(len(weights)), key=lambda i: (exact[i] - out[i], i), reverse=True)
    for i in order[:left]:
        out[i] += 1
    return out


def priority_select(cached_len: Sequence[int], prompt_len: Sequence[int], P: int, n_pick: int) -> List[int]:
    """Indices (into the waiting queue, which is in arrival order) of the requests of the next batch."""
    groups: List[List[int]] = [[] for _ in range(P + 1)]
    for i, (c, n) in enumerate(zip(cached_len, prompt_len)):
        groups[priority_group(c, n, P)].append(i)
    taken = [0] * (P + 1)
    left = min(n_pick, len(cached_len))
    while left > 0:
        weights = [p if taken[p] < len(groups[p]) else 0 for p in range(P + 1)]
        if sum(weights) == 0:
            break
        share = _apportion(left, weights)
        for p in range(P + 1):
            k = min(share[p], len(groups[p]) - taken[p])
            taken[p] += k
            left -= k
    k0 = min(left, len(groups[0]) - taken[0])
    taken[0] += k0
    batch: List[int] = []
    for p in range(P, -1, -1):
        batch.extend(groups[p][:taken[p]])
    return batch


class CostModel:
    def __init__(self, prefill_per_token: float, prefill_base: float, decode_per_token: float, decode_base: float,
                 default_output_len: float):
        self.prefill_per_token = prefill_per_token
        self.prefill_base = prefill_base
        self.decode_per_token = decode_per_token
        self.decode_base = decode_base
        self.default_output_len = default_output_len

    def prefill_time(self, n: float) -> float:
        return self.prefill_per_token * n + self.prefill_base if n > 0 else 0.0

    def decode_time(self, n: float) -> float:
        return self.decode_per_token * n + self.decode_base if n > 0 else 0.0


def load_cost(model: CostModel, hist_missed_len: Sequence[int], avg_output_len: float, evict_tokens: Sequence[int],
              evict_sharers: Sequence[int], n_requests_in_window: int, missed_len_k: int) -> Tuple[float, float, float]:
    """(L, M, P) of Algorithm 2 for one GPU and one new request."""
    L = 0.0
    for m in hist_missed_len:
        L += model.prefill_time(m)
        L += model.decode_time(avg_output_len)
    M = 0.0
    for length, sharers in zip(evict_tokens, evict_sharers):
        N_j = sharers / n_requests_in_window if n_requests_in_window > 0 else 0.0
        M += model.prefill_time(length) * N_j
    P = model.prefill_time(missed_len_k)
    return L, M, P


def e2_schedule(prompt_len: int, cached_len: int, on_longest_node: Sequence[bool], cost: Sequence[float],
                decode_ratio: Sequence[float], imbal_r: float) -> Tuple[int, int]:
    """(gpu, mode) of Algorithm 1."""
    n = len(cost)
    missed_len = prompt_len - cached_len
    if missed_len < cached_len:
        K = [i for i in range(n) if on_longest_node[i]]
        if K:
            best = min(K, key=lambda i: (cost[i], i))
            return best, EXPLOIT
    top = max(range(n), key=lambda i: (decode_ratio[i], -i))
    if decode_ratio[top] > imbal_r:
        return top, EXPLORE_DECODE
    return min(range(n), key=lambda i: (cost[i], i)), EXPLORE_COST


def longest_piece(cached_len: Sequence[int]) -> List[bool]:
    """Which GPUs cache the longest node of the matched path, when only each GPU's cached length is known: the path
    is cut at every distinct cached length, the longest piece (the earliest among equals) is the node."""
    pieces, prev = [], 0
    for cut in sorted(set(c for c in cached_len if c > 0)):
        pieces.append((cut - prev, -cut))  # (length, minus its end): max() prefers longer, then earlier
        prev = cut
    if not pieces:
        return [False] * len(cached_len)
    end = -max(pieces)[1]
    return [c >= end for c in cached_len]


class ClusterHistory:
    """Requests assigned to each GPU and the output lengths seen on it, looked at through a window H."""

    def __init__(self, n_gpus: int, window: int, model: CostModel):
        self.window = window
        self.model = model
        self.assigned: List[List[Tuple[int, int]]] = [[] for _ in range(n_gpus)]  # (time, missed_len)
        self.finished: List[List[Tuple[int, int]]] = [[] for _ in range(n_gpus)]  # (time, output_len)

    def assign(self, gpu: int, now: int, missed_len: int) -> None:
        self.assigned[gpu].append((now, missed_len))

    def complete(self, gpu: int, now: int, output_len: int) -> None:
        self.finished[gpu].append((now, output_len))

    def gpu_load(self, gpu: int, now: int) -> Tuple[float, float, int, float]:
        """(L, decode ratio, requests in the window, average output length) of one GPU at time `now`."""
        lo = now - self.window
        outs = [o for (t, o) in self.finished[gpu] if lo < t <= now]
        avg = sum(outs) / len(outs) if outs else self.model.default_output_len
        missed = [m for (t, m) in self.assigned[gpu] if lo < t <= now]
        pt = sum(self.model.prefill_time(m) for m in missed)
        dt = sum(self.model.decode_time(avg) for _ in missed)
        ratio = dt / (pt + dt) if pt + dt > 0 else 0.0
        return pt + dt, ratio, len(missed), avg
