"""Shared set-up for the GPU parity tests: put a generated workload on the device through the
C-ABI (tree inserts + upload, pool filled only by pa_append_kv) and build the oracle's view of
the same workload.  The two sides meet only in the arrays of ``workloads``."""
from __future__ import annotations

import numpy as np
import torch

import oracle
from paper_2407_00023_amd import workloads as W
from paper_2407_00023_amd.resident import ResidentWorkload as GpuSide  # noqa: F401  (the device side of a workload)
from paper_2407_00023_amd.resident import to_torch  # noqa: F401


def out_to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


class OracleSide:
    def __init__(self, wl: W.Workload):
        self.wl = wl
        self.trie = oracle.Trie()
        for i in range(wl.n_cached):
            self.trie.insert(*wl.cached_seq(i))
        self.pool_k, self.pool_v = oracle.new_pool(wl.num_slots, wl.Hkv, wl.D, wl.dtype)
        oracle.append_kv(self.pool_k, self.pool_v, wl.pool_slots, wl.pool_k, wl.pool_v, wl.dtype)

    def match(self):
        return self.trie.match(self.wl.tokens, self.wl.offsets)

    def extend(self, prefix_len, slot_idx, rows=None):
        wl = self.wl
        return oracle.extend_attention(wl.q_ext, wl.k_ext, wl.v_ext, self.pool_k, self.pool_v, slot_idx, wl.offsets,
                                       prefix_len, wl.ext_len, wl.ext_offsets, wl.scale, wl.dtype, rows=rows)

    def append(self):
        wl = self.wl
        oracle.append_kv(self.pool_k, self.pool_v, wl.new_slots, wl.k_ext, wl.v_ext, wl.dtype)


def assert_match_equal(wl, pl_gpu, si_gpu, pl_ref, si_ref):
    """Bit-exact: prefix lengths, and slot ids on the matched span (entries past it are unspecified)."""
    pl_gpu, si_gpu = pl_gpu.cpu().numpy(), si_gpu.cpu().numpy()
    np.testing.assert_array_equal(pl_gpu, pl_ref)
    for r in range(wl.B):
        lo, P = int(wl.offsets[r]), int(pl_ref[r])
        np.testing.assert_array_equal(si_gpu[lo:lo + P], si_ref[lo:lo + P])


def sample_rows(wl, n, seed=0):
    """(r, i, h) triples: first/last extend row of the shortest and longest requests, plus random rows."""
    rng = np.random.default_rng(seed)
    rows = []
    for r in {int(np.argmin(wl.ext_len)), int(np.argmax(wl.ext_len)), 0, wl.B - 1}:
        for i in {0, int(wl.ext_len[r]) - 1, int(wl.ext_len[r]) // 2}:
            rows.append((r, i, int(rng.integers(0, wl.Hq))))
    while len(rows) < n:
        r = int(rng.integers(0, wl.B))
        rows.append((r, int(rng.integers(0, wl.ext_len[r])), int(rng.integers(0, wl.Hq))))
    return np.asarray(rows, np.int32)
