"""Shared set-up for the GPU parity tests: put a generated workload on the device through the
C-ABI (tree inserts + upload, pool filled only by pa_append_kv) and build the oracle's view of
the same workload.  The two sides meet only in the arrays of ``workloads``."""
from __future__ import annotations

import numpy as np
import torch

import oracle
from paper_2407_00023_amd import workloads as W


def to_torch(a: np.ndarray, dtype: str, device) -> torch.Tensor:
    if a.dtype == np.uint16:
        assert dtype == "bf16"
        return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(a).to(device)


def out_to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


class GpuSide:
    def __init__(self, wl: W.Workload, device, insert_cached=True):
        from paper_2407_00023_amd import binding as pa
        self.pa, self.wl, self.device = pa, wl, device
        self.tdtype = torch.float32 if wl.dtype == "f32" else torch.bfloat16
        self.tree = pa.Tree()
        if insert_cached:
            for i in range(wl.n_cached):
                self.tree.insert(*wl.cached_seq(i))
        self.tree.upload()
        nbytes = pa.kv_pool_bytes(wl.num_slots, wl.Hkv, wl.D, self.tdtype, wl.page_size)
        self.pool = torch.zeros(nbytes, dtype=torch.uint8, device=device)
        self.kw = dict(page_size=wl.page_size, num_slots=wl.num_slots)
        if len(wl.pool_slots):
            pa.append_kv(self.pool, torch.from_numpy(wl.pool_slots).to(device), to_torch(wl.pool_k, wl.dtype, device),
                         to_torch(wl.pool_v, wl.dtype, device), **self.kw)
        self.tokens = torch.from_numpy(wl.tokens).to(device)
        self.offsets = torch.from_numpy(wl.offsets).to(device)
        self.ext_len = torch.from_numpy(wl.ext_len).to(device)
        self.ext_offsets = torch.from_numpy(wl.ext_offsets).to(device)
        self.new_slots = torch.from_numpy(wl.new_slots).to(device)
        self.q = to_torch(wl.q_ext, wl.dtype, device)
        self.k = to_torch(wl.k_ext, wl.dtype, device)
        self.v = to_torch(wl.v_ext, wl.dtype, device)
        self.max_kv_len = int((wl.offsets[1:] - wl.offsets[:-1]).max()) if wl.B else 0

    def match(self):
        return self.pa.match_prefixes(self.tree, self.tokens, self.offsets)

    def extend(self, prefix_len, slot_idx, **over):
        kw = dict(self.kw, max_kv_len=self.max_kv_len)
        kw.update(over)
        return self.pa.extend_attention(self.q, self.k, self.v, self.pool, slot_idx, self.offsets, prefix_len,
                                        self.ext_len, self.ext_offsets, self.wl.scale, **kw)

    def append(self):
        self.pa.append_kv(self.pool, self.new_slots, self.k, self.v, **self.kw)

    def step(self):
        """One pass of the hot path: match -> extend attention -> append."""
        pl, si = self.match()
        out = self.extend(pl, si)
        self.append()
        return pl, si, out


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
