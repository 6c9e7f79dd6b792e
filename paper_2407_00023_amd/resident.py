"""A generated workload made resident on the GPU through the library's own calls: the radix tree filled by
pa_tree_insert and uploaded, the KV pool filled only by pa_append_kv, every tensor of the step in device memory.
Argument marshalling and set-up only; used by the benchmark, the smoke check and the GPU tests."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as pa
from . import workloads as W


def to_torch(a: np.ndarray, dtype: str, device) -> torch.Tensor:
    """Host array of the generators (bf16 as uint16 bit patterns) -> device tensor of the same bits."""
    if a.dtype == np.uint16:
        assert dtype in ("bf16", "bf16_kv8")
        return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(a).to(device)


class ResidentWorkload:
    def __init__(self, wl: W.Workload, device, insert_cached: bool = True):
        self.pa, self.wl, self.device = pa, wl, device
        self.tdtype = torch.float32 if wl.dtype == "f32" else torch.bfloat16
        self.tree = pa.Tree()
        if insert_cached:
            for i in range(wl.n_cached):
                self.tree.insert(*wl.cached_seq(i))
        self.tree.upload()
        self.kv8 = wl.dtype == "bf16_kv8"   # bf16 tensors, the KV pool in its fp8 form
        nbytes = pa.kv_pool_bytes(wl.num_slots, wl.Hkv, wl.D, self.tdtype, wl.page_size, self.kv8)
        self.pool = torch.zeros(nbytes, dtype=torch.uint8, device=device)
        self.kw = dict(page_size=wl.page_size, num_slots=wl.num_slots, kv8=self.kv8)
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
        return pa.match_prefixes(self.tree, self.tokens, self.offsets)

    def extend(self, prefix_len, slot_idx, **over):
        kw = dict(self.kw, max_kv_len=self.max_kv_len)
        kw.update(over)
        return pa.extend_attention(self.q, self.k, self.v, self.pool, slot_idx, self.offsets, prefix_len,
                                   self.ext_len, self.ext_offsets, self.wl.scale, **kw)

    def append(self):
        pa.append_kv(self.pool, self.new_slots, self.k, self.v, **self.kw)

    def step(self):
        """One pass of the hot path: match -> extend attention -> append."""
        pl, si = self.match()
        out = self.extend(pl, si)
        self.append()
        return pl, si, out
