"""GPU test of pa_extend_attention_static, the entry point for callers that cannot allocate: its output against
pa_extend_attention's on the same inputs, on calls in a row that share the library's scratch buffer."""
import numpy as np
import pytest
import torch

from harness import GpuSide, OracleSide, out_to_f64
from paper_2407_00023_amd import workloads as W

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}


def _both(pa, g, wl):
    pl, si = g.match()
    nbytes = pa.extend_workspace_bytes(wl.B, wl.T, g.max_kv_len, wl.Hq, wl.Hkv, wl.D, g.tdtype)
    ws = torch.zeros(nbytes, dtype=torch.uint8, device=g.device)
    ref = g.extend(pl, si, workspace=ws)
    torch.cuda.synchronize()
    merged = ws[:16].view(torch.int32).tolist()[2] if wl.dtype == "bf16" else 0
    out = torch.full_like(ref, 3.0)
    before = torch.cuda.memory_allocated()
    pa.extend_attention_static(g.q, g.k, g.v, g.pool, si, g.offsets, pl, g.ext_len, g.ext_offsets, wl.scale,
                               max_kv_len=g.max_kv_len, out=out, **g.kw)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    return pl, si, ref, out, merged


def test_static_scratch_entry_point_matches_the_one_with_a_workspace(gpu_device):
    """Three calls in a row on one GPU, each smaller than the one before (the buffer keeps the earlier call's work list and
    partial results): the full tool-use configuration, a reduced long-document one whose key ranges are split into parts
    and merged, the tiny fp32 one.  Bar: bit for bit where pa_extend_attention split no row tile (the plans are then
    the same), within the dtype's tolerance otherwise (fewer parts: another order of summation) - and the reduced
    configurations against the oracle as well.  A batch whose plan exceeds the buffer is refused."""
    from paper_2407_00023_amd import binding as pa
    cases = [("tool_use", W.CONFIGS["tool_use"](), False), ("long_doc_qa", W.small_variant("long_doc_qa", 1), True),
             ("tiny_fp32", W.small_variant("tiny_fp32", 0), True)]
    sizes = [wl.T * wl.Hq * wl.D for _, wl, _ in cases]
    assert sizes[0] > sizes[1] > sizes[2]
    for name, wl, with_oracle in cases:
        print(f"[case] static scratch: {name}, T = {wl.T}", flush=True)
        g = GpuSide(wl, gpu_device)
        pl, si, ref, out, merged = _both(pa, g, wl)
        diff = float((out.double() - ref.double()).abs().max())
        same = torch.equal(out.view(torch.int16 if wl.dtype == "bf16" else torch.int32),
                           ref.view(torch.int16 if wl.dtype == "bf16" else torch.int32))
        print(f"  tiles merged from parts by pa_extend_attention: {merged}; max abs difference {diff:.3e}, bit-equal {same}", flush=True)
        assert diff <= TOL[wl.dtype]
        if merged == 0:
            assert same
        if with_oracle:
            o = OracleSide(wl)
            err = np.abs(out_to_f64(out) - o.extend(*o.match())).max()
            print(f"  against the oracle: max abs err {err:.3e}", flush=True)
            assert err <= TOL[wl.dtype]
        if name == "tool_use":
            # a batch far beyond the buffer (the host sizes alone decide): refused, nothing launched, out untouched
            mark = torch.full_like(ref, 5.0)
            rc = pa._lib.pa_extend_attention_static(pa._ptr(g.q), pa._ptr(g.k), pa._ptr(g.v), pa._ptr(g.pool), pa._ptr(si),
                                                    pa._ptr(g.offsets), pa._ptr(pl), pa._ptr(g.ext_len), pa._ptr(g.ext_offsets),
                                                    wl.B, 40_000_000, g.max_kv_len, wl.Hq, wl.Hkv, wl.D, wl.page_size,
                                                    wl.num_slots, pa.BF16, float(wl.scale), pa._ptr(mark), pa._stream(None))
            torch.cuda.synchronize()
            assert rc == -2 and b"bytes" in pa._lib.pa_last_error()
            assert bool((mark == 5.0).all())
