"""GPU parity of the fp8 form of the KV pool (dtype PA_BF16_KV8): what pa_append_kv stores, read back through
pa_gather_kv, equals the oracle's stored values bit for bit; extend attention over such a pool stays within the bf16
bar (max-abs 2e-2) of the fp64 oracle run over those stored values.
"""
import dataclasses

import numpy as np
import pytest
import torch

import oracle
from harness import GpuSide, OracleSide, assert_match_equal, out_to_f64, to_torch
from paper_2407_00023_amd import workloads as W

pytestmark = pytest.mark.gpu
TOL = 2e-2


def say(*a):
    print(*a, flush=True)


@pytest.fixture(scope="module")
def pa(gpu_device):
    from paper_2407_00023_amd import binding
    return binding


def _table():
    return np.array([(c & 7) * 2.0 ** -9 if c < 8 else (1 + (c & 7) / 8) * 2.0 ** ((c >> 3) - 7) for c in range(127)])


def _rows_that_cover_the_format(rng, D):
    """bfloat16 rows [n, D]: every code at several row exponents (the smallest and largest allowed among them), every
    midpoint between two codes, rows of zeros, rows spanning 14 binades below their largest element (so that codes
    below the normal range and values rounded to zero occur), random rows at many magnitudes."""
    t = _table()
    rows = []
    for k in (-100, -9, 0, 4, 119):
        r = np.zeros(D)
        n = min(D, 127)
        for first in range(0, 127, n - 1):          # (every code, 448 in each row so that its exponent is k)
            r[:] = 0
            part = t[first:first + n - 1]
            r[:len(part)] = part * (-1.0) ** np.arange(len(part))
            r[D - 1] = 448.0
            rows.append(W.f32_to_bf16_bits((r * 2.0 ** k).astype(np.float32)))
    mid = (t[:-1] + t[1:]) / 2
    for first in range(0, 126, D - 1):
        r = np.zeros(D)
        part = mid[first:first + D - 1]
        r[:len(part)] = part
        r[D - 1] = -448.0
        rows.append(W.f32_to_bf16_bits(r.astype(np.float32)))
    rows.append(np.zeros(D, np.uint16))
    rows.append(np.full(D, 0x8000, np.uint16))       # minus zero
    rows.append(np.array([0x7F7F, 0xFF7F] * (D // 2), np.uint16))   # the largest bfloat16
    for _ in range(300):
        e = int(rng.integers(20, 250))
        ex = rng.integers(max(1, e - 14), e + 1, D)
        bits = (rng.integers(0, 2, D) << 15) | (ex << 7) | rng.integers(0, 128, D)
        rows.append(bits.astype(np.uint16))
    x = rng.standard_normal((300, D)).astype(np.float32) * np.exp2(rng.integers(-40, 40, (300, 1))).astype(np.float32)
    rows.extend(W.f32_to_bf16_bits(x))
    return np.stack(rows)


@pytest.mark.parametrize("Hkv,D,page,nslots", [(2, 128, 16, 4096), (4, 64, 16, 2048), (2, 128, 12, 3072), (1, 64, 1, 2048)])
def test_fp8_rows_stored_bit_exact(pa, gpu_device, Hkv, D, page, nslots):
    """Bit-exact, both ways: the codes and row exponents the append kernel writes are the oracle's (or the stored
    values would differ), and the decode the attention kernel uses gives exactly code * 2^k."""
    say(f"[case] fp8 rows Hkv={Hkv} D={D} page={page}")
    rng = np.random.default_rng(3)
    rows = _rows_that_cover_the_format(rng, D)
    ntok = len(rows) // (2 * Hkv)                          # K takes the first half of the rows, V the second
    k = rows[:ntok * Hkv].reshape(ntok, Hkv, D)
    v = rows[ntok * Hkv:2 * ntok * Hkv].reshape(ntok, Hkv, D)
    assert ntok <= nslots
    slots = rng.permutation(nslots)[:ntok].astype(np.int32)
    pool = torch.zeros(pa.kv_pool_bytes(nslots, Hkv, D, torch.bfloat16, page, kv8=True), dtype=torch.uint8, device=gpu_device)
    assert pool.numel() == nslots * 2 * Hkv * (D + 1)
    kw = dict(page_size=page, num_slots=nslots, kv8=True)
    bad = np.concatenate([slots, np.array([nslots + 3, -1], np.int32)])       # slots outside the pool are skipped
    pa.append_kv(pool, torch.from_numpy(bad).to(gpu_device), to_torch(np.concatenate([k, k[:2]]), "bf16", gpu_device),
                 to_torch(np.concatenate([v, v[:2]]), "bf16", gpu_device), **kw)
    every = np.arange(nslots, dtype=np.int32)
    gk, gv = pa.gather_kv(pool, torch.from_numpy(every).to(gpu_device), Hkv=Hkv, D=D, dtype=torch.bfloat16, **kw)
    torch.cuda.synchronize()
    gk, gv = gk.view(torch.int16).cpu().numpy().view(np.uint16), gv.view(torch.int16).cpu().numpy().view(np.uint16)
    want_k, want_v = np.zeros((nslots, Hkv, D), np.uint16), np.zeros((nslots, Hkv, D), np.uint16)
    want_k[slots], want_v[slots] = oracle.fp8_rows(k)[2], oracle.fp8_rows(v)[2]
    np.testing.assert_array_equal(gk, want_k)
    np.testing.assert_array_equal(gv, want_v)
    # the same through the oracle's own append: its pool holds the stored values
    opk, opv = oracle.new_pool(nslots, Hkv, D, "bf16_kv8")
    oracle.append_kv(opk, opv, slots, k, v, "bf16_kv8")
    np.testing.assert_array_equal(gk, opk)


SMALL = ["tool_use", "long_doc_qa", "agent_tree", "video_qa", "programming", "tool_use_zipf", "decode"]


@pytest.mark.parametrize("name", SMALL)
@pytest.mark.parametrize("seed", [0, 1])
def test_fp8_pool_small_config_whole_path(pa, gpu_device, name, seed):
    """match -> extend -> append with the pool in its fp8 form, every output element against the oracle; the appended
    rows read back as the oracle's stored values."""
    say(f"[case] fp8 small {name} seed={seed}")
    wl = dataclasses.replace(W.small_variant(name, seed), dtype="bf16_kv8")
    g, o = GpuSide(wl, gpu_device), OracleSide(wl)
    pl, si, out = g.step()
    torch.cuda.synchronize()
    pl_ref, si_ref = o.match()
    assert_match_equal(wl, pl, si, pl_ref, si_ref)
    ref = o.extend(pl_ref, si_ref)
    err = np.abs(out_to_f64(out) - ref).max()
    say(f"  max abs err {err:.3e}")
    assert err <= TOL
    o.append()
    allslots = np.concatenate([wl.pool_slots, wl.new_slots])
    gk, gv = pa.gather_kv(g.pool, torch.from_numpy(allslots).to(gpu_device), Hkv=wl.Hkv, D=wl.D, dtype=g.tdtype, **g.kw)
    np.testing.assert_array_equal(gk.view(torch.int16).cpu().numpy(), o.pool_k[allslots].view(np.int16))
    np.testing.assert_array_equal(gv.view(torch.int16).cpu().numpy(), o.pool_v[allslots].view(np.int16))


@pytest.mark.parametrize("Hq,Hkv,D,page,p_hi,e_hi,B", [
    (8, 2, 128, 16, 700, 90, 6),      # several key tiles, ragged tails
    (4, 4, 64, 16, 300, 200, 4),      # D = 64
    (16, 2, 128, 1, 200, 33, 4),      # page size 1
    (8, 8, 128, 16, 5000, 10, 3),     # long prefix, short extend: split key ranges
    (8, 2, 128, 12, 700, 90, 6),      # a page size that is no power of two
    (4, 2, 64, 24, 400, 150, 4),
])
def test_fp8_pool_extend_random_shapes(pa, gpu_device, Hq, Hkv, D, page, p_hi, e_hi, B):
    """Ragged prefixes and extends including prefix_len = 0 and ext_len = 0; row magnitudes vary by powers of two from
    token to token, so that row exponents differ inside every tile."""
    from test_gpu_parity import _random_case
    say(f"[case] fp8 extend_random Hq={Hq} Hkv={Hkv} D={D} page={page} p_hi={p_hi} e_hi={e_hi}")
    rng = np.random.default_rng(12)
    nslots = 16384 if 16384 % page == 0 else 18432
    c = _random_case(rng, B, Hq, Hkv, D, p_hi, e_hi, "bf16", page, nslots)
    # K rows scaled by 2^-3..2^1 per (token, head) (exact in bfloat16); V rows by 2^-8..2^0 (not up: the bar is an
    # absolute one, set for values of magnitude one)
    def rescale(a, lo, hi):
        f = np.exp2(rng.integers(lo, hi + 1, a.shape[:2] + (1,))).astype(np.float32)
        return W.f32_to_bf16_bits(W.bf16_bits_to_f32(a) * f)
    c["pk"], c["pv"] = rescale(c["pk"], -3, 1), rescale(c["pv"], -8, 0)
    dev = gpu_device
    pool = torch.zeros(pa.kv_pool_bytes(nslots, Hkv, D, torch.bfloat16, page, kv8=True), dtype=torch.uint8, device=dev)
    kw = dict(page_size=page, num_slots=nslots, kv8=True)
    pa.append_kv(pool, torch.from_numpy(c["backed"]).to(dev), to_torch(c["pk"], "bf16", dev), to_torch(c["pv"], "bf16", dev), **kw)
    tt = lambda a: torch.from_numpy(a).to(dev)
    scale = 1.0 / np.sqrt(D)
    out = pa.extend_attention(to_torch(c["q"], "bf16", dev), to_torch(c["k"], "bf16", dev), to_torch(c["v"], "bf16", dev), pool,
                              tt(c["si"]), tt(c["off"]), tt(c["P"]), tt(c["E"]), tt(c["eo"]), scale,
                              max_kv_len=int((c["P"] + c["E"]).max()), **kw)
    torch.cuda.synchronize()
    opk, opv = oracle.new_pool(nslots, Hkv, D, "bf16_kv8")
    oracle.append_kv(opk, opv, c["backed"], c["pk"], c["pv"], "bf16_kv8")
    ref = oracle.extend_attention(c["q"], c["k"], c["v"], opk, opv, c["si"], c["off"], c["P"], c["E"], c["eo"], scale, "bf16_kv8")
    err = np.abs(out_to_f64(out) - ref).max() if c["T"] else 0.0
    # (and the quantisation itself is visible: against the unquantised pool the same output is off by more)
    upk, upv = oracle.new_pool(nslots, Hkv, D, "bf16")
    oracle.append_kv(upk, upv, c["backed"], c["pk"], c["pv"], "bf16")
    ref_unq = oracle.extend_attention(c["q"], c["k"], c["v"], upk, upv, c["si"], c["off"], c["P"], c["E"], c["eo"], scale, "bf16")
    say(f"  max abs err {err:.3e}   (fp8 storage itself moves the fp64 result by {np.abs(ref - ref_unq).max():.3e})")
    assert err <= TOL


def test_fp8_pool_static_entry_point_agrees(pa, gpu_device):
    """The entry point that allocates nothing takes the fp8 pool too."""
    wl = dataclasses.replace(W.small_variant("long_doc_qa", 0), dtype="bf16_kv8")
    g = GpuSide(wl, gpu_device)
    pl, si = g.match()
    out = g.extend(pl, si)
    out2 = torch.empty_like(out)
    pa.extend_attention_static(g.q, g.k, g.v, g.pool, si, g.offsets, pl, g.ext_len, g.ext_offsets, wl.scale,
                               max_kv_len=g.max_kv_len, out=out2, **g.kw)
    torch.cuda.synchronize()
    assert float((out.float() - out2.float()).abs().max()) <= TOL


@pytest.mark.parametrize("name", ["tool_use", "long_doc_qa"])
def test_fp8_pool_full_config_extend_every_element(pa, gpu_device, name):
    """Full sizes, in the launch configuration the benchmark times, every output element against the oracle."""
    say(f"[case] fp8 full extend {name}")
    wl = dataclasses.replace(W.CONFIGS[name](), dtype="bf16_kv8")
    g, o = GpuSide(wl, gpu_device), OracleSide(wl)
    pl, si = g.match()
    ws = torch.zeros(pa.extend_workspace_bytes(wl.B, wl.T, g.max_kv_len, wl.Hq, wl.Hkv, wl.D, g.tdtype), dtype=torch.uint8, device=gpu_device)
    out = g.extend(pl, si, workspace=ws)
    torch.cuda.synchronize()
    pa.extend_status(ws)
    pl_ref, si_ref = o.match()
    assert_match_equal(wl, pl, si, pl_ref, si_ref)
    err = np.abs(out_to_f64(out) - o.extend(pl_ref, si_ref)).max()
    say(f"  all {wl.T * wl.Hq} rows: max abs err {err:.3e}")
    assert err <= TOL


def test_fp8_pool_beyond_4_gib(pa, gpu_device):
    """Codes of 4.8 GB: rows on both sides of the 4 GiB line.  The runs of assembly tiles address the codes by 32-bit
    offsets and stand back here; the other tiles, append and gather compute in 64 bits.  Every element, and the stored
    rows bit-exact."""
    say("[case] fp8 pool beyond 4 GiB")
    wl = dataclasses.replace(W.tool_use(22, B=8, sys_len=1300, n_tools=3, tool_lo=100, tool_hi=500, ext_lo=20, ext_hi=160,
                                        num_slots=2_359_296), dtype="bf16_kv8")
    page_off = (wl.pool_slots.astype(np.int64) // wl.page_size) * wl.page_size * 2 * wl.Hkv * wl.D
    assert (page_off < 2 ** 32).sum() > 100 and (page_off >= 2 ** 32).sum() > 100
    g, o = GpuSide(wl, gpu_device), OracleSide(wl)
    pl, si, out = g.step()
    torch.cuda.synchronize()
    pl_ref, si_ref = o.match()
    assert_match_equal(wl, pl, si, pl_ref, si_ref)
    err = np.abs(out_to_f64(out) - o.extend(pl_ref, si_ref)).max()
    say(f"  max abs err {err:.3e}")
    assert err <= TOL
    o.append()
    allslots = np.concatenate([wl.pool_slots, wl.new_slots])
    gk, gv = pa.gather_kv(g.pool, torch.from_numpy(allslots).to(gpu_device), Hkv=wl.Hkv, D=wl.D, dtype=g.tdtype, **g.kw)
    np.testing.assert_array_equal(gk.view(torch.int16).cpu().numpy(), o.pool_k[allslots].view(np.int16))
    np.testing.assert_array_equal(gv.view(torch.int16).cpu().numpy(), o.pool_v[allslots].view(np.int16))
    del g
    torch.cuda.empty_cache()
