"""Pins for the oracle's extend attention and append_kv (CPU only).

Each test fixes the oracle against something that is not the oracle: a library routine
(torch scaled_dot_product_attention with a causal mask), the losslessness of prefix reuse
(Sec. 5 contrasts lossless prefix sharing with lossy non-prefix sharing; Sec. 3.2 prices a
request by its missed tokens only): a prompt split into cached prefix + extend must give
the rows of plain causal attention over the whole prompt; and closed forms of softmax.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2407_00023_amd import workloads as W


def rand_case(rng, B, Hq, Hkv, D, lens_prefix, lens_ext, num_slots, dtype="f32"):
    """Random pool + requests with shuffled prefix slots (no sharing)."""
    perm = rng.permutation(num_slots).astype(np.int32)
    so = np.zeros(B + 1, np.int32)
    eo = np.zeros(B + 1, np.int32)
    so[1:] = np.cumsum(np.asarray(lens_prefix) + np.asarray(lens_ext))
    eo[1:] = np.cumsum(lens_ext)
    si = np.full(so[-1], -1, np.int32)
    cur = 0
    for r in range(B):
        si[so[r]:so[r] + lens_prefix[r]] = perm[cur:cur + lens_prefix[r]]
        cur += lens_prefix[r]
    T = int(eo[-1])

    def draw(*shape):
        x = rng.standard_normal(shape).astype(np.float32)
        return x if dtype == "f32" else W.f32_to_bf16_bits(x)

    pk, pv = draw(num_slots, Hkv, D), draw(num_slots, Hkv, D)
    return dict(q=draw(T, Hq, D), k=draw(T, Hkv, D), v=draw(T, Hkv, D), pk=pk, pv=pv, si=si, so=so,
                pl=np.asarray(lens_prefix, np.int32), el=np.asarray(lens_ext, np.int32), eo=eo)


def run(c, scale, dtype="f32", rows=None):
    return oracle.extend_attention(c["q"], c["k"], c["v"], c["pk"], c["pv"], c["si"], c["so"], c["pl"], c["el"],
                                   c["eo"], scale, dtype, rows=rows)


def as_f64(a, dtype):
    return (a if dtype == "f32" else W.bf16_bits_to_f32(a)).astype(np.float64)


@pytest.mark.parametrize("Hq,Hkv,D,dtype", [(4, 2, 64, "f32"), (8, 2, 32, "bf16"), (6, 6, 16, "f32"), (4, 1, 8, "f32")])
def test_no_prefix_equals_library_causal_attention(Hq, Hkv, D, dtype):
    """prefix_len = 0: textbook causal GQA attention (workloads without sharing behave as usual)."""
    rng = np.random.default_rng(1)
    ext = [17, 1, 40]
    c = rand_case(rng, 3, Hq, Hkv, D, [0, 0, 0], ext, 8, dtype)
    scale = 0.37
    out = run(c, scale, dtype)
    G = Hq // Hkv
    for r, E in enumerate(ext):
        lo = c["eo"][r]
        q = torch.from_numpy(as_f64(c["q"][lo:lo + E], dtype)).permute(1, 0, 2)          # [Hq, E, D]
        k = torch.from_numpy(as_f64(c["k"][lo:lo + E], dtype)).permute(1, 0, 2).repeat_interleave(G, dim=0)
        v = torch.from_numpy(as_f64(c["v"][lo:lo + E], dtype)).permute(1, 0, 2).repeat_interleave(G, dim=0)
        ref = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True, scale=scale)
        np.testing.assert_allclose(out[lo:lo + E], ref.permute(1, 0, 2).numpy(), rtol=0, atol=1e-12)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_split_invariance(dtype):
    """Cached prefix (through shuffled slots) + extend == rows of causal attention over the whole prompt."""
    rng = np.random.default_rng(2)
    Hq, Hkv, D, N = 4, 2, 32, 37
    full = rand_case(rng, 1, Hq, Hkv, D, [0], [N], 64, dtype)
    ref = run(full, 0.2, dtype)                                    # [N, Hq, D], no prefix at all
    for cut in [1, 5, 18, 36]:
        slots = rng.permutation(64)[:cut].astype(np.int32)
        pk, pv = oracle.new_pool(64, Hkv, D, dtype)
        oracle.append_kv(pk, pv, slots, full["k"][:cut], full["v"][:cut], dtype)
        E = N - cut
        c = dict(q=full["q"][cut:], k=full["k"][cut:], v=full["v"][cut:], pk=pk, pv=pv,
                 si=np.concatenate([slots, np.full(E, -1, np.int32)]), so=np.array([0, N], np.int32),
                 pl=np.array([cut], np.int32), el=np.array([E], np.int32), eo=np.array([0, E], np.int32))
        np.testing.assert_allclose(run(c, 0.2, dtype), ref[cut:], rtol=0, atol=1e-13)


def test_closed_forms():
    rng = np.random.default_rng(3)
    Hq, Hkv, D = 4, 2, 16
    c = rand_case(rng, 2, Hq, Hkv, D, [9, 3], [4, 6], 32)
    # all V rows equal (per kv head): output is that row, whatever the scores
    c1 = dict(c)
    row = rng.standard_normal((Hkv, D)).astype(np.float32)
    c1["pv"] = np.broadcast_to(row, c["pv"].shape).copy()
    c1["v"] = np.broadcast_to(row, c["v"].shape).copy()
    out = run(c1, 1.0)
    want = np.repeat(row.astype(np.float64), Hq // Hkv, axis=0)
    np.testing.assert_allclose(out, np.broadcast_to(want, out.shape), atol=1e-14)
    # q = 0: uniform weights -> arithmetic mean of the visible V rows
    c2 = dict(c)
    c2["q"] = np.zeros_like(c["q"])
    out = run(c2, 1.0)
    for r in range(2):
        P, E = int(c["pl"][r]), int(c["el"][r])
        pref = c["pv"][c["si"][c["so"][r]:c["so"][r] + P]].astype(np.float64)
        for i in range(E):
            vis = np.concatenate([pref, c["v"][c["eo"][r]:c["eo"][r] + i + 1].astype(np.float64)])  # [n, Hkv, D]
            for h in range(Hq):
                np.testing.assert_allclose(out[c["eo"][r] + i, h], vis[:, h // (Hq // Hkv)].mean(0), atol=1e-14)
    # one key with an overwhelming score: output -> its V row
    c3 = dict(c)
    c3["pk"] = c["pk"].copy()
    c3["q"] = np.ones_like(c["q"])
    c3["pk"][:] = 0
    c3["k"] = np.zeros_like(c["k"])
    hot = int(c["si"][c["so"][0] + 4])
    c3["pk"][hot] = 50.0
    out = run(c3, 1.0)
    for h in range(Hq):
        np.testing.assert_allclose(out[0, h], c["pv"][hot, h // (Hq // Hkv)].astype(np.float64), atol=1e-12)


def test_scale_and_head_mapping_by_hand():
    """Two keys, D = 2, numbers small enough to evaluate on paper."""
    q = np.zeros((1, 2, 2), np.float32)
    q[0, 0] = [1, 0]
    q[0, 1] = [0, 2]                        # Hq = 2, Hkv = 1: both heads read kv head 0
    k = np.array([[[0.0, 1.0]]], np.float32)  # the extend token itself
    v = np.array([[[10.0, 20.0]]], np.float32)
    pk = np.zeros((4, 1, 2), np.float32)
    pv = np.zeros((4, 1, 2), np.float32)
    pk[3, 0] = [2.0, 0.0]
    pv[3, 0] = [1.0, -1.0]
    out = oracle.extend_attention(q, k, v, pk, pv, np.array([3, -1], np.int32), np.array([0, 2], np.int32),
                                  np.array([1], np.int32), np.array([1], np.int32), np.array([0, 1], np.int32), 0.5, "f32")
    # head 0: scores 0.5*[2, 0] = [1, 0] -> weights e/(e+1), 1/(e+1)
    w = np.e / (np.e + 1)
    np.testing.assert_allclose(out[0, 0], w * np.array([1, -1]) + (1 - w) * np.array([10, 20]), atol=1e-14)
    # head 1: scores 0.5*[0, 2] = [0, 1] -> weights 1/(e+1), e/(e+1)
    np.testing.assert_allclose(out[0, 1], (1 - w) * np.array([1, -1]) + w * np.array([10, 20]), atol=1e-14)


def test_slot_permutation_and_batch_invariance_and_rows():
    rng = np.random.default_rng(4)
    Hq, Hkv, D = 4, 2, 16
    c = rand_case(rng, 3, Hq, Hkv, D, [7, 0, 12], [5, 3, 1], 40)
    ref = run(c, 0.3)
    # re-shuffle the pool and remap slot ids: same output
    perm = rng.permutation(40).astype(np.int32)
    c2 = dict(c)
    c2["pk"], c2["pv"] = np.empty_like(c["pk"]), np.empty_like(c["pv"])
    c2["pk"][perm], c2["pv"][perm] = c["pk"], c["pv"]
    c2["si"] = np.where(c["si"] >= 0, perm[np.maximum(c["si"], 0)], -1).astype(np.int32)
    np.testing.assert_array_equal(run(c2, 0.3), ref)
    # request 2 alone == request 2 inside the batch
    lo, hi = c["so"][2], c["so"][3]
    e0 = c["eo"][2]
    solo = dict(q=c["q"][e0:], k=c["k"][e0:], v=c["v"][e0:], pk=c["pk"], pv=c["pv"], si=c["si"][lo:hi],
                so=np.array([0, hi - lo], np.int32), pl=c["pl"][2:], el=c["el"][2:], eo=np.array([0, 1], np.int32))
    np.testing.assert_array_equal(run(solo, 0.3), ref[e0:])
    # the row-sampling entry point returns the same numbers
    rows = np.array([[0, 4, 3], [1, 0, 0], [2, 0, 1], [0, 0, 2]], np.int32)
    got = run(c, 0.3, rows=rows)
    for x, (r, i, h) in enumerate(rows):
        np.testing.assert_array_equal(got[x], ref[c["eo"][r] + i, h])


def test_append_kv_round_trip():
    rng = np.random.default_rng(5)
    for dtype in ["f32", "bf16"]:
        pk, pv = oracle.new_pool(50, 2, 8, dtype)
        pk[:] = 7
        pv[:] = 9
        before_k = pk.copy()
        slots = rng.permutation(50)[:11].astype(np.int32)
        k = rng.integers(0, 60000, (11, 2, 8)).astype(pk.dtype)
        v = rng.integers(0, 60000, (11, 2, 8)).astype(pk.dtype)
        oracle.append_kv(pk, pv, slots, k, v, dtype)
        np.testing.assert_array_equal(pk[slots], k)
        np.testing.assert_array_equal(pv[slots], v)
        rest = np.setdiff1d(np.arange(50), slots)
        np.testing.assert_array_equal(pk[rest], before_k[rest])
        assert (pv[rest] == 9).all()


def test_bf16_values_are_widened_exactly():
    # 0x3FC0 = 1.5, 0xC000 = -2.0, 0x3F80 = 1.0
    assert list(W.bf16_bits_to_f32(np.array([0x3FC0, 0xC000, 0x3F80], np.uint16))) == [1.5, -2.0, 1.0]
    q = np.array([[[0x3F80]]], np.uint16)
    k = np.array([[[0x3F80]]], np.uint16)
    v = np.array([[[0x3FC0]]], np.uint16)
    pk = np.array([[[0x3F80]]], np.uint16)
    pv = np.array([[[0xC000]]], np.uint16)
    out = oracle.extend_attention(q, k, v, pk, pv, np.array([0, -1], np.int32), np.array([0, 2], np.int32),
                                  np.array([1], np.int32), np.array([1], np.int32), np.array([0, 1], np.int32), 1.0, "bf16")
    assert out[0, 0, 0] == pytest.approx(0.5 * 1.5 + 0.5 * -2.0, abs=1e-15)   # equal scores: plain average
    # round-to-nearest-even of the generator's fp32 -> bf16
    x = np.array([1.0, 1.00390625, 1.01171875, -3.0e38], np.float32)  # 1+2^-8 (tie -> even), 1+3*2^-8 (tie -> even up)
    assert list(W.f32_to_bf16_bits(x)[:3]) == [0x3F80, 0x3F80, 0x3F82]


def test_small_workload_split_invariance_through_generator():
    """On a generated workload: request = designed prefix + extend; recompute as one causal pass over
    the whole prompt's K/V (prefix rows read straight from the generator's pool arrays)."""
    wl = W.small_variant("tool_use", seed=1)
    pk, pv = oracle.new_pool(wl.num_slots, wl.Hkv, wl.D, wl.dtype)
    oracle.append_kv(pk, pv, wl.pool_slots, wl.pool_k, wl.pool_v, wl.dtype)
    out = oracle.extend_attention(wl.q_ext, wl.k_ext, wl.v_ext, pk, pv, wl.designed_slots, wl.offsets,
                                  wl.designed_prefix_len, wl.ext_len, wl.ext_offsets, wl.scale, wl.dtype)
    where = {int(s): i for i, s in enumerate(wl.pool_slots)}
    G = wl.Hq // wl.Hkv
    for r in [0, wl.B - 1]:
        P, E = int(wl.designed_prefix_len[r]), int(wl.ext_len[r])
        lo, e0 = int(wl.offsets[r]), int(wl.ext_offsets[r])
        idx = [where[int(s)] for s in wl.designed_slots[lo:lo + P]]
        K = np.concatenate([as_f64(wl.pool_k[idx], "bf16"), as_f64(wl.k_ext[e0:e0 + E], "bf16")])  # [N, Hkv, D]
        V = np.concatenate([as_f64(wl.pool_v[idx], "bf16"), as_f64(wl.v_ext[e0:e0 + E], "bf16")])
        Q = as_f64(wl.q_ext[e0:e0 + E], "bf16")
        k = torch.from_numpy(K).permute(1, 0, 2).repeat_interleave(G, dim=0)
        v = torch.from_numpy(V).permute(1, 0, 2).repeat_interleave(G, dim=0)
        q = torch.from_numpy(Q).permute(1, 0, 2)
        mask = torch.ones(E, P + E, dtype=torch.bool).tril(diagonal=P)
        ref = torch.nn.functional.scaled_dot_product_attention(q, k, v, attn_mask=mask, scale=wl.scale)
        np.testing.assert_allclose(out[e0:e0 + E], ref.permute(1, 0, 2).numpy(), atol=1e-12)
