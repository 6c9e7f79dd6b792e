"""GPU parity: the HIP path, called through the C-ABI binding, against the CPU oracle on the
same seeded inputs.

Bars (written out in each test): prefix lengths and slot indices bit-exact; KV round trips
bit-exact; extend attention within max-abs 1e-4 (fp32) and 2e-2 (bf16 in/out) of the fp64
oracle, whose output is not rounded.
"""
import os

import numpy as np
import pytest
import torch

from harness import GpuSide, OracleSide, assert_match_equal, out_to_f64, sample_rows, to_torch
from paper_2407_00023_amd import workloads as W

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "radix_hand_example.txt")
SMALL = ["tiny_fp32", "tool_use", "long_doc_qa", "agent_tree", "video_qa", "programming", "tool_use_zipf", "decode"]
FULL = ["tool_use", "long_doc_qa", "agent_tree", "video_qa", "programming", "tool_use_zipf", "decode"]


def say(*a):
    print(*a, flush=True)


@pytest.fixture(scope="module")
def pa(gpu_device):
    from paper_2407_00023_amd import binding
    return binding


# ------------------------------------------------------------------------------------ matcher

def test_match_hand_worked_example(pa, gpu_device):
    """The hand-derived radix example of tests/golden (Sec. 3.2 insert/split rules, Algorithm 1 cached_len)."""
    tree, queries = pa.Tree(), []
    for line in open(GOLDEN):
        line = line.strip()
        if line.startswith("insert"):
            pairs = [x.split(":") for x in line.split()[1:]]
            tree.insert(np.array([int(a) for a, _ in pairs], np.int32), np.array([int(b) for _, b in pairs], np.int32))
        elif line.startswith("query"):
            a, b, c = line[len("query"):].split("|")
            queries.append(([int(x) for x in a.split()], int(b), [int(x) for x in c.split()]))
    tree.upload()
    toks = np.concatenate([np.asarray(q[0], np.int32) for q in queries])
    off = np.zeros(len(queries) + 1, np.int32)
    off[1:] = np.cumsum([len(q[0]) for q in queries])
    pl, si = pa.match_prefixes(tree, torch.from_numpy(toks).to(gpu_device), torch.from_numpy(off).to(gpu_device))
    pl, si = pl.cpu().numpy(), si.cpu().numpy()
    for r, (_, want_len, want_slots) in enumerate(queries):
        assert pl[r] == want_len, r
        assert list(si[off[r]:off[r] + want_len]) == want_slots, r


@pytest.mark.parametrize("vocab,seed", [(2, 0), (3, 1), (4, 2), (1000, 3)])
def test_match_random_small_vocab(pa, gpu_device, vocab, seed):
    """Tiny vocabularies force many splits, mid-edge stops and full matches; bit-exact vs the oracle trie."""
    import oracle
    rng = np.random.default_rng(seed)
    cached, nslot = [], 0
    for _ in range(150):
        n = int(rng.integers(0, 40 if vocab < 10 else 3000))
        cached.append((rng.integers(0, vocab, n).astype(np.int32), np.arange(nslot, nslot + n, dtype=np.int32)))
        nslot += n
    prompts = []
    for _ in range(97):
        if rng.random() < 0.5 and cached:
            base = cached[int(rng.integers(0, len(cached)))][0]
            cut = int(rng.integers(0, len(base) + 1))
            tail = rng.integers(0, vocab, int(rng.integers(0, 20))).astype(np.int32)
            prompts.append(np.concatenate([base[:cut], tail]))
        else:
            prompts.append(rng.integers(0, vocab, int(rng.integers(0, 30))).astype(np.int32))
    toks = np.concatenate(prompts).astype(np.int32)
    off = np.zeros(len(prompts) + 1, np.int32)
    off[1:] = np.cumsum([len(p) for p in prompts])
    pl_ref, si_ref = oracle.match_prefixes(cached, toks, off)
    tree = pa.Tree()
    for c in cached:
        tree.insert(*c)
    tree.upload()
    pl, si = pa.match_prefixes(tree, torch.from_numpy(toks).to(gpu_device), torch.from_numpy(off).to(gpu_device))
    pl, si = pl.cpu().numpy(), si.cpu().numpy()
    np.testing.assert_array_equal(pl, pl_ref)
    for r in range(len(prompts)):
        np.testing.assert_array_equal(si[off[r]:off[r] + pl_ref[r]], si_ref[off[r]:off[r] + pl_ref[r]])


@pytest.mark.parametrize("copies,trunk_len", [(1, 9000), (2, 9000), (5, 9000), (1, 40000)])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_match_long_paths_of_mixed_edge_lengths(pa, gpu_device, seed, copies, trunk_len):
    """A trunk with branch points at spacings from 1 to thousands of tokens: the prompt's path runs through
    hundreds of nodes whose edges are short, medium and very long in turn, stops at node boundaries, inside
    edges of every class, at the trunk's end and inside side branches; bit-exact vs the oracle trie.
    copies = 1: 64 prompts, several workgroups per prompt (a trunk of 40,000 tokens reaches past the windows that get a
    workgroup of their own); 2: 128 prompts, one workgroup each; 5: 320 prompts, shorter windows."""
    import oracle
    rng = np.random.default_rng(100 + seed)
    vocab = 50000
    spacing = []
    while sum(spacing) < trunk_len:
        kind = rng.integers(0, 4)
        lo, hi = [(1, 9), (20, 200), (260, 1000), (1100, 3000)][kind]
        run = int(rng.integers(20, 150)) if kind == 0 else 1
        spacing += [int(rng.integers(lo, hi)) for _ in range(run)]
    trunk = rng.integers(0, vocab, sum(spacing) + 50).astype(np.int32)
    cuts = np.cumsum(spacing)
    cached, nslot = [], 0

    def add(seq):
        nonlocal nslot
        cached.append((seq.astype(np.int32), np.arange(nslot, nslot + len(seq), dtype=np.int32)))
        nslot += len(seq)

    add(trunk)
    for c in cuts:
        branch = rng.integers(0, vocab, int(rng.integers(1, 600))).astype(np.int32)
        branch[0] = (trunk[c] + 1) % vocab  # leaves the trunk exactly at c
        add(np.concatenate([trunk[:c], branch]))
    prompts = [trunk.copy(), trunk[:1], trunk[: cuts[0]], np.concatenate([trunk, rng.integers(0, vocab, 7).astype(np.int32)])]
    for _ in range(60):
        which = int(rng.integers(0, len(cached)))
        base = cached[which][0]
        mode = rng.integers(0, 3)
        cut = int(cuts[rng.integers(0, len(cuts))]) if mode == 0 else int(rng.integers(0, len(base) + 1))
        cut = min(cut, len(base))
        tail = rng.integers(0, vocab, int(rng.integers(0, 30))).astype(np.int32)
        prompts.append(np.concatenate([base[:cut], tail]))
    prompts = prompts * copies
    toks = np.concatenate(prompts).astype(np.int32)
    off = np.zeros(len(prompts) + 1, np.int32)
    off[1:] = np.cumsum([len(p) for p in prompts])
    pl_ref, si_ref = oracle.match_prefixes(cached, toks, off)
    assert pl_ref.max() >= len(trunk) and len(cuts) > 100
    tree = pa.Tree()
    for c in cached:
        tree.insert(*c)
    tree.upload()
    pl, si = pa.match_prefixes(tree, torch.from_numpy(toks).to(gpu_device), torch.from_numpy(off).to(gpu_device))
    pl, si = pl.cpu().numpy(), si.cpu().numpy()
    np.testing.assert_array_equal(pl, pl_ref)
    for r in range(len(prompts)):
        np.testing.assert_array_equal(si[off[r]:off[r] + pl_ref[r]], si_ref[off[r]:off[r] + pl_ref[r]])


@pytest.mark.parametrize("seed", [0, 1])
def test_match_long_edges_in_a_tree_of_short_ones(pa, gpu_device, seed):
    """Edges of 10,000 to 18,000 tokens, three or four matcher windows long, in a tree whose edges are short on
    average - so that small batches get several workgroups per prompt (a tree of long edges only gets one) and the
    walks cross whole windows inside one edge: prompts that end at and next to window boundaries, inside the long
    edges, at their ends and in the branches that leave them; bit-exact vs the oracle trie."""
    import oracle
    rng = np.random.default_rng(300 + seed)
    vocab = 60000
    cached, nslot = [], 0

    def add(seq):
        nonlocal nslot
        cached.append((np.asarray(seq, np.int32), np.arange(nslot, nslot + len(seq), dtype=np.int32)))
        nslot += len(seq)

    docs = [rng.integers(0, vocab, int(n)).astype(np.int32) for n in (18000, 12500, 10000)]
    for d in docs:
        add(d)
    for _ in range(4):  # branches that leave a document inside its edge
        d = docs[int(rng.integers(0, 3))]
        cut = int(rng.integers(1, len(d)))
        tail = rng.integers(0, vocab, int(rng.integers(5, 400))).astype(np.int32)
        tail[0] = (d[cut] + 1) % vocab
        add(np.concatenate([d[:cut], tail]))
    firsts = set(int(d[0]) for d in docs)
    for _ in range(300):  # many short sequences
        seq = rng.integers(0, vocab, int(rng.integers(3, 20))).astype(np.int32)
        while int(seq[0]) in firsts:
            seq[0] = rng.integers(0, vocab)
        add(seq)
    prompts = []
    for d in docs:
        for cut in (len(d), 4096, 4095, 4097, 8192, 8191, 8193, 12288, 1, int(rng.integers(1, len(d)))):
            cut = min(cut, len(d))
            prompts.append(np.concatenate([d[:cut], rng.integers(0, vocab, int(rng.integers(0, 40))).astype(np.int32)]))
    for c in cached[3:7]:
        prompts.append(np.concatenate([c[0], rng.integers(0, vocab, 9).astype(np.int32)]))
        prompts.append(c[0][: len(c[0]) - 2].copy())
    for _ in range(64 - len(prompts)):
        c = cached[int(rng.integers(0, len(cached)))][0]
        prompts.append(np.concatenate([c[: int(rng.integers(0, len(c) + 1))], rng.integers(0, vocab, 3).astype(np.int32)]))
    assert len(prompts) == 64
    toks = np.concatenate(prompts).astype(np.int32)
    off = np.zeros(len(prompts) + 1, np.int32)
    off[1:] = np.cumsum([len(p) for p in prompts])
    pl_ref, si_ref = oracle.match_prefixes(cached, toks, off)
    assert pl_ref.max() == 18000
    tree = pa.Tree()
    for c in cached:
        tree.insert(*c)
    n_nodes, n_tokens = tree.stats()
    assert n_tokens <= 4096 * (n_nodes - 1)  # (short edges on average: the several-workgroup form)
    tree.upload()
    pl, si = pa.match_prefixes(tree, torch.from_numpy(toks).to(gpu_device), torch.from_numpy(off).to(gpu_device))
    pl, si = pl.cpu().numpy(), si.cpu().numpy()
    np.testing.assert_array_equal(pl, pl_ref)
    for r in range(len(prompts)):
        np.testing.assert_array_equal(si[off[r]:off[r] + pl_ref[r]], si_ref[off[r]:off[r] + pl_ref[r]])


def test_match_empty_tree_and_empty_batch(pa, gpu_device):
    tree = pa.Tree()
    tree.upload()
    toks = torch.arange(10, dtype=torch.int32, device=gpu_device)
    off = torch.tensor([0, 4, 4, 10], dtype=torch.int32, device=gpu_device)
    pl, _ = pa.match_prefixes(tree, toks, off)
    assert pl.cpu().tolist() == [0, 0, 0]
    pl, si = pa.match_prefixes(tree, toks[:0], torch.zeros(1, dtype=torch.int32, device=gpu_device))
    assert pl.numel() == 0 and si.numel() == 0


# ------------------------------------------------------------------------------------ append / gather

@pytest.mark.parametrize("dtype,Hkv,D,page,nslots", [("f32", 2, 64, 1, 512), ("bf16", 8, 128, 16, 4096),
                                                     ("bf16", 2, 64, 16, 1024), ("f32", 1, 128, 4, 64)])
def test_append_gather_round_trip_bit_exact(pa, gpu_device, dtype, Hkv, D, page, nslots):
    """append_kv then gather_kv returns the rows bit for bit, untouched slots keep their previous content
    (Sec. 3.2: computed KV stays cached), and an out-of-pool slot is skipped."""
    rng = np.random.default_rng(5)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    pool = torch.zeros(pa.kv_pool_bytes(nslots, Hkv, D, tdt, page), dtype=torch.uint8, device=gpu_device)
    kw = dict(page_size=page, num_slots=nslots)
    perm = rng.permutation(nslots).astype(np.int32)
    n1, n2 = nslots // 3, nslots // 4
    s1, s2 = perm[:n1], perm[n1:n1 + n2]

    def vals(n):
        x = rng.standard_normal((n, Hkv, D)).astype(np.float32)
        return x if dtype == "f32" else W.f32_to_bf16_bits(x)

    k1, v1, k2, v2 = vals(n1), vals(n1), vals(n2), vals(n2)
    pa.append_kv(pool, torch.from_numpy(s1).to(gpu_device), to_torch(k1, dtype, gpu_device), to_torch(v1, dtype, gpu_device), **kw)
    s2_bad = np.concatenate([s2, np.array([nslots + 7, -3], np.int32)])
    k2b, v2b = np.concatenate([k2, k2[:2]]), np.concatenate([v2, v2[:2]])
    pa.append_kv(pool, torch.from_numpy(s2_bad).to(gpu_device), to_torch(k2b, dtype, gpu_device), to_torch(v2b, dtype, gpu_device), **kw)
    gk, gv = pa.gather_kv(pool, torch.from_numpy(perm).to(gpu_device), Hkv=Hkv, D=D, dtype=tdt, **kw)

    def bits(t):
        return t.view(torch.int16 if dtype == "bf16" else torch.int32).cpu().numpy()

    def ref_bits(a):
        return a.view(np.int16 if dtype == "bf16" else np.int32)

    gk, gv = bits(gk), bits(gv)
    np.testing.assert_array_equal(gk[:n1], ref_bits(k1))
    np.testing.assert_array_equal(gv[:n1], ref_bits(v1))
    np.testing.assert_array_equal(gk[n1:n1 + n2], ref_bits(k2))
    np.testing.assert_array_equal(gv[n1:n1 + n2], ref_bits(v2))
    assert not gk[n1 + n2:].any() and not gv[n1 + n2:].any()


# ------------------------------------------------------------------------------------ whole path, small

@pytest.mark.parametrize("name", SMALL)
@pytest.mark.parametrize("seed", [0, 1])
def test_small_config_whole_path(pa, gpu_device, name, seed):
    """match -> extend -> append on the reduced configs, every output element against the oracle."""
    say(f"[case] small {name} seed={seed}")
    wl = W.small_variant(name, seed)
    g, o = GpuSide(wl, gpu_device), OracleSide(wl)
    pl, si, out = g.step()
    torch.cuda.synchronize()
    pl_ref, si_ref = o.match()
    assert_match_equal(wl, pl, si, pl_ref, si_ref)
    np.testing.assert_array_equal(pl_ref, wl.designed_prefix_len)
    ref = o.extend(pl_ref, si_ref)
    err = np.abs(out_to_f64(out) - ref).max()
    say(f"  max abs err {err:.3e}")
    assert err <= TOL[wl.dtype]
    # the appended rows must read back bit-exactly and leave the prefix rows alone
    o.append()
    allslots = np.concatenate([wl.pool_slots, wl.new_slots])
    gk, gv = pa.gather_kv(g.pool, torch.from_numpy(allslots).to(gpu_device), Hkv=wl.Hkv, D=wl.D, dtype=g.tdtype, **g.kw)
    view = torch.int32 if wl.dtype == "f32" else torch.int16
    npview = np.int32 if wl.dtype == "f32" else np.int16
    np.testing.assert_array_equal(gk.view(view).cpu().numpy(), o.pool_k[allslots].view(npview))
    np.testing.assert_array_equal(gv.view(view).cpu().numpy(), o.pool_v[allslots].view(npview))


def _random_case(rng, B, Hq, Hkv, D, p_hi, e_hi, dtype, page, nslots):
    """Requests with independent random prefixes (slots: whole random pages each) and extends, incl. P=0."""
    from paper_2407_00023_amd.workloads import _normal
    P = rng.integers(0, p_hi + 1, B).astype(np.int32)
    E = rng.integers(0, e_hi + 1, B).astype(np.int32)
    P[0], E[-1] = 0, max(1, E[-1])
    if B > 2:
        E[1] = 0
    pages = rng.permutation(nslots // page)
    cur, slots = 0, []
    for r in range(B):
        npg = (P[r] + page - 1) // page
        t = np.arange(P[r])
        slots.append((pages[cur:cur + npg][t // page] * page + t % page).astype(np.int32) if P[r] else np.zeros(0, np.int32))
        cur += npg
    off = np.zeros(B + 1, np.int32)
    off[1:] = np.cumsum(P + E)
    si = np.full(off[-1], -1, np.int32)
    for r in range(B):
        si[off[r]:off[r] + P[r]] = slots[r]
    eo = np.zeros(B + 1, np.int32)
    eo[1:] = np.cumsum(E)
    T = int(eo[-1])
    ss = np.random.SeedSequence(int(rng.integers(1 << 30))).spawn(5)
    backed = np.concatenate(slots) if B else np.zeros(0, np.int32)
    mk = lambda s, n, h: _normal(s, n * h * D, dtype).reshape(n, h, D)
    return dict(P=P, E=E, off=off, si=si, eo=eo, T=T, backed=backed, q=mk(ss[0], T, Hq), k=mk(ss[1], T, Hkv),
                v=mk(ss[2], T, Hkv), pk=mk(ss[3], len(backed), Hkv), pv=mk(ss[4], len(backed), Hkv))


@pytest.mark.parametrize("dtype,Hq,Hkv,D,page,p_hi,e_hi,B", [
    ("f32", 4, 2, 64, 1, 150, 40, 5),
    ("f32", 2, 1, 128, 4, 70, 20, 3),
    ("bf16", 8, 2, 128, 16, 700, 90, 6),     # several key tiles, ragged tails, packed rows > 128
    ("bf16", 4, 4, 64, 16, 300, 200, 4),     # G = 1, D = 64
    ("bf16", 16, 2, 128, 1, 200, 33, 4),     # G = 8, page size 1
    ("bf16", 8, 8, 128, 16, 5000, 10, 3),    # long prefix, short extend: split path
    ("bf16", 8, 2, 128, 12, 700, 90, 6),     # page sizes that are not powers of two: the page of a slot by division
    ("bf16", 16, 4, 128, 48, 3000, 40, 5),
    ("bf16", 4, 2, 64, 24, 400, 150, 4),
    ("f32", 4, 2, 64, 3, 150, 40, 5),
])
def test_extend_random_shapes(pa, gpu_device, dtype, Hq, Hkv, D, page, p_hi, e_hi, B):
    """Ragged prefixes and extends including prefix_len = 0 and ext_len = 0 requests."""
    import oracle
    say(f"[case] extend_random {dtype} Hq={Hq} Hkv={Hkv} D={D} page={page} p_hi={p_hi} e_hi={e_hi}")
    rng = np.random.default_rng(11)
    nslots = 16384 if 16384 % page == 0 else 18432  # (= 2^11 x 9: divisible by 3, 12, 24, 48)
    c = _random_case(rng, B, Hq, Hkv, D, p_hi, e_hi, dtype, page, nslots)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    dev = gpu_device
    pool = torch.zeros(pa.kv_pool_bytes(nslots, Hkv, D, tdt, page), dtype=torch.uint8, device=dev)
    kw = dict(page_size=page, num_slots=nslots)
    pa.append_kv(pool, torch.from_numpy(c["backed"]).to(dev), to_torch(c["pk"], dtype, dev), to_torch(c["pv"], dtype, dev), **kw)
    tt = lambda a: torch.from_numpy(a).to(dev)
    scale = 1.0 / np.sqrt(D)
    out = pa.extend_attention(to_torch(c["q"], dtype, dev), to_torch(c["k"], dtype, dev), to_torch(c["v"], dtype, dev), pool,
                              tt(c["si"]), tt(c["off"]), tt(c["P"]), tt(c["E"]), tt(c["eo"]), scale,
                              max_kv_len=int((c["P"] + c["E"]).max()), **kw)
    torch.cuda.synchronize()
    opk, opv = oracle.new_pool(nslots, Hkv, D, dtype)
    oracle.append_kv(opk, opv, c["backed"], c["pk"], c["pv"], dtype)
    ref = oracle.extend_attention(c["q"], c["k"], c["v"], opk, opv, c["si"], c["off"], c["P"], c["E"], c["eo"], scale, dtype)
    err = np.abs(out_to_f64(out) - ref).max() if c["T"] else 0.0
    say(f"  max abs err {err:.3e}")
    assert err <= TOL[dtype]


@pytest.mark.parametrize("direction", ["growing", "shrinking"])
def test_extend_running_maximum_rescale(pa, gpu_device, direction):
    """Scores whose magnitude grows (or shrinks) along the key axis by far more than the lag the kernel allows its
    running maximum: the accumulators have to be rescaled many times after the first tile (the online-softmax
    path that random N(0,1) data never takes).  Same bar as everywhere: 2e-2 against the fp64 oracle."""
    import oracle
    rng = np.random.default_rng(21)
    Hq, Hkv, D, page, nslots, B = 8, 2, 128, 16, 8192, 3
    c = _random_case(rng, B, Hq, Hkv, D, 1500, 150, "bf16", page, nslots)
    # multiply key j of every request by a ramp, so that |q.k| scale sweeps over two orders of magnitude
    def ramp(n):
        r = np.linspace(0.05, 6.0, max(n, 1))[:n]
        return r if direction == "growing" else r[::-1]
    pk = W.bf16_bits_to_f32(c["pk"]).copy()
    k = W.bf16_bits_to_f32(c["k"]).copy()
    cur = 0
    for r in range(B):
        P, E = int(c["P"][r]), int(c["E"][r])
        f = ramp(P + E)
        pk[cur:cur + P] *= f[:P, None, None]
        k[c["eo"][r]:c["eo"][r] + E] *= f[P:, None, None]
        cur += P
    c["pk"], c["k"] = W.f32_to_bf16_bits(pk), W.f32_to_bf16_bits(k)
    dev = gpu_device
    pool = torch.zeros(pa.kv_pool_bytes(nslots, Hkv, D, torch.bfloat16, page), dtype=torch.uint8, device=dev)
    kw = dict(page_size=page, num_slots=nslots)
    pa.append_kv(pool, torch.from_numpy(c["backed"]).to(dev), to_torch(c["pk"], "bf16", dev), to_torch(c["pv"], "bf16", dev), **kw)
    tt = lambda a: torch.from_numpy(a).to(dev)
    scale = 1.0 / np.sqrt(D)
    out = pa.extend_attention(to_torch(c["q"], "bf16", dev), to_torch(c["k"], "bf16", dev), to_torch(c["v"], "bf16", dev), pool,
                              tt(c["si"]), tt(c["off"]), tt(c["P"]), tt(c["E"]), tt(c["eo"]), scale,
                              max_kv_len=int((c["P"] + c["E"]).max()), **kw)
    torch.cuda.synchronize()
    opk, opv = oracle.new_pool(nslots, Hkv, D, "bf16")
    oracle.append_kv(opk, opv, c["backed"], c["pk"], c["pv"], "bf16")
    ref = oracle.extend_attention(c["q"], c["k"], c["v"], opk, opv, c["si"], c["off"], c["P"], c["E"], c["eo"], scale, "bf16")
    err = np.abs(out_to_f64(out) - ref).max()
    say(f"  {direction}: max abs err {err:.3e}")
    assert np.isfinite(out_to_f64(out)).all() and err <= TOL["bf16"]


@pytest.mark.parametrize("jump_at", [0.3, 0.6, 0.9])
def test_extend_score_jump_leaves_the_steady_state_run(pa, gpu_device, jump_at):
    """Keys whose scores jump by far more than 2^40 (in probability) part of the way through the prefix or the
    extend tokens: the runs of steady-state tiles, which never move the running maximum, have to hand the tile
    that outgrows it to the general code (in its first or its second key block) and the result must still meet the
    same bar.  Requests are long enough for such runs to exist."""
    import oracle
    rng = np.random.default_rng(int(jump_at * 100))
    Hq, Hkv, D, page, nslots, B = 8, 2, 128, 16, 16384, 4
    c = _random_case(rng, B, Hq, Hkv, D, 3000, 400, "bf16", page, nslots)
    pk = W.bf16_bits_to_f32(c["pk"]).copy()
    k = W.bf16_bits_to_f32(c["k"]).copy()
    cur = 0
    for r in range(B):
        P, E = int(c["P"][r]), int(c["E"][r])
        f = np.ones(P + E, np.float32)
        j = int((P + E) * jump_at) + r  # not tile-aligned, differs per request
        f[j:] = 48.0                    # scores x 48: tens of log2 units above anything before
        pk[cur:cur + P] *= f[:P, None, None]
        k[c["eo"][r]:c["eo"][r] + E] *= f[P:, None, None]
        cur += P
    c["pk"], c["k"] = W.f32_to_bf16_bits(pk), W.f32_to_bf16_bits(k)
    dev = gpu_device
    pool = torch.zeros(pa.kv_pool_bytes(nslots, Hkv, D, torch.bfloat16, page), dtype=torch.uint8, device=dev)
    kw = dict(page_size=page, num_slots=nslots)
    pa.append_kv(pool, torch.from_numpy(c["backed"]).to(dev), to_torch(c["pk"], "bf16", dev), to_torch(c["pv"], "bf16", dev), **kw)
    tt = lambda a: torch.from_numpy(a).to(dev)
    scale = 1.0 / np.sqrt(D)
    out = pa.extend_attention(to_torch(c["q"], "bf16", dev), to_torch(c["k"], "bf16", dev), to_torch(c["v"], "bf16", dev), pool,
                              tt(c["si"]), tt(c["off"]), tt(c["P"]), tt(c["E"]), tt(c["eo"]), scale,
                              max_kv_len=int((c["P"] + c["E"]).max()), **kw)
    torch.cuda.synchronize()
    opk, opv = oracle.new_pool(nslots, Hkv, D, "bf16")
    oracle.append_kv(opk, opv, c["backed"], c["pk"], c["pv"], "bf16")
    ref = oracle.extend_attention(c["q"], c["k"], c["v"], opk, opv, c["si"], c["off"], c["P"], c["E"], c["eo"], scale, "bf16")
    err = np.abs(out_to_f64(out) - ref).max()
    say(f"  jump at {jump_at}: max abs err {err:.3e}")
    assert np.isfinite(out_to_f64(out)).all() and err <= TOL["bf16"]


def test_extend_slot_permutation_invariance(pa, gpu_device):
    """Moving the cached rows to other slots (and renaming slot_idx accordingly) must not change a single bit."""
    wl = W.small_variant("tool_use", 3)
    g = GpuSide(wl, gpu_device)
    pl, si = g.match()
    out1 = g.extend(pl, si).clone()
    rng = np.random.default_rng(0)
    remap = rng.permutation(wl.num_slots).astype(np.int32)
    pool2 = torch.zeros_like(g.pool)
    g.pa.append_kv(pool2, torch.from_numpy(remap[wl.pool_slots]).to(gpu_device), to_torch(wl.pool_k, wl.dtype, gpu_device),
                   to_torch(wl.pool_v, wl.dtype, gpu_device), **g.kw)
    si2 = torch.from_numpy(remap).to(gpu_device)[si.clamp(0, wl.num_slots - 1).long()].to(torch.int32)
    out2 = g.pa.extend_attention(g.q, g.k, g.v, pool2, si2, g.offsets, pl, g.ext_len, g.ext_offsets, wl.scale,
                                 max_kv_len=g.max_kv_len, **g.kw)
    torch.cuda.synchronize()
    assert torch.equal(out1.view(torch.int16), out2.view(torch.int16))


@pytest.mark.parametrize("page", [12, 48])
def test_whole_path_with_a_page_size_that_is_no_power_of_two(pa, gpu_device, page):
    """Tool-use-shaped batch on a pool of 12- or 48-token pages: tree, match, attention (whole tiles, shared tiles of
    left-over rows, split key ranges) and append all address the pool by dividing by the page size; every element against
    the oracle and the appended rows bit-exact."""
    say(f"[case] page size {page}")
    wl = W.tool_use(7, B=10, sys_len=900, n_tools=3, tool_lo=50, tool_hi=400, ext_lo=5, ext_hi=200, Hq=16, Hkv=4,
                    num_slots=36864, page_size=page)
    g, o = GpuSide(wl, gpu_device), OracleSide(wl)
    pl, si, out = g.step()
    torch.cuda.synchronize()
    pl_ref, si_ref = o.match()
    assert_match_equal(wl, pl, si, pl_ref, si_ref)
    err = np.abs(out_to_f64(out) - o.extend(pl_ref, si_ref)).max()
    say(f"  max abs err {err:.3e}")
    assert err <= TOL[wl.dtype]
    o.append()
    allslots = np.concatenate([wl.pool_slots, wl.new_slots])
    gk, gv = pa.gather_kv(g.pool, torch.from_numpy(allslots).to(gpu_device), Hkv=wl.Hkv, D=wl.D, dtype=g.tdtype, **g.kw)
    np.testing.assert_array_equal(gk.view(torch.int16).cpu().numpy(), o.pool_k[allslots].view(np.int16))
    np.testing.assert_array_equal(gv.view(torch.int16).cpu().numpy(), o.pool_v[allslots].view(np.int16))


def _hand_built_lists(rng, kind, nslots, page):
    """Five requests whose slot lists were NOT read off one prefix tree: they end in the same slot (and, by kind, also
    have the same length, first and middle slot) but differ elsewhere."""
    B, P0 = 5, 640
    base = rng.permutation(nslots)[:P0].astype(np.int32)
    lists = []
    for r in range(B):
        if kind == "unequal_length":       # same last slot, different lengths: tails of one list
            lst = base[r * 17:].copy()
        elif kind == "differs_early":      # same length and last slot, other slots before the middle
            lst = base.copy()
            lst[1 + r:200 + r] = rng.permutation(nslots)[:199].astype(np.int32)
            lst[0] = base[r]                # (and a first slot of its own)
        else:                              # "differs_between_probes": equal at every place a planner could cheaply look
            lst = base.copy()
            if r:
                lst[3 + r] = base[400 + r]
                lst[500 + r] = base[40 + r]
        lists.append(lst)
    return lists


@pytest.mark.parametrize("kind,sharing", [("unequal_length", True), ("differs_early", True),
                                          ("differs_between_probes", False), ("unequal_length", False)])
def test_extend_slot_lists_that_do_not_come_from_one_tree(pa, gpu_device, kind, sharing):
    """Slot lists built by hand.  Lists that end in the same slot but differ in length or in their early slots must
    not be taken for a shared prefix (every element against the oracle with row sharing on); lists that agree at every
    place the grouping looks at and differ in between are what pa_extend_set_row_sharing(0) is for."""
    import oracle
    say(f"[case] hand-built slot lists: {kind}, row sharing {'on' if sharing else 'off'}")
    rng = np.random.default_rng(31)
    Hq, Hkv, D, page, nslots = 8, 2, 128, 16, 8192
    lists = _hand_built_lists(rng, kind, nslots, page)
    B = len(lists)
    P = np.array([len(x) for x in lists], np.int32)
    E = rng.integers(3, 30, B).astype(np.int32)   # a few rows each: left-over rows only, the ones that get packed
    off = np.zeros(B + 1, np.int32)
    off[1:] = np.cumsum(P + E)
    si = np.full(off[-1], -1, np.int32)
    for r in range(B):
        si[off[r]:off[r] + P[r]] = lists[r]
    eo = np.zeros(B + 1, np.int32)
    eo[1:] = np.cumsum(E)
    T = int(eo[-1])
    ss = np.random.SeedSequence(5).spawn(5)
    mk = lambda s_, n, h: W._normal(s_, n * h * D, "bf16").reshape(n, h, D)
    backed = np.arange(nslots, dtype=np.int32)
    q, k, v, pk, pv = mk(ss[0], T, Hq), mk(ss[1], T, Hkv), mk(ss[2], T, Hkv), mk(ss[3], nslots, Hkv), mk(ss[4], nslots, Hkv)
    dev = gpu_device
    pool = torch.zeros(pa.kv_pool_bytes(nslots, Hkv, D, torch.bfloat16, page), dtype=torch.uint8, device=dev)
    kw = dict(page_size=page, num_slots=nslots)
    pa.append_kv(pool, torch.from_numpy(backed).to(dev), to_torch(pk, "bf16", dev), to_torch(pv, "bf16", dev), **kw)
    tt = lambda a: torch.from_numpy(a).to(dev)
    scale = 1.0 / np.sqrt(D)
    pa.extend_set_row_sharing(sharing)
    try:
        out = pa.extend_attention(to_torch(q, "bf16", dev), to_torch(k, "bf16", dev), to_torch(v, "bf16", dev), pool, tt(si),
                                  tt(off), tt(P), tt(E), tt(eo), scale, max_kv_len=int((P + E).max()), **kw)
        torch.cuda.synchronize()
    finally:
        pa.extend_set_row_sharing(True)
    opk, opv = oracle.new_pool(nslots, Hkv, D, "bf16")
    oracle.append_kv(opk, opv, backed, pk, pv, "bf16")
    ref = oracle.extend_attention(q, k, v, opk, opv, si, off, P, E, eo, scale, "bf16")
    err = np.abs(out_to_f64(out) - ref).max()
    say(f"  max abs err {err:.3e}")
    assert err <= TOL["bf16"]


def test_extend_reports_a_batch_larger_than_the_host_sizes(pa, gpu_device):
    """pa_extend_attention sizes its launch from the host values T and max_kv_len.  Given a T smaller than what ext_len
    on the device adds up to, the work list does not fit: no output row is written, and pa_extend_status says so
    (PA_EOVERFLOW); after a proper call on the same workspace it reports success again."""
    import ctypes as C
    wl = W.small_variant("agent_tree", 2)
    g = GpuSide(wl, gpu_device)
    pl, si = g.match()
    nbytes = pa.extend_workspace_bytes(wl.B, wl.T, g.max_kv_len, wl.Hq, wl.Hkv, wl.D, g.tdtype)
    ws = torch.zeros(nbytes, dtype=torch.uint8, device=gpu_device)
    out = torch.full_like(g.q, 7.0)
    lib = pa._lib
    T_lie = 64  # the device-side ext_len adds up to wl.T, far more row tiles than 64 tokens make
    assert wl.T * (wl.Hq // wl.Hkv) // 128 > T_lie * (wl.Hq // wl.Hkv) // 128 + wl.B + 1
    rc = lib.pa_extend_attention(pa._ptr(g.q), pa._ptr(g.k), pa._ptr(g.v), pa._ptr(g.pool), pa._ptr(si), pa._ptr(g.offsets),
                                 pa._ptr(pl), pa._ptr(g.ext_len), pa._ptr(g.ext_offsets), wl.B, T_lie, g.max_kv_len, wl.Hq,
                                 wl.Hkv, wl.D, wl.page_size, wl.num_slots, pa.BF16, float(wl.scale), pa._ptr(out), pa._ptr(ws),
                                 nbytes, pa._stream(None))
    assert rc == 0  # the call itself cannot know: it never waits for the device
    with pytest.raises(pa.PrefixAttnError) as e:
        pa.extend_status(ws)
    assert e.value.code == -5
    assert bool((out == 7.0).all())  # nothing was written
    g.extend(pl, si, workspace=ws, out=out)
    pa.extend_status(ws)
    assert torch.isfinite(out.float()).all() and not bool((out == 7.0).all())


def test_extend_pool_beyond_4_gib(pa, gpu_device):
    """A KV pool of 6.4 GB (1.5 M slots x 8 KV heads x 128 x bf16 x K and V): pool rows lie on either side of the 4 GiB line, so
    byte offsets no longer fit 32 bits - the assembly runs address rows in units of 256 bytes and form the address in
    64 bits, the general tile and append / gather compute in 64 bits throughout.  Every element against the oracle, and
    the appended rows bit-exact."""
    say("[case] pool beyond 4 GiB")
    wl = W.tool_use(21, B=8, sys_len=1300, n_tools=3, tool_lo=100, tool_hi=500, ext_lo=20, ext_hi=160, num_slots=1_572_864)
    row_bytes = 2 * wl.Hkv * wl.D * 2
    page_off = (wl.pool_slots.astype(np.int64) // wl.page_size) * wl.page_size * row_bytes
    assert (page_off < 2 ** 32).sum() > 100 and (page_off >= 2 ** 32).sum() > 100
    g, o = GpuSide(wl, gpu_device), OracleSide(wl)
    pl, si, out = g.step()
    torch.cuda.synchronize()
    pl_ref, si_ref = o.match()
    assert_match_equal(wl, pl, si, pl_ref, si_ref)
    err = np.abs(out_to_f64(out) - o.extend(pl_ref, si_ref)).max()
    say(f"  max abs err {err:.3e}")
    assert err <= TOL[wl.dtype]
    o.append()
    allslots = np.concatenate([wl.pool_slots, wl.new_slots])
    gk, gv = pa.gather_kv(g.pool, torch.from_numpy(allslots).to(gpu_device), Hkv=wl.Hkv, D=wl.D, dtype=g.tdtype, **g.kw)
    np.testing.assert_array_equal(gk.view(torch.int16).cpu().numpy(), o.pool_k[allslots].view(np.int16))
    np.testing.assert_array_equal(gv.view(torch.int16).cpu().numpy(), o.pool_v[allslots].view(np.int16))
    del g
    torch.cuda.empty_cache()


# ------------------------------------------------------------------------------------ full configs

@pytest.fixture(scope="module")
def full_cache():
    return {}


def _full(name, device, cache):
    if name not in cache:
        cache.clear()  # one full config resident at a time
        wl = W.CONFIGS[name]()
        cache[name] = (wl, GpuSide(wl, device), OracleSide(wl))
    return cache[name]


@pytest.mark.parametrize("name", FULL)
def test_full_config_match_bit_exact(pa, gpu_device, full_cache, name):
    say(f"[case] full match {name}")
    wl, g, o = _full(name, gpu_device, full_cache)
    pl, si = g.match()
    torch.cuda.synchronize()
    pl_ref, si_ref = o.match()
    assert_match_equal(wl, pl, si, pl_ref, si_ref)
    np.testing.assert_array_equal(pl_ref, wl.designed_prefix_len)


def _pairs_for_partial_check(wl, frac, seed=1):
    """(request, query head) pairs whose every row is compared when the oracle cannot do the whole batch: all heads of
    the longest and the shortest request, of requests that share their whole prefix with another one (their left-over
    rows sit in shared row tiles), then random pairs up to `frac` of all pairs."""
    rng = np.random.default_rng(seed)
    want = int(np.ceil(frac * wl.B * wl.Hq))
    chosen, seen = [], set()

    def add(r, h):
        if (r, h) not in seen:
            seen.add((r, h))
            chosen.append((r, h))

    for r in (int(np.argmax(wl.ext_len)), int(np.argmin(wl.ext_len))):
        for h in range(wl.Hq):
            add(r, h)
    key = {}
    for r in range(wl.B):
        lo, P = int(wl.offsets[r]), int(wl.designed_prefix_len[r])
        key.setdefault((P, int(wl.designed_slots[lo + P - 1]) if P else -1 - r), []).append(r)
    sharers = [r for rs in key.values() if len(rs) > 1 for r in rs]
    for r in sharers[:max(2, want // (2 * wl.Hq))]:
        for h in range(wl.Hq):
            add(r, h)
    while len(chosen) < want:
        add(int(rng.integers(0, wl.B)), int(rng.integers(0, wl.Hq)))
    return chosen


@pytest.mark.parametrize("name", FULL)
def test_full_config_extend_every_element(pa, gpu_device, full_cache, name):
    """Full sizes, in the launch configuration the benchmark times.  Every output element against the oracle; on
    agent_tree, whose oracle run would take a minute, every row of a quarter of the (request, head) pairs: all heads of
    the longest and shortest requests and of requests whose left-over rows are packed into shared tiles, the rest drawn
    at random.  The error is reported for rows in full 128-row tiles and for left-over rows apart (the latter are the
    ones that shared tiles hold), next to what the work list says about tiles, items and merged tiles.  Plus a property
    that holds at any size: every output element lies inside the range of the visible V."""
    say(f"[case] full extend {name}")
    wl, g, o = _full(name, gpu_device, full_cache)
    pl, si = g.match()
    nbytes = pa.extend_workspace_bytes(wl.B, wl.T, g.max_kv_len, wl.Hq, wl.Hkv, wl.D, g.tdtype)
    ws = torch.zeros(nbytes, dtype=torch.uint8, device=gpu_device)
    out = g.extend(pl, si, workspace=ws)
    torch.cuda.synchronize()
    pa.extend_status(ws)
    n_tiles, n_items, n_merge, overflow = ws[:16].view(torch.int32).tolist()
    assert overflow == 0 and n_items >= n_tiles >= 1
    assert torch.isfinite(out.float()).all()
    pl_ref, si_ref = o.match()
    G = wl.Hq // wl.Hkv
    if name == "agent_tree":
        pairs = _pairs_for_partial_check(wl, 0.25)
        rows = np.concatenate([np.stack([np.full(wl.ext_len[r], r), np.arange(wl.ext_len[r]), np.full(wl.ext_len[r], h)], 1)
                               for r, h in pairs]).astype(np.int32)
        ref = o.extend(pl_ref, si_ref, rows=rows)
        flat = torch.from_numpy(wl.ext_offsets[rows[:, 0]].astype(np.int64) + rows[:, 1]).to(gpu_device)
        got = out_to_f64(out[flat, torch.from_numpy(rows[:, 2].astype(np.int64)).to(gpu_device)])
        covered = f"{len(pairs)} of {wl.B * wl.Hq} (request, head) pairs, {len(rows)} rows"
    else:
        ref = o.extend(pl_ref, si_ref).reshape(wl.T * wl.Hq, wl.D)
        got = out_to_f64(out).reshape(wl.T * wl.Hq, wl.D)
        r_of = np.repeat(np.arange(wl.B), wl.ext_len)
        i_of = np.arange(wl.T) - wl.ext_offsets[r_of]
        rows = np.stack([np.repeat(r_of, wl.Hq), np.repeat(i_of, wl.Hq), np.tile(np.arange(wl.Hq), wl.T)], 1)
        covered = f"all {len(rows)} rows"
    err_rows = np.abs(got - ref).max(axis=1)
    rho = rows[:, 1].astype(np.int64) * G + rows[:, 2] % G
    n_rows = wl.ext_len[rows[:, 0]].astype(np.int64) * G
    leftover = rho >= (n_rows // 128) * 128
    e_full = float(err_rows[~leftover].max()) if (~leftover).any() else 0.0
    e_left = float(err_rows[leftover].max()) if leftover.any() else 0.0
    say(f"  {covered}: max abs err {err_rows.max():.3e} (rows of full tiles {e_full:.3e}, left-over rows {e_left:.3e}); "
        f"work list: {n_tiles} row tiles, {n_items} items, {n_merge} tiles merged from parts")
    assert err_rows.max() <= TOL[wl.dtype]
    # softmax weights are a convex combination: |out| can never exceed the largest |V| in the inputs
    vmax = max(float(np.abs(W.bf16_bits_to_f32(wl.pool_v)).max()), float(np.abs(W.bf16_bits_to_f32(wl.v_ext)).max()))
    assert float(out.float().abs().max()) <= vmax * (1 + 2 ** -7)


def test_the_path_on_a_stream_of_the_callers(pa, gpu_device):
    """Every call takes the stream it enqueues on.  Upload, match, extend and append on a side stream, with the
    default stream kept busy by unrelated work, give bit for bit what the same calls give on the default stream."""
    wl = W.small_variant("agent_tree", 9)
    ga, gb = GpuSide(wl, gpu_device), GpuSide(wl, gpu_device)
    pl_a, si_a = ga.match()
    out_a = ga.extend(pl_a, si_a)
    ga.append()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    busy = torch.randn(4096, 4096, device=gpu_device)
    for _ in range(4):
        busy = busy @ busy * 1e-3          # on the default stream, meanwhile
    with torch.cuda.stream(side):
        gb.tree.insert(np.array([5, 6, 7], np.int32), np.array([0, 1, 2], np.int32) + wl.num_slots)  # makes the mirror stale
        gb.tree.upload(stream=side)
        pl_b, si_b = pa.match_prefixes(gb.tree, gb.tokens, gb.offsets, stream=side)
        out_b = pa.extend_attention(gb.q, gb.k, gb.v, gb.pool, si_b, gb.offsets, pl_b, gb.ext_len, gb.ext_offsets, wl.scale,
                                    max_kv_len=gb.max_kv_len, stream=side, **gb.kw)
        pa.append_kv(gb.pool, gb.new_slots, gb.k, gb.v, stream=side, **gb.kw)
    side.synchronize()
    torch.cuda.synchronize()
    assert torch.equal(pl_a, pl_b)
    for r in range(wl.B):
        lo, P = int(wl.offsets[r]), int(pl_a[r])
        assert torch.equal(si_a[lo:lo + P], si_b[lo:lo + P])
    assert torch.equal(out_a, out_b)
    assert torch.equal(ga.pool, gb.pool)


def test_match_calls_in_flight_on_several_streams(pa, gpu_device):
    """Matches of long prompts (several workgroups per prompt, which meet in buffers of the library's own) enqueued on
    eight streams at once, many times over, each with outputs of its own: every one of them bit for bit what the same
    call gives alone."""
    wl = W.small_variant("video_qa", 3)
    wl2 = W.video_qa(5, B=6, vis_len=9000, n_templates=2, tmpl_len=60, ext_lo=4, ext_hi=9, n_cached=300, len_lo=200,
                     len_hi=9500, Hq=16, Hkv=2, num_slots=32768)
    sides = [GpuSide(w, gpu_device) for w in (wl, wl2)]
    want = [g.match() for g in sides]
    torch.cuda.synchronize()
    assert int(want[1][0].max()) > 8192          # (prompts that reach into a third window)
    streams = [torch.cuda.Stream() for _ in range(8)]
    got = []
    for rep in range(12):
        for k in range(len(streams)):
            got.append(((rep + k) % 2, torch.full_like(want[(rep + k) % 2][0], -7), torch.full_like(want[(rep + k) % 2][1], -7)))
    torch.cuda.synchronize()  # (the outputs are filled on the current stream: done before any match on another one starts)
    for i, (which, pl, si) in enumerate(got):
        g = sides[which]
        pa.match_prefixes(g.tree, g.tokens, g.offsets, pl, si, stream=streams[i % len(streams)])
    for st in streams:
        st.synchronize()
    torch.cuda.synchronize()
    for which, pl, si in got:
        w, (pl_w, si_w) = sides[which].wl, want[which]
        assert torch.equal(pl, pl_w)
        for r in range(w.B):
            lo, P = int(w.offsets[r]), int(pl_w[r])
            assert torch.equal(si[lo:lo + P], si_w[lo:lo + P])


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_extend_packs_leftover_rows_of_requests_with_a_common_prefix(pa, gpu_device, seed):
    """Requests that share a prefix of 512 keys or more have the rows past their last full 128-row tile laid end to
    end into shared tiles, which walk the prefix and then each member's extend tokens: every element against the
    oracle, and the header of the work list says that there are fewer tiles than one request at a time would need."""
    say(f"[case] packed left-over rows, seed {seed}")
    wl = W.tool_use(seed, B=9, sys_len=520, n_tools=2, tool_lo=30, tool_hi=140, ext_lo=3, ext_hi=90, Hq=8, Hkv=2,
                    num_slots=8192)
    assert (wl.designed_prefix_len >= 512).all()
    g, o = GpuSide(wl, gpu_device), OracleSide(wl)
    pl, si = g.match()
    nbytes = pa.extend_workspace_bytes(wl.B, wl.T, g.max_kv_len, wl.Hq, wl.Hkv, wl.D, g.tdtype)
    ws = torch.zeros(nbytes, dtype=torch.uint8, device=gpu_device)
    out = g.extend(pl, si, workspace=ws)
    torch.cuda.synchronize()
    n_tiles, n_items, n_merge, overflow = ws[:16].view(torch.int32).tolist()
    groups = len(set(wl.notes["tool_of_request"].tolist()))
    rows = wl.ext_len.astype(np.int64) * (wl.Hq // wl.Hkv)
    unpacked = int(((rows + 127) // 128).sum())
    say(f"  tiles {n_tiles} (one request at a time: {unpacked}), items {n_items}, merged tiles {n_merge}; {groups} prefix groups")
    assert overflow == 0 and n_tiles < unpacked
    pl_ref, si_ref = o.match()
    assert_match_equal(wl, pl, si, pl_ref, si_ref)
    ref = o.extend(pl_ref, si_ref)
    err = np.abs(out_to_f64(out) - ref).max()
    say(f"  max abs err {err:.3e}")
    assert err <= TOL[wl.dtype]


@pytest.mark.parametrize("case", ["one_trunk", "two_levels", "exact_multiple", "long_own_parts", "three_tokens"])
def test_extend_shares_tiles_between_requests_with_a_common_first_part(pa, gpu_device, case):
    """Decode-shaped batches: every request has prefix keys of its own behind a part it shares with others.  Requests
    with the same first part are packed into shared row tiles that walk the common keys once and then every member's
    own (rest of its prefix from the pool through its own slot list, then its new tokens): every element against the
    oracle, and fewer tiles than requests."""
    say(f"[case] common first part, {case}")
    kw = dict(Hq=8, Hkv=2, num_slots=16384)
    if case == "one_trunk":        # one tool: a common part of sys + tool, found by bisection between two probe depths
        wl = W.decode(1, B=9, sys_len=600, n_tools=1, tool_lo=77, tool_hi=77, own_lo=1, own_hi=120, **kw)
    elif case == "two_levels":     # three tools behind one system prompt
        wl = W.decode(2, B=14, sys_len=700, n_tools=3, tool_lo=400, tool_hi=900, own_lo=3, own_hi=90, **kw)
    elif case == "exact_multiple":  # the common part ends on a probe depth and on a tile boundary
        wl = W.decode(3, B=7, sys_len=1000, n_tools=1, tool_lo=24, tool_hi=24, own_lo=1, own_hi=70, **kw)
    elif case == "long_own_parts":  # own parts of several tiles, shared tiles split into parts
        wl = W.decode(4, B=12, sys_len=4000, n_tools=2, tool_lo=10, tool_hi=40, own_lo=200, own_hi=900,
                      **dict(kw, num_slots=32768))
    else:                          # three new tokens per request instead of one
        wl = W.decode(5, B=10, sys_len=800, n_tools=2, tool_lo=100, tool_hi=300, own_lo=1, own_hi=200, ext=3, **kw)
    g, o = GpuSide(wl, gpu_device), OracleSide(wl)
    pl, si = g.match()
    nbytes = pa.extend_workspace_bytes(wl.B, wl.T, g.max_kv_len, wl.Hq, wl.Hkv, wl.D, g.tdtype)
    ws = torch.zeros(nbytes, dtype=torch.uint8, device=gpu_device)
    out = g.extend(pl, si, workspace=ws)
    torch.cuda.synchronize()
    n_tiles, n_items, n_merge, overflow = ws[:16].view(torch.int32).tolist()
    say(f"  {wl.B} requests, tiles {n_tiles}, items {n_items}, merged tiles {n_merge}")
    assert overflow == 0 and n_tiles < wl.B
    pl_ref, si_ref = o.match()
    assert_match_equal(wl, pl, si, pl_ref, si_ref)
    ref = o.extend(pl_ref, si_ref)
    err = np.abs(out_to_f64(out) - ref).max()
    say(f"  max abs err {err:.3e}")
    assert err <= TOL[wl.dtype]


@pytest.mark.parametrize("seed", range(12))
def test_extend_random_decode_batches_against_the_oracle(pa, gpu_device, seed):
    """Random batches of requests with prefix keys of their own behind a shared part: how long the shared levels are
    (below and above the 512 keys that grouping asks for), how many second-level prefixes, how long the own parts, one
    to forty new tokens per request (so that some requests have more than a tile of rows and stay out of the groups),
    head counts and page size - every element against the oracle."""
    rng = np.random.default_rng(1000 + seed)
    Hkv = int(rng.choice([1, 2, 4]))
    G = int(rng.choice([1, 4, 8]))
    wl = W.decode(seed, B=int(rng.integers(2, 25)), sys_len=int(rng.choice([100, 500, 511, 512, 640, 1500])),
                  n_tools=int(rng.integers(1, 5)), tool_lo=1, tool_hi=int(rng.choice([2, 60, 700])), own_lo=1,
                  own_hi=int(rng.choice([1, 30, 300])), ext=(1, int(rng.choice([1, 3, 40]))), Hq=Hkv * G, Hkv=Hkv,
                  num_slots=32768, page_size=int(rng.choice([1, 16, 64])))
    say(f"[case] random decode batch, seed {seed}: B {wl.B}, Hq {wl.Hq}, Hkv {wl.Hkv}, page {wl.page_size}, "
        f"prefixes {wl.designed_prefix_len.min()}..{wl.designed_prefix_len.max()}, new tokens {wl.ext_len.min()}..{wl.ext_len.max()}")
    g, o = GpuSide(wl, gpu_device), OracleSide(wl)
    pl, si = g.match()
    nbytes = pa.extend_workspace_bytes(wl.B, wl.T, g.max_kv_len, wl.Hq, wl.Hkv, wl.D, g.tdtype)
    ws = torch.zeros(nbytes, dtype=torch.uint8, device=gpu_device)
    out = g.extend(pl, si, workspace=ws)
    torch.cuda.synchronize()
    n_tiles, n_items, n_merge, overflow = ws[:16].view(torch.int32).tolist()
    say(f"  tiles {n_tiles}, items {n_items}, merged {n_merge}")
    assert overflow == 0
    pl_ref, si_ref = o.match()
    assert_match_equal(wl, pl, si, pl_ref, si_ref)
    ref = o.extend(pl_ref, si_ref)
    err = np.abs(out_to_f64(out) - ref).max()
    say(f"  max abs err {err:.3e}")
    assert err <= TOL[wl.dtype]


@pytest.mark.parametrize("seed", range(24))
def test_extend_random_shapes_against_the_oracle(pa, gpu_device, seed):
    """Small batches of random shape - head counts, head size, page size, number of requests, how many share a
    prefix and whether it is long enough to be packed, extend lengths from one token to a few tiles - every element
    against the oracle.  (The work list, the packing of left-over rows and the split of long key ranges all take
    their decisions from these numbers.)"""
    rng = np.random.default_rng(7000 + seed)
    Hkv = int(rng.choice([1, 2, 4]))
    G = int(rng.choice([1, 2, 4, 8]))
    D = int(rng.choice([64, 128]))
    page = int(rng.choice([1, 4, 16, 32]))
    B = int(rng.integers(1, 24))
    sys_len = int(rng.choice([1, 40, 300, 520, 700, 1500]))
    n_tools = int(rng.integers(1, 5))
    tool_hi = int(rng.choice([2, 30, 200, 600]))
    ext_hi = int(rng.choice([1, 3, 40, 130, 400]))
    say(f"[case] random shape {seed}: B={B} Hq={Hkv * G} Hkv={Hkv} D={D} page={page} sys={sys_len} tools={n_tools}x<={tool_hi} "
        f"ext<={ext_hi}")
    wl = W.tool_use(seed, B=B, sys_len=sys_len, n_tools=n_tools, tool_lo=1, tool_hi=tool_hi, ext_lo=1, ext_hi=ext_hi,
                    Hq=Hkv * G, Hkv=Hkv, D=D, num_slots=32768, page_size=page)
    g, o = GpuSide(wl, gpu_device), OracleSide(wl)
    pl, si = g.match()
    nbytes = pa.extend_workspace_bytes(wl.B, wl.T, g.max_kv_len, wl.Hq, wl.Hkv, wl.D, g.tdtype)
    ws = torch.zeros(nbytes, dtype=torch.uint8, device=gpu_device)
    out = g.extend(pl, si, workspace=ws)
    torch.cuda.synchronize()
    n_tiles, n_items, n_merge, overflow = ws[:16].view(torch.int32).tolist()
    assert overflow == 0 and n_items >= n_tiles >= 1
    pl_ref, si_ref = o.match()
    assert_match_equal(wl, pl, si, pl_ref, si_ref)
    ref = o.extend(pl_ref, si_ref)
    err = np.abs(out_to_f64(out) - ref).max()
    say(f"  tiles {n_tiles}, items {n_items}, merged {n_merge}; max abs err {err:.3e}")
    assert err <= TOL[wl.dtype]


@pytest.mark.parametrize("case", ["many_requests", "many_tiles", "pack_256", "no_pack_300"])
def test_extend_work_list_beyond_the_small_table_sizes(pa, gpu_device, case):
    """The kernel that plans a launch keeps its tables in LDS for up to 1,024 requests and 3,072 row tiles and in
    global memory beyond (more than 1,024 requests also keep their given order), and packs left-over rows in batches
    of up to 256 requests: shapes on either side of these limits against the oracle."""
    say(f"[case] work list {case}")
    if case == "many_requests":
        wl = W.tiny_fp32(seed=11, B=1100, prefix=96, ext_lo=1, ext_hi=5, n_distract=2, Hq=8, Hkv=2, D=64,
                         num_slots=32768, page_size=16, dtype="bf16")
    elif case == "pack_256":   # one prefix of 600 keys shared by 256 requests of 1..9 new tokens: 4..36 rows each
        wl = W.tiny_fp32(seed=13, B=256, prefix=600, ext_lo=1, ext_hi=9, n_distract=2, Hq=8, Hkv=2, D=128,
                         num_slots=32768, page_size=16, dtype="bf16")
    elif case == "no_pack_300":
        wl = W.tiny_fp32(seed=14, B=300, prefix=600, ext_lo=1, ext_hi=9, n_distract=2, Hq=8, Hkv=2, D=128,
                         num_slots=32768, page_size=16, dtype="bf16")
    else:
        wl = W.tiny_fp32(seed=12, B=8, prefix=200, ext_lo=12800, ext_hi=13100, n_distract=0, Hq=8, Hkv=2, D=128,
                         num_slots=131072, page_size=16, dtype="bf16")
        assert wl.T * (wl.Hq // wl.Hkv) // 128 > 3072
    g, o = GpuSide(wl, gpu_device), OracleSide(wl)
    pl, si = g.match()
    out = g.extend(pl, si)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()
    pl_ref, si_ref = o.match()
    assert_match_equal(wl, pl, si, pl_ref, si_ref)
    rows = sample_rows(wl, 256, seed=3)
    ref = o.extend(pl_ref, si_ref, rows=rows)
    outn = out_to_f64(out)
    got = np.stack([outn[wl.ext_offsets[r] + i, h] for r, i, h in rows])
    err = np.abs(got - ref).max()
    say(f"  max abs err over {len(rows)} rows: {err:.3e}")
    assert err <= TOL[wl.dtype]


def test_full_config_append_then_reuse(pa, gpu_device, full_cache):
    """After append_kv the new tokens are cached: re-running a request whose whole prompt is now the prefix
    of a longer one gives the same attention rows for the old positions (prefix reuse is lossless, Sec. 5)."""
    wl = W.small_variant("agent_tree", 4)
    g, o = GpuSide(wl, gpu_device), OracleSide(wl)
    pl, si, out = g.step()
    # second turn: every request's prompt is now fully cached under new_slots; extend = last 7 tokens of the old extend
    P2 = (wl.designed_prefix_len + wl.ext_len - 7).astype(np.int32)
    E2 = np.full(wl.B, 7, np.int32)
    si2 = np.full_like(wl.tokens, -1)
    rows_q = []
    for r in range(wl.B):
        lo, e0, Pd, E = int(wl.offsets[r]), int(wl.ext_offsets[r]), int(wl.designed_prefix_len[r]), int(wl.ext_len[r])
        si2[lo:lo + Pd] = wl.designed_slots[lo:lo + Pd]
        si2[lo + Pd:lo + Pd + E - 7] = wl.new_slots[e0:e0 + E - 7]
        rows_q.append(np.arange(e0 + E - 7, e0 + E))
    rows_q = np.concatenate(rows_q)
    eo2 = np.arange(0, 7 * wl.B + 1, 7, dtype=np.int32)
    dev = gpu_device
    tt = lambda a: torch.from_numpy(a).to(dev)
    idx = tt(rows_q).long()
    out2 = g.pa.extend_attention(g.q[idx].contiguous(), g.k[idx].contiguous(), g.v[idx].contiguous(), g.pool, tt(si2),
                                 g.offsets, tt(P2), tt(E2), tt(eo2), wl.scale, max_kv_len=g.max_kv_len, **g.kw)
    torch.cuda.synchronize()
    ref = o.extend(*o.match())
    err = np.abs(out_to_f64(out2) - ref[rows_q]).max()
    say(f"  reuse max abs err {err:.3e}")
    assert err <= TOL[wl.dtype]


def test_chunked_prefill_through_the_cache_loop(pa, gpu_device):
    """Chunked prefill (Sec. 3.3: long non-shared prompts are chunked): the extend part of every request is
    prefilled 48 tokens at a time, and between chunks the new KV is appended to the pool and the tokens are inserted
    into the tree, so that chunk k finds cached prefix + chunks < k as its prefix.  Every round goes through
    match -> extend -> append -> insert/upload; matches are bit-exact, and the stitched output meets the same bar
    against the oracle's one-shot result (prefix reuse is lossless, Sec. 5)."""
    wl = W.small_variant("tool_use", 5)
    g, o = GpuSide(wl, gpu_device), OracleSide(wl)
    ref = o.extend(*o.match())  # [T, Hq, D] one shot
    dev, C = gpu_device, 48
    tt = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    out_all = torch.zeros_like(g.q)
    Pd, E, off, eo = wl.designed_prefix_len.astype(int), wl.ext_len.astype(int), wl.offsets.astype(int), wl.ext_offsets.astype(int)
    for k in range(int((E.max() + C - 1) // C)):
        live = [r for r in range(wl.B) if k * C < E[r]]
        done = [min(E[r], k * C) for r in live]          # extend tokens already cached
        upto = [min(E[r], (k + 1) * C) for r in live]    # ... after this round
        prompts = [wl.tokens[off[r]:off[r] + Pd[r] + u] for r, u in zip(live, upto)]
        toks = np.concatenate(prompts).astype(np.int32)
        offs = np.zeros(len(live) + 1, np.int32)
        offs[1:] = np.cumsum([len(p) for p in prompts])
        pl, si = pa.match_prefixes(g.tree, tt(toks), tt(offs))
        want_pl = np.array([Pd[r] + d for r, d in zip(live, done)], np.int32)
        np.testing.assert_array_equal(pl.cpu().numpy(), want_pl)
        sin = si.cpu().numpy()
        for j, (r, d) in enumerate(zip(live, done)):
            want = np.concatenate([wl.designed_slots[off[r]:off[r] + Pd[r]], wl.new_slots[eo[r]:eo[r] + d]])
            np.testing.assert_array_equal(sin[offs[j]:offs[j] + want_pl[j]], want)
        rows = np.concatenate([np.arange(eo[r] + d, eo[r] + u) for r, d, u in zip(live, done, upto)])
        idx = tt(rows).long()
        el = np.array([u - d for d, u in zip(done, upto)], np.int32)
        eo_k = np.zeros(len(live) + 1, np.int32)
        eo_k[1:] = np.cumsum(el)
        qk, kk, vk = g.q[idx].contiguous(), g.k[idx].contiguous(), g.v[idx].contiguous()
        out = pa.extend_attention(qk, kk, vk, g.pool, si, tt(offs), pl, tt(el), tt(eo_k), wl.scale,
                                  max_kv_len=int((offs[1:] - offs[:-1]).max()), **g.kw)
        out_all[idx] = out
        pa.append_kv(g.pool, tt(wl.new_slots[rows]), kk, vk, **g.kw)
        for r, u in zip(live, upto):
            g.tree.insert(wl.tokens[off[r]:off[r] + Pd[r] + u],
                          np.concatenate([wl.designed_slots[off[r]:off[r] + Pd[r]], wl.new_slots[eo[r]:eo[r] + u]]).astype(np.int32))
        g.tree.upload()
    torch.cuda.synchronize()
    err = np.abs(out_to_f64(out_all) - ref).max()
    say(f"  chunked prefill max abs err {err:.3e}")
    assert err <= TOL[wl.dtype]


def test_decode_shape_one_new_token(pa, gpu_device):
    """A fully cached prompt plus one new token per request (the decoding-phase unit of Sec. 3.2): E = 1 rows only."""
    import oracle
    rng = np.random.default_rng(77)
    Hq, Hkv, D, page, nslots, B = 32, 8, 128, 16, 131072, 33
    c = _random_case(rng, B, Hq, Hkv, D, 2500, 1, "bf16", page, nslots)
    dev = gpu_device
    pool = torch.zeros(pa.kv_pool_bytes(nslots, Hkv, D, torch.bfloat16, page), dtype=torch.uint8, device=dev)
    kw = dict(page_size=page, num_slots=nslots)
    pa.append_kv(pool, torch.from_numpy(c["backed"]).to(dev), to_torch(c["pk"], "bf16", dev), to_torch(c["pv"], "bf16", dev), **kw)
    tt = lambda a: torch.from_numpy(a).to(dev)
    scale = 1.0 / np.sqrt(D)
    out = pa.extend_attention(to_torch(c["q"], "bf16", dev), to_torch(c["k"], "bf16", dev), to_torch(c["v"], "bf16", dev), pool,
                              tt(c["si"]), tt(c["off"]), tt(c["P"]), tt(c["E"]), tt(c["eo"]), scale,
                              max_kv_len=int((c["P"] + c["E"]).max()), **kw)
    torch.cuda.synchronize()
    opk, opv = oracle.new_pool(nslots, Hkv, D, "bf16")
    oracle.append_kv(opk, opv, c["backed"], c["pk"], c["pv"], "bf16")
    ref = oracle.extend_attention(c["q"], c["k"], c["v"], opk, opv, c["si"], c["off"], c["P"], c["E"], c["eo"], scale, "bf16")
    err = np.abs(out_to_f64(out) - ref).max() if c["T"] else 0.0
    say(f"  decode shape: T = {c['T']}, max abs err {err:.3e}")
    assert c["T"] >= 8 and err <= TOL["bf16"]


@pytest.mark.parametrize("seed", [0, 1])
def test_uploads_that_copy_only_the_changes(pa, gpu_device, seed):
    """Many rounds of admissions (new leaves, splits), releases and evictions (shortened and deleted nodes) with an
    upload after each: the mirror that follows the changes piece by piece and a second tree that is re-flattened
    whole every time must both give the matcher what the per-token cache oracle says, for prompts along cached
    paths, cut anywhere, with fresh tails.  The numbers of either kind of upload are checked too."""
    from oracle.cache_oracle import CacheOracle
    rng = np.random.default_rng(900 + seed)
    page, nslots = 16, 16384
    dev = gpu_device
    trees = [pa.Tree(), pa.Tree()]
    trees[1].set_incremental_upload(False)
    co = CacheOracle(nslots, page)
    for t in trees:
        t.attach_pool(nslots, page)
    tt = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    history, live, now, evictions, matched = [], [], 0, 0, 0
    for rnd in range(60):
        for _ in range(int(rng.integers(1, 5))):
            if history and rng.random() < 0.75:
                base = history[int(rng.integers(len(history)))]
                head = base[:int(rng.integers(1, len(base) + 1))]
            else:
                head = np.zeros(0, np.int32)
            p = np.concatenate([head, rng.integers(0, 300, int(rng.integers(1, 400)))]).astype(np.int32)
            need = (len(p) + page - 1) // page * page
            if co.free_slots() < need:
                while len(live) > 2:
                    hs = live.pop(0)
                    for t, h in zip(trees, hs[:2]):
                        t.release(h)
                    co.release(hs[2])
                want = co.evict(need)
                for t in trees:
                    assert t.evict(need) == want
                evictions += 1
            now += 1
            ref = co.admit(list(p), now)
            if ref is None:
                now -= 1
                continue
            hs = []
            for t in trees:
                got = t.admit(p, now)
                assert got[0] == ref[0] and got[1].tolist() == ref[1]
                hs.append(got[2])
            live.append((hs[0], hs[1], ref[2]))
            history.append(p)
        # what the matcher sees after this round's upload
        prompts = []
        for _ in range(6):
            base = history[int(rng.integers(len(history)))]
            prompts.append(np.concatenate([base[:int(rng.integers(1, len(base) + 1))],
                                           rng.integers(0, 300, int(rng.integers(0, 40)))]).astype(np.int32))
        toks = np.concatenate(prompts)
        off = np.zeros(len(prompts) + 1, np.int32)
        off[1:] = np.cumsum([len(p) for p in prompts])
        want = [co.match(p) for p in prompts]
        for t in trees:
            t.upload()
            pl, si = pa.match_prefixes(t, tt(toks), tt(off))
            pln, sin = pl.cpu().numpy(), si.cpu().numpy()
            for j in range(len(prompts)):
                assert pln[j] == want[j][0], (rnd, j)
                assert list(sin[off[j]:off[j] + want[j][0]]) == want[j][1], (rnd, j)
                matched += want[j][0]
    full_a, incr_a, last_a = trees[0].upload_stats()
    full_b, incr_b, last_b = trees[1].upload_stats()
    say(f"  following the changes: {full_a} whole + {incr_a} partial uploads, last {last_a} B; "
        f"re-flattened: {full_b} whole, last {last_b} B; {evictions} evictions, {matched} tokens matched")
    assert incr_b == 0 and full_b == 60
    assert incr_a >= 40 and full_a >= 2        # the first one, and at least one after the flat form was outgrown
    assert last_a * 20 < last_b or full_a + incr_a == 60
    assert evictions >= 3


def test_cache_loop_with_eviction(pa, gpu_device):
    """Rounds of upload -> match (GPU) -> admit (host: pages for the new tokens, pins) -> extend -> append, with
    releases and LRU evictions in between, so that pages are reused and pool rows overwritten.  Every round the
    GPU match has to agree with what the admission finds cached and with the per-token cache oracle, and the
    attention output with the fp64 oracle on the oracle's own copy of the pool."""
    import oracle
    from oracle.cache_oracle import CacheOracle
    rng = np.random.default_rng(404)
    Hq, Hkv, D, page, nslots = 8, 2, 128, 16, 2048
    dev, tdt = gpu_device, torch.bfloat16
    tree, co = pa.Tree(), CacheOracle(nslots, page)
    tree.attach_pool(nslots, page)
    pool = torch.zeros(pa.kv_pool_bytes(nslots, Hkv, D, tdt, page), dtype=torch.uint8, device=dev)
    opk, opv = oracle.new_pool(nslots, Hkv, D, "bf16")
    kw = dict(page_size=page, num_slots=nslots)
    tt = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    history, live, now, worst, evictions = [], [], 0, 0.0, 0
    for rnd in range(14):
        # prompts: continuations of earlier prompts (cut anywhere) or fresh ones; new parts are random, so distinct
        prompts = []
        for _ in range(int(rng.integers(1, 4))):
            if history and rng.random() < 0.7:
                base = history[int(rng.integers(len(history)))]
                head = base[:int(rng.integers(1, len(base) + 1))]
            else:
                head = np.zeros(0, np.int32)
            prompts.append(np.concatenate([head, rng.integers(0, 50000, int(rng.integers(20, 300)))]).astype(np.int32))
        need = sum((len(p) + page - 1) // page * page for p in prompts)
        if tree.free_slots() < need:
            for _ in range(len(live) // 2 + 1):  # finish some requests, then make room by LRU
                if live:
                    hl, ho = live.pop(0)
                    tree.release(hl)
                    co.release(ho)
            assert tree.evict(need) == co.evict(need)
            evictions += 1
        # two requests of one batch must not share tokens that are not cached (any more): the second would find them
        # in the tree, put there by the first's admission, before their KV exists.  Such a request is dropped here.
        lcp = lambda a, b: int((np.cumprod(a[:min(len(a), len(b))] == b[:min(len(a), len(b))])).sum())
        kept = []
        for cand in prompts:
            if all(lcp(cand, q) <= co.match(cand)[0] for q in kept):
                kept.append(cand)
        prompts = kept
        tree.upload()
        toks = np.concatenate(prompts)
        off = np.zeros(len(prompts) + 1, np.int32)
        off[1:] = np.cumsum([len(p) for p in prompts])
        pl, si = pa.match_prefixes(tree, tt(toks), tt(off))
        pln, sin = pl.cpu().numpy(), si.cpu().numpy()
        el, new_slots = [], []
        want = [co.match(p) for p in prompts]  # before any of the batch is admitted
        for j, p in enumerate(prompts):
            want_n, want_slots = want[j]
            assert pln[j] == want_n and list(sin[off[j]:off[j] + want_n]) == want_slots
            now += 1
            got, ref = tree.admit(p, now), co.admit(list(p), now)
            assert ref is not None and got[0] == want_n == ref[0] and got[1].tolist() == ref[1]
            live.append((got[2], ref[2]))
            history.append(p)
            el.append(len(p) - want_n)
            new_slots.append(np.asarray(ref[1], np.int32))
        el = np.asarray(el, np.int32)
        eo = np.zeros(len(prompts) + 1, np.int32)
        eo[1:] = np.cumsum(el)
        T = int(eo[-1])
        ss = np.random.SeedSequence(rnd).spawn(3)
        mk = lambda s_, h: W._normal(s_, T * h * D, "bf16").reshape(T, h, D)
        q, k, v = mk(ss[0], Hq), mk(ss[1], Hkv), mk(ss[2], Hkv)
        scale = 1.0 / np.sqrt(D)
        out = pa.extend_attention(to_torch(q, "bf16", dev), to_torch(k, "bf16", dev), to_torch(v, "bf16", dev), pool, si, tt(off),
                                  pl, tt(el), tt(eo), scale, max_kv_len=int((off[1:] - off[:-1]).max()), **kw)
        ref_out = oracle.extend_attention(q, k, v, opk, opv, sin, off, pln, el, eo, scale, "bf16")
        worst = max(worst, float(np.abs(out_to_f64(out) - ref_out).max()))
        ns = np.concatenate(new_slots)
        pa.append_kv(pool, tt(ns), to_torch(k, "bf16", dev), to_torch(v, "bf16", dev), **kw)
        oracle.append_kv(opk, opv, ns, k, v, "bf16")
    say(f"  cache loop: {evictions} evictions, worst max abs err over the rounds {worst:.3e}")
    assert evictions >= 2 and worst <= TOL["bf16"]


@pytest.mark.gpu
def test_calibration_kernels(pa, gpu_device):
    """The two benchmark-support kernels: the copy copies, and the MFMA loop reports its work and a plausible clock."""
    say("calibration kernels")
    src = torch.randint(0, 256, (1 << 22,), dtype=torch.uint8, device=gpu_device)
    dst = torch.zeros_like(src)
    pa.calib_copy(dst, src)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)
    cal = torch.zeros(1 << 16, dtype=torch.uint8, device=gpu_device)
    flops = pa.calib_mfma(cal, 64)
    torch.cuda.synchronize()
    assert flops == 512 * 4 * 64 * 4 * 2 * 32 * 32 * 16
    cycles, ticks = cal[:16].view(torch.int64).tolist()
    assert cycles > 0 and ticks > 0 and 200.0 < 100.0 * cycles / ticks < 4000.0
    with pytest.raises(Exception):
        pa.calib_mfma(torch.zeros(64, dtype=torch.uint8, device=gpu_device), 64)  # output buffer too small
