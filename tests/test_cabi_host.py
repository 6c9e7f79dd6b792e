"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header declares,
and its host-side logic (radix-tree inserts, size queries, argument errors) behaves.
No kernel is launched here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def pa():
    from paper_2407_00023_amd import binding
    return binding


def test_every_declared_symbol_is_exported(pa):
    header = open(os.path.join(ROOT, "include", "prefixattn.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(pa_[a-z0-9_]+)\s*\(", header))
    assert {"pa_match_prefixes", "pa_extend_attention", "pa_append_kv"} <= declared
    lib = C.CDLL(pa.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(pa.EXPORTED)


def lcp(a, b):
    n = min(len(a), len(b))
    k = 0
    while k < n and a[k] == b[k]:
        k += 1
    return k


def test_insert_reports_longest_cached_prefix(pa):
    """n_already_cached must equal the longest common prefix with anything inserted before (Sec. 3.2 insert rule)."""
    rng = np.random.default_rng(0)
    for vocab in (2, 3, 50):
        tree = pa.Tree()
        seen, ntok = [], 0
        for _ in range(200):
            n = int(rng.integers(0, 14))
            seq = rng.integers(0, vocab, n).astype(np.int32)
            want = max([lcp(seq, s) for s in seen], default=0)
            got = tree.insert(seq, np.arange(n, dtype=np.int32))
            assert got == want
            ntok += n - want
            seen.append(seq)
            assert tree.stats()[1] == ntok
        tree.close()


def test_split_keeps_node_count_minimal(pa):
    tree = pa.Tree()
    tree.insert(np.array([1, 2, 3, 4], np.int32), np.arange(4, dtype=np.int32))
    assert tree.stats() == (2, 4)                       # root + one leaf
    tree.insert(np.array([1, 2, 9], np.int32), np.arange(3, dtype=np.int32))
    assert tree.stats() == (4, 5)                       # [1 2] -> {[3 4], [9]}
    tree.insert(np.array([1, 2], np.int32), np.arange(2, dtype=np.int32))
    assert tree.stats() == (4, 5)                       # ends on a node boundary: nothing new
    tree.insert(np.array([1], np.int32), np.arange(1, dtype=np.int32))
    assert tree.stats() == (4, 5)                       # ends inside an edge: no split needed to store nothing
    tree.insert(np.array([7], np.int32), np.arange(1, dtype=np.int32))
    assert tree.stats() == (5, 6)                       # nothing matched: new child of the virtual root


def test_size_queries_and_errors(pa):
    import torch
    assert pa.kv_pool_bytes(512, 2, 64, torch.float32, 1) == 512 * 2 * 2 * 64 * 4
    assert pa.kv_pool_bytes(262144, 8, 128, torch.bfloat16, 16) == 262144 * 2 * 8 * 128 * 2
    with pytest.raises(ValueError):
        pa.kv_pool_bytes(100, 8, 128, torch.bfloat16, 16)          # page size does not divide
    small = pa.extend_workspace_bytes(64, 6400, 2550, 32, 8, 128, torch.bfloat16)
    split = pa.extend_workspace_bytes(16, 800, 16464, 32, 8, 128, torch.bfloat16)
    tiny = pa.extend_workspace_bytes(4, 100, 128, 8, 2, 64, torch.bfloat16)
    # partial results of split row tiles dominate: bounded by the work-list rule at serving sizes, by the number of
    # 1,024-key pieces at small ones
    assert 0 < tiny < 4 << 20 and tiny < small <= 512 << 20 and 0 < split <= 512 << 20
    with pytest.raises(ValueError):
        pa.extend_workspace_bytes(1, 1, 1, 32, 5, 128, torch.bfloat16)  # Hq not a multiple of Hkv
    lib = C.CDLL(pa.LIB_PATH)
    lib.pa_last_error.restype = C.c_char_p
    # matching against a tree that was never uploaded is a state error, raised before any GPU call
    tree = pa.Tree()
    tree.insert(np.array([1], np.int32), np.array([0], np.int32))
    lib.pa_match_prefixes.argtypes = [C.c_void_p] * 3 + [C.c_int] + [C.c_void_p] * 3
    rc = lib.pa_match_prefixes(tree._h, None, None, 1, None, None, None)
    assert rc == -3 and b"upload" in lib.pa_last_error()
    lib.pa_append_kv.argtypes = [C.c_void_p] * 4 + [C.c_int64, C.c_int, C.c_int, C.c_int, C.c_int64, C.c_int, C.c_void_p]
    assert lib.pa_append_kv(None, None, None, None, 4, 8, 100, 16, 64, 1, None) == -1   # D unsupported
    assert lib.pa_append_kv(None, None, None, None, 0, 8, 128, 16, 64, 1, None) == 0    # empty append is a no-op
    # the calibration kernels refuse bad arguments before any GPU call
    lib.pa_calib_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    assert lib.pa_calib_copy(None, None, 1024, None) == -1
    lib.pa_calib_mfma.argtypes = [C.c_void_p, C.c_size_t, C.c_int, C.POINTER(C.c_int64), C.c_void_p]
    assert lib.pa_calib_mfma(None, 1 << 16, 16, None, None) == -1


def test_status_and_switch_calls_check_their_arguments(pa):
    """The two support calls beside pa_extend_attention refuse bad arguments before any GPU call, and pool sizes
    accept page sizes that are not powers of two."""
    import torch
    lib = C.CDLL(pa.LIB_PATH)
    lib.pa_extend_status.argtypes = [C.c_void_p, C.c_void_p]
    assert lib.pa_extend_status(None, None) == -1
    assert lib.pa_extend_set_row_sharing(0) == 0 and lib.pa_extend_set_row_sharing(1) == 0
    assert pa.kv_pool_bytes(36864, 4, 128, torch.bfloat16, 12) == 36864 * 2 * 4 * 128 * 2
    assert pa.kv_pool_bytes(36864, 4, 128, torch.bfloat16, 48) == 36864 * 2 * 4 * 128 * 2
    # the fp8 pool: one byte per element and one exponent byte per row; it goes with bf16 tensors only
    assert pa.kv_pool_bytes(4096, 8, 128, torch.bfloat16, 16, kv8=True) == 4096 * 2 * 8 * 129
    assert pa.kv_pool_bytes(4096, 2, 64, torch.bfloat16, 16, kv8=True) == 4096 * 2 * 2 * 65
    with pytest.raises(TypeError):
        pa.kv_pool_bytes(4096, 8, 128, torch.float32, 16, kv8=True)
    lib.pa_kv_pool_bytes.restype = C.c_size_t
    lib.pa_kv_pool_bytes.argtypes = [C.c_int64, C.c_int, C.c_int, C.c_int, C.c_int]
    assert lib.pa_kv_pool_bytes(4096, 8, 128, 3, 16) == 0       # no such dtype
    assert pa.extend_workspace_bytes(16, 800, 16464, 32, 8, 128, torch.bfloat16) == lib_ws(lib, 16, 800, 16464, 32, 8, 128, 2)


def lib_ws(lib, B, T, kv, Hq, Hkv, D, dtype):
    lib.pa_extend_workspace_bytes.restype = C.c_size_t
    lib.pa_extend_workspace_bytes.argtypes = [C.c_int, C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_int, C.c_int]
    return lib.pa_extend_workspace_bytes(B, T, kv, Hq, Hkv, D, dtype)
