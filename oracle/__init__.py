"""ctypes front end of the CPU oracle (``prefix_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
benchmark's ``cpu_baseline`` leg.  The product package never imports it, and this
package never imports the product's HIP binding.  See the header of
``prefix_oracle.c`` for what each function computes and which passage of the paper
it follows.  Parity pins (brute-force longest common prefix, library causal
attention, split invariance, closed forms) live in ``tests/test_oracle_*.py``;
nothing here is "parity unpinned".
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "prefix_oracle.c")
_LIB = os.path.join(_HERE, "_prefix_oracle.so")

F32, BF16 = 0, 1
_DT = {"f32": F32, "bf16": BF16}


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (fp64 arithmetic, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c11", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.ora_trie_new.restype = C.c_void_p
        _lib.ora_trie_free.argtypes = [C.c_void_p]
        _lib.ora_trie_num_nodes.argtypes = [C.c_void_p]
        _lib.ora_trie_num_nodes.restype = C.c_int64
        _lib.ora_trie_insert.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64]
        _lib.ora_trie_insert.restype = C.c_int64
        _lib.ora_trie_match.argtypes = [C.c_void_p] * 3 + [C.c_int] + [C.c_void_p] * 2
        _lib.ora_fp8_rows.argtypes = [C.c_void_p, C.c_int64, C.c_int] + [C.c_void_p] * 3
        _lib.ora_append_kv.argtypes = [C.c_void_p] * 5 + [C.c_int64, C.c_int, C.c_int, C.c_int]
        _lib.ora_extend_attention.argtypes = [C.c_void_p] * 10 + [C.c_int] * 5 + [C.c_double, C.c_void_p]
        _lib.ora_extend_attention_rows.argtypes = ([C.c_void_p] * 9 + [C.c_int] * 4 + [C.c_double, C.c_void_p,
                                                                                       C.c_int64, C.c_void_p])
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _vals(a: np.ndarray, dtype: str) -> np.ndarray:
    want = np.float32 if dtype == "f32" else np.uint16
    assert a.dtype == want, (a.dtype, dtype)
    return np.ascontiguousarray(a)


class Trie:
    """One-token-per-node trie of the cached sequences (first insertion of a position keeps its slot)."""

    def __init__(self):
        self._h = lib().ora_trie_new()

    def __del__(self):
        if getattr(self, "_h", None):
            lib().ora_trie_free(self._h)
            self._h = None

    def insert(self, tokens, slots) -> int:
        t, s = _i32(tokens), _i32(slots)
        assert t.shape == s.shape and t.ndim == 1
        return int(lib().ora_trie_insert(self._h, _p(t), _p(s), len(t)))

    @property
    def num_nodes(self) -> int:
        return int(lib().ora_trie_num_nodes(self._h))

    def match(self, tokens, offsets):
        """-> (prefix_len int32 [B], slot_idx int32 [offsets[B]], -1 past the match)."""
        t, o = _i32(tokens), _i32(offsets)
        B = len(o) - 1
        pl = np.zeros(B, np.int32)
        si = np.full(int(o[-1]) if B >= 0 and len(o) else 0, -1, np.int32)
        lib().ora_trie_match(self._h, _p(t), _p(o), B, _p(pl), _p(si))
        return pl, si


def match_prefixes(cached, tokens, offsets):
    """cached: iterable of (tokens, slots) in insertion order."""
    tr = Trie()
    for tok, slot in cached:
        tr.insert(tok, slot)
    return tr.match(tokens, offsets)


def new_pool(num_slots: int, Hkv: int, D: int, dtype: str):
    """The oracle's own dense pool: K and V arrays [num_slots, Hkv, D], zero-filled."""
    dt = np.float32 if dtype == "f32" else np.uint16   # ('bf16_kv8': the values the fp8 form stores, as bfloat16)
    return np.zeros((num_slots, Hkv, D), dt), np.zeros((num_slots, Hkv, D), dt)


def fp8_rows(rows: np.ndarray):
    """rows: bfloat16 bit patterns [..., D] -> (codes uint8 like rows, exps int8 [...], stored bfloat16 bit patterns like
    rows): the fp8 form of KV rows (one power-of-two scale per row of D elements) and the values it stores."""
    r = _vals(rows, "bf16")
    D = r.shape[-1]
    n = r.size // D
    codes, exps, stored = np.zeros(r.shape, np.uint8), np.zeros(r.shape[:-1], np.int8), np.zeros(r.shape, np.uint16)
    lib().ora_fp8_rows(_p(r), n, D, _p(codes), _p(exps), _p(stored))
    return codes, exps, stored


def append_kv(pool_k, pool_v, new_slots, k_ext, v_ext, dtype: str):
    """dtype 'bf16_kv8': the pool holds the rows in their fp8 form; the oracle keeps the values that form stores (exactly
    bfloat16) in its bfloat16 pool, so that attention over the pool needs no other change."""
    s = _i32(new_slots)
    if dtype == "bf16_kv8":
        k_ext, v_ext, dtype = fp8_rows(k_ext)[2], fp8_rows(v_ext)[2], "bf16"
    k, v = _vals(k_ext, dtype), _vals(v_ext, dtype)
    T, Hkv, D = k.shape
    assert v.shape == k.shape and len(s) == T and pool_k.shape[1:] == (Hkv, D)
    assert pool_k.flags.c_contiguous and pool_v.flags.c_contiguous
    assert T == 0 or (s.min() >= 0 and s.max() < pool_k.shape[0])
    lib().ora_append_kv(_p(pool_k), _p(pool_v), _p(s), _p(k), _p(v), T, Hkv, D, _DT[dtype])


def extend_attention(q_ext, k_ext, v_ext, pool_k, pool_v, slot_idx, slot_offsets, prefix_len, ext_len,
                     ext_offsets, scale: float, dtype: str, rows=None) -> np.ndarray:
    """fp64 output [T, Hq, D]; with rows = int array [n,3] of (r, i, h): only those rows, [n, D]."""
    if dtype == "bf16_kv8":   # the pool given here already holds the values its fp8 form stores (see append_kv)
        dtype = "bf16"
    q, k, v = _vals(q_ext, dtype), _vals(k_ext, dtype), _vals(v_ext, dtype)
    T, Hq, D = q.shape
    Hkv = k.shape[1]
    si, so, pl, el, eo = map(_i32, (slot_idx, slot_offsets, prefix_len, ext_len, ext_offsets))
    B = len(pl)
    assert Hq % Hkv == 0 and k.shape == (T, Hkv, D) and v.shape == k.shape
    assert len(so) == B + 1 and len(eo) == B + 1 and int(eo[-1]) == T
    for r in range(B):
        assert so[r + 1] - so[r] >= pl[r] >= 0
        if pl[r]:
            seg = si[so[r]:so[r] + pl[r]]
            assert seg.min() >= 0 and seg.max() < pool_k.shape[0], "prefix slot outside the oracle pool"
    if rows is None:
        out = np.zeros((T, Hq, D), np.float64)
        lib().ora_extend_attention(_p(q), _p(k), _p(v), _p(pool_k), _p(pool_v), _p(si), _p(so), _p(pl), _p(el),
                                   _p(eo), B, Hq, Hkv, D, _DT[dtype], float(scale), _p(out))
        return out
    rw = _i32(rows).reshape(-1, 3)
    for r, i, h in rw:
        assert 0 <= r < B and 0 <= i < el[r] and 0 <= h < Hq
    out = np.zeros((len(rw), D), np.float64)
    lib().ora_extend_attention_rows(_p(q), _p(k), _p(v), _p(pool_k), _p(pool_v), _p(si), _p(so), _p(pl), _p(eo),
                                    Hq, Hkv, D, _DT[dtype], float(scale), _p(rw), len(rw), _p(out))
    return out
