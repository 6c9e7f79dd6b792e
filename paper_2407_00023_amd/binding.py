"""Thin ctypes binding of libprefixattn (argument marshalling only).

Every function below forwards to the C entry point of the same name (``pa_`` prefix
dropped); all computation happens in the HIP kernels of the library.  PyTorch supplies
device memory and the stream, nothing else.  There is no fallback: if the shared library
has not been built the import fails.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libprefixattn.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it first (python -m paper_2407_00023_amd.build, or __graft_entry__.build()). "
        "There is no CPU fallback.")

_lib = C.CDLL(LIB_PATH)

F32, BF16 = 0, 1
_DTYPES = {torch.float32: F32, torch.bfloat16: BF16}

_vp, _i, _i64, _sz, _f = C.c_void_p, C.c_int, C.c_int64, C.c_size_t, C.c_float
_SIGS = {
    "pa_last_error": (C.c_char_p, []),
    "pa_tree_create": (_i, [C.POINTER(_vp)]),
    "pa_tree_insert": (_i, [_vp, _vp, _vp, C.c_int32, C.POINTER(C.c_int32)]),
    "pa_tree_upload": (_i, [_vp, _vp]),
    "pa_tree_set_incremental_upload": (_i, [_vp, _i]),
    "pa_tree_upload_stats": (_i, [_vp, C.POINTER(_i64), C.POINTER(_i64), C.POINTER(_i64)]),
    "pa_tree_stats": (_i, [_vp, C.POINTER(_i64), C.POINTER(_i64)]),
    "pa_tree_destroy": (_i, [_vp]),
    "pa_tree_attach_pool": (_i, [_vp, _i64, _i]),
    "pa_tree_free_slots": (_i, [_vp, C.POINTER(_i64)]),
    "pa_tree_admit": (_i, [_vp, _vp, C.c_int32, _i64, _vp, C.POINTER(C.c_int32), C.POINTER(_i64)]),
    "pa_tree_release": (_i, [_vp, _i64]),
    "pa_tree_evict": (_i, [_vp, _i64, C.POINTER(_i64), C.POINTER(_i64)]),
    "pa_tree_set_hit_window": (_i, [_vp, _i64]),
    "pa_tree_evict_plan": (_i, [_vp, _i64, _i64, _i64, _vp, _vp, C.POINTER(_i64), C.POINTER(_i64)]),
    "pa_tree_evict_for": (_i, [_vp, _vp, C.c_int32, C.POINTER(_i64), C.POINTER(_i64)]),
    "pa_tree_evict_plan_for": (_i, [_vp, _vp, C.c_int32, _i64, _i64, _vp, _vp, C.POINTER(_i64), C.POINTER(_i64)]),
    "pa_priority_group": (_i, [C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_int32)]),
    "pa_priority_select": (_i, [_vp, _vp, _i64, C.c_int32, _i64, _vp, C.POINTER(_i64)]),
    "pa_e2_load_cost": (_i, [_vp, _vp, _i64, C.c_double, _vp, _vp, _i64, _i64, C.c_int32] + [C.POINTER(C.c_double)] * 3),
    "pa_e2_schedule": (_i, [C.c_int32, C.c_int32, _vp, _vp, _vp, C.c_double, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]),
    "pa_e2_longest_piece": (_i, [_vp, C.c_int32, _vp]),
    "pa_history_create": (_i, [C.c_int32, _i64, _vp, C.POINTER(_vp)]),
    "pa_history_destroy": (_i, [_vp]),
    "pa_history_assign": (_i, [_vp, C.c_int32, _i64, C.c_int32]),
    "pa_history_complete": (_i, [_vp, C.c_int32, _i64, C.c_int32]),
    "pa_history_gpu_load": (_i, [_vp, C.c_int32, _i64, C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(_i64), C.POINTER(C.c_double)]),
    "pa_kv_pool_bytes": (_sz, [_i64, _i, _i, _i, _i]),
    "pa_extend_workspace_bytes": (_sz, [_i, _i64, _i64, _i, _i, _i, _i]),
    "pa_match_prefixes": (_i, [_vp, _vp, _vp, _i, _vp, _vp, _vp]),
    "pa_extend_attention": (_i, [_vp] * 9 + [_i, _i64, _i64, _i, _i, _i, _i, _i64, _i, _f, _vp, _vp, _sz, _vp]),
    "pa_extend_attention_static": (_i, [_vp] * 9 + [_i, _i64, _i64, _i, _i, _i, _i, _i64, _i, _f, _vp, _vp]),
    "pa_extend_status": (_i, [_vp, _vp]),
    "pa_extend_set_row_sharing": (_i, [_i]),
    "pa_append_kv": (_i, [_vp, _vp, _vp, _vp, _i64, _i, _i, _i, _i64, _i, _vp]),
    "pa_gather_kv": (_i, [_vp, _vp, _i64, _i, _i, _i, _i64, _i, _vp, _vp, _vp]),
    "pa_profile_enable": (_i, [_i]),
    "pa_profile_read": (_i, [C.c_char_p, C.POINTER(C.c_double), C.POINTER(_i64)]),
    "pa_profile_clock": (_i, [_vp, _i, C.POINTER(C.c_double)]),
    "pa_calib_copy": (_i, [_vp, _vp, _sz, _vp]),
    "pa_calib_mfma": (_i, [_vp, _sz, _i, C.POINTER(_i64), _vp]),
}
for _name, (_res, _args) in _SIGS.items():
    _fn = getattr(_lib, _name)
    _fn.restype, _fn.argtypes = _res, _args

EXPORTED = tuple(_SIGS)


class PrefixAttnError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where} failed with code {code}: {_lib.pa_last_error().decode()}")


def _check(rc: int, where: str):
    if rc != 0:
        raise PrefixAttnError(rc, where)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream) -> C.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _dev_i32(t: torch.Tensor, name: str) -> torch.Tensor:
    if t.dtype != torch.int32 or not t.is_cuda or not t.is_contiguous():
        raise TypeError(f"{name} must be a contiguous int32 CUDA tensor")
    return t


class Tree:
    """Radix tree of cached sequences (pa_tree_*): host inserts, then upload() before matching."""

    def __init__(self):
        h = _vp()
        _check(_lib.pa_tree_create(C.byref(h)), "pa_tree_create")
        self._h = h

    def insert(self, tokens, slots) -> int:
        """tokens, slots: host int32 arrays (numpy or CPU tensors).  Returns how many leading tokens were cached."""
        t = torch.as_tensor(tokens, dtype=torch.int32).contiguous()
        s = torch.as_tensor(slots, dtype=torch.int32).contiguous()
        if t.is_cuda or s.is_cuda or t.shape != s.shape or t.dim() != 1:
            raise TypeError("tokens and slots must be host int32 vectors of equal length")
        already = C.c_int32(0)
        _check(_lib.pa_tree_insert(self._h, _ptr(t), _ptr(s), t.numel(), C.byref(already)), "pa_tree_insert")
        return int(already.value)

    def upload(self, stream=None):
        _check(_lib.pa_tree_upload(self._h, _stream(stream)), "pa_tree_upload")

    def set_incremental_upload(self, on: bool) -> None:
        _check(_lib.pa_tree_set_incremental_upload(self._h, 1 if on else 0), "pa_tree_set_incremental_upload")

    def upload_stats(self):
        """-> (uploads that copied everything, uploads that copied only the changes, bytes of the last one)."""
        a, b, c = _i64(0), _i64(0), _i64(0)
        _check(_lib.pa_tree_upload_stats(self._h, C.byref(a), C.byref(b), C.byref(c)), "pa_tree_upload_stats")
        return int(a.value), int(b.value), int(c.value)

    # ---- cache bookkeeping on the host (pa_tree_attach_pool / admit / release / evict) ----
    def attach_pool(self, num_slots: int, page_size: int) -> None:
        _check(_lib.pa_tree_attach_pool(self._h, num_slots, page_size), "pa_tree_attach_pool")

    def free_slots(self) -> int:
        n = _i64(0)
        _check(_lib.pa_tree_free_slots(self._h, C.byref(n)), "pa_tree_free_slots")
        return int(n.value)

    def admit(self, tokens, now: int):
        """-> (n_cached, new_slots int32 tensor of the tokens that were not cached, handle)."""
        t = torch.as_tensor(tokens, dtype=torch.int32).contiguous()
        if t.is_cuda or t.dim() != 1:
            raise TypeError("tokens must be a host int32 vector")
        slots = torch.full_like(t, -1)
        cached, handle = C.c_int32(0), _i64(0)
        _check(_lib.pa_tree_admit(self._h, _ptr(t), t.numel(), now, _ptr(slots), C.byref(cached), C.byref(handle)), "pa_tree_admit")
        return int(cached.value), slots[int(cached.value):].clone(), int(handle.value)

    def release(self, handle: int) -> None:
        _check(_lib.pa_tree_release(self._h, handle), "pa_tree_release")

    def evict(self, need_slots: int):
        """-> (slots in pages that became free, tokens dropped)."""
        freed, gone = _i64(0), _i64(0)
        _check(_lib.pa_tree_evict(self._h, need_slots, C.byref(freed), C.byref(gone)), "pa_tree_evict")
        return int(freed.value), int(gone.value)

    def set_hit_window(self, window: int) -> None:
        _check(_lib.pa_tree_set_hit_window(self._h, window), "pa_tree_set_hit_window")

    def evict_plan(self, need_slots: int, since: int, cap: int = 4096):
        """-> (tokens each victim node would lose, admissions after `since` through each, admissions after `since`)."""
        toks = torch.zeros(cap, dtype=torch.int32)
        shr = torch.zeros(cap, dtype=torch.int32)
        n, nreq = _i64(0), _i64(0)
        _check(_lib.pa_tree_evict_plan(self._h, need_slots, since, cap, _ptr(toks), _ptr(shr), C.byref(n), C.byref(nreq)),
               "pa_tree_evict_plan")
        k = int(n.value)
        return toks[:k].clone(), shr[:k].clone(), int(nreq.value)

    def evict_for(self, tokens):
        """Make room for this prompt without touching its cached part -> (slots freed, tokens dropped)."""
        t = _host_i32(tokens)
        freed, gone = _i64(0), _i64(0)
        _check(_lib.pa_tree_evict_for(self._h, _ptr(t), t.numel(), C.byref(freed), C.byref(gone)), "pa_tree_evict_for")
        return int(freed.value), int(gone.value)

    def evict_plan_for(self, tokens, since: int, cap: int = 4096):
        """What evict_for(tokens) would drop -> (tokens per node, sharers per node, admissions after `since`)."""
        t = _host_i32(tokens)
        toks = torch.zeros(cap, dtype=torch.int32)
        shr = torch.zeros(cap, dtype=torch.int32)
        n, nreq = _i64(0), _i64(0)
        _check(_lib.pa_tree_evict_plan_for(self._h, _ptr(t), t.numel(), since, cap, _ptr(toks), _ptr(shr), C.byref(n),
                                           C.byref(nreq)), "pa_tree_evict_plan_for")
        k = int(n.value)
        return toks[:k].clone(), shr[:k].clone(), int(nreq.value)

    def stats(self) -> Tuple[int, int]:
        a, b = _i64(0), _i64(0)
        _check(_lib.pa_tree_stats(self._h, C.byref(a), C.byref(b)), "pa_tree_stats")
        return int(a.value), int(b.value)

    def close(self):
        if getattr(self, "_h", None) and _lib is not None:  # (module globals may be gone at interpreter exit)
            _lib.pa_tree_destroy(self._h)
            self._h = None

    __del__ = close


EXPLOIT, EXPLORE_DECODE, EXPLORE_COST = 0, 1, 2


class CostModel(C.Structure):
    """pa_cost_model: PrefillTime(n) = prefill_per_token * n + prefill_base (n > 0), DecodeTime likewise."""
    _fields_ = [("prefill_per_token", C.c_double), ("prefill_base", C.c_double), ("decode_per_token", C.c_double),
                ("decode_base", C.c_double), ("default_output_len", C.c_double)]


def _host_i32(x) -> torch.Tensor:
    t = torch.as_tensor(x, dtype=torch.int32).contiguous()
    if t.is_cuda or t.dim() != 1:
        raise TypeError("expected a host int32 vector")
    return t


def priority_group(cached_len: int, prompt_len: int, P: int) -> int:
    g = C.c_int32(0)
    _check(_lib.pa_priority_group(cached_len, prompt_len, P, C.byref(g)), "pa_priority_group")
    return int(g.value)


def priority_select(cached_len, prompt_len, P: int, n_pick: int) -> torch.Tensor:
    """-> queue indices of the next batch (int32 host tensor), higher groups first."""
    c, n = _host_i32(cached_len), _host_i32(prompt_len)
    if c.numel() != n.numel():
        raise ValueError("cached_len and prompt_len differ in length")
    picked = torch.zeros(max(0, min(n_pick, c.numel())), dtype=torch.int32)
    k = _i64(0)
    _check(_lib.pa_priority_select(_ptr(c), _ptr(n), c.numel(), P, n_pick, _ptr(picked), C.byref(k)), "pa_priority_select")
    return picked[:int(k.value)]


def e2_load_cost(model: CostModel, hist_missed_len, avg_output_len: float, evict_tokens, evict_sharers,
                 n_requests: int, missed_len_k: int) -> Tuple[float, float, float]:
    """-> (L, M, P) of Algorithm 2."""
    h, et, es = _host_i32(hist_missed_len), _host_i32(evict_tokens), _host_i32(evict_sharers)
    if et.numel() != es.numel():
        raise ValueError("evict_tokens and evict_sharers differ in length")
    L, M, P = C.c_double(0), C.c_double(0), C.c_double(0)
    _check(_lib.pa_e2_load_cost(C.byref(model), _ptr(h), h.numel(), avg_output_len, _ptr(et), _ptr(es), et.numel(),
                                n_requests, missed_len_k, C.byref(L), C.byref(M), C.byref(P)), "pa_e2_load_cost")
    return float(L.value), float(M.value), float(P.value)


def e2_schedule(prompt_len: int, cached_len: int, on_longest_node, cost, decode_ratio, imbal_r: float) -> Tuple[int, int]:
    """-> (gpu, mode) of Algorithm 1."""
    f = torch.as_tensor(on_longest_node).to(torch.uint8).contiguous()
    c = torch.as_tensor(cost, dtype=torch.float64).contiguous()
    r = torch.as_tensor(decode_ratio, dtype=torch.float64).contiguous()
    if not (f.numel() == c.numel() == r.numel()):
        raise ValueError("per-GPU arrays differ in length")
    gpu, mode = C.c_int32(-1), C.c_int32(-1)
    _check(_lib.pa_e2_schedule(prompt_len, cached_len, _ptr(f), _ptr(c), _ptr(r), imbal_r, c.numel(), C.byref(gpu),
                               C.byref(mode)), "pa_e2_schedule")
    return int(gpu.value), int(mode.value)


def e2_longest_piece(cached_len) -> torch.Tensor:
    """-> flags (uint8 host tensor): the GPUs that cache the longest piece of the matched path."""
    c = _host_i32(cached_len)
    flags = torch.zeros(c.numel(), dtype=torch.uint8)
    _check(_lib.pa_e2_longest_piece(_ptr(c), c.numel(), _ptr(flags)), "pa_e2_longest_piece")
    return flags


class History:
    """Owner of a pa_history handle (per-GPU request history over the window H)."""

    def __init__(self, n_gpus: int, window: int, model: CostModel):
        h = C.c_void_p()
        _check(_lib.pa_history_create(n_gpus, window, C.byref(model), C.byref(h)), "pa_history_create")
        self._h = h

    def assign(self, gpu: int, now: int, missed_len: int) -> None:
        _check(_lib.pa_history_assign(self._h, gpu, now, missed_len), "pa_history_assign")

    def complete(self, gpu: int, now: int, output_len: int) -> None:
        _check(_lib.pa_history_complete(self._h, gpu, now, output_len), "pa_history_complete")

    def gpu_load(self, gpu: int, now: int) -> Tuple[float, float, int, float]:
        """-> (L, decode ratio, requests in the window, average output length)."""
        L, r, n, a = C.c_double(0), C.c_double(0), _i64(0), C.c_double(0)
        _check(_lib.pa_history_gpu_load(self._h, gpu, now, C.byref(L), C.byref(r), C.byref(n), C.byref(a)), "pa_history_gpu_load")
        return float(L.value), float(r.value), int(n.value), float(a.value)

    def close(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.pa_history_destroy(self._h)
            self._h = None

    __del__ = close


def _code(dtype: torch.dtype, kv8: bool) -> int:
    """The library's dtype value; kv8 = bf16 tensors with the KV pool in its fp8 form (PA_BF16_KV8)."""
    if kv8:
        if dtype != torch.bfloat16:
            raise TypeError("the fp8 KV pool goes with bfloat16 tensors")
        return 2
    return _DTYPES[dtype]


def kv_pool_bytes(num_slots: int, Hkv: int, D: int, dtype: torch.dtype, page_size: int, kv8: bool = False) -> int:
    n = int(_lib.pa_kv_pool_bytes(num_slots, Hkv, D, _code(dtype, kv8), page_size))
    if n == 0:
        raise ValueError("pa_kv_pool_bytes: invalid arguments")
    return n


def extend_workspace_bytes(B: int, T: int, max_kv_len: int, Hq: int, Hkv: int, D: int, dtype: torch.dtype) -> int:
    n = int(_lib.pa_extend_workspace_bytes(B, T, max_kv_len, Hq, Hkv, D, _DTYPES[dtype]))
    if n == 0:
        raise ValueError("pa_extend_workspace_bytes: invalid arguments")
    return n


def match_prefixes(tree: Tree, tokens: torch.Tensor, offsets: torch.Tensor, prefix_len: Optional[torch.Tensor] = None,
                   slot_idx: Optional[torch.Tensor] = None, stream=None):
    """-> (prefix_len int32 [B], slot_idx int32 like tokens).  Asynchronous on the stream."""
    _dev_i32(tokens, "tokens"), _dev_i32(offsets, "offsets")
    B = offsets.numel() - 1
    if prefix_len is None:
        prefix_len = torch.empty(B, dtype=torch.int32, device=tokens.device)
    if slot_idx is None:
        slot_idx = torch.empty_like(tokens)
    _dev_i32(prefix_len, "prefix_len"), _dev_i32(slot_idx, "slot_idx")
    if prefix_len.numel() < B or slot_idx.numel() < tokens.numel():
        raise ValueError("output tensors too small")
    _check(_lib.pa_match_prefixes(tree._h, _ptr(tokens), _ptr(offsets), B, _ptr(prefix_len), _ptr(slot_idx),
                                  _stream(stream)), "pa_match_prefixes")
    return prefix_len, slot_idx


def extend_attention(q_ext: torch.Tensor, k_ext: torch.Tensor, v_ext: torch.Tensor, kv_pool: torch.Tensor,
                     slot_idx: torch.Tensor, slot_offsets: torch.Tensor, prefix_len: torch.Tensor,
                     ext_len: torch.Tensor, ext_offsets: torch.Tensor, scale: float, *, page_size: int,
                     num_slots: int, max_kv_len: int, out: Optional[torch.Tensor] = None,
                     workspace: Optional[torch.Tensor] = None, stream=None, kv8: bool = False) -> torch.Tensor:
    """q_ext [T,Hq,D], k_ext/v_ext [T,Hkv,D] -> out [T,Hq,D].  Asynchronous on the stream."""
    T, Hq, D = q_ext.shape
    Hkv = k_ext.shape[1]
    dt = _code(q_ext.dtype, kv8)
    for name, t in (("q_ext", q_ext), ("k_ext", k_ext), ("v_ext", v_ext)):
        if not (t.is_cuda and t.is_contiguous() and t.dtype == q_ext.dtype):
            raise TypeError(f"{name} must be a contiguous CUDA tensor of dtype {q_ext.dtype}")
    if k_ext.shape != (T, Hkv, D) or v_ext.shape != k_ext.shape:
        raise ValueError("k_ext / v_ext shape mismatch")
    for name, t in (("slot_idx", slot_idx), ("slot_offsets", slot_offsets), ("prefix_len", prefix_len),
                    ("ext_len", ext_len), ("ext_offsets", ext_offsets)):
        _dev_i32(t, name)
    B = prefix_len.numel()
    if slot_offsets.numel() != B + 1 or ext_offsets.numel() != B + 1 or ext_len.numel() != B:
        raise ValueError("per-request arrays disagree on B")
    if kv_pool.numel() * kv_pool.element_size() < kv_pool_bytes(num_slots, Hkv, D, q_ext.dtype, page_size, kv8):
        raise ValueError("kv_pool smaller than pa_kv_pool_bytes")
    if out is None:
        out = torch.empty_like(q_ext)
    elif out.shape != q_ext.shape or out.dtype != q_ext.dtype or not out.is_contiguous() or not out.is_cuda:
        raise ValueError("bad out tensor")
    need = extend_workspace_bytes(B, T, max_kv_len, Hq, Hkv, D, q_ext.dtype)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=q_ext.device)
    wbytes = workspace.numel() * workspace.element_size()
    _check(_lib.pa_extend_attention(_ptr(q_ext), _ptr(k_ext), _ptr(v_ext), _ptr(kv_pool), _ptr(slot_idx),
                                    _ptr(slot_offsets), _ptr(prefix_len), _ptr(ext_len), _ptr(ext_offsets), B, T,
                                    max_kv_len, Hq, Hkv, D, page_size, num_slots, dt, float(scale), _ptr(out),
                                    _ptr(workspace), wbytes, _stream(stream)), "pa_extend_attention")
    return out


def extend_attention_static(q_ext: torch.Tensor, k_ext: torch.Tensor, v_ext: torch.Tensor, kv_pool: torch.Tensor,
                            slot_idx: torch.Tensor, slot_offsets: torch.Tensor, prefix_len: torch.Tensor,
                            ext_len: torch.Tensor, ext_offsets: torch.Tensor, scale: float, *, page_size: int,
                            num_slots: int, max_kv_len: int, out: torch.Tensor, stream=None, kv8: bool = False) -> torch.Tensor:
    """pa_extend_attention_static: as extend_attention, with the library's own scratch buffer as workspace; `out` is
    the caller's (nothing is allocated here either)."""
    T, Hq, D = q_ext.shape
    Hkv = k_ext.shape[1]
    B = prefix_len.numel()
    _check(_lib.pa_extend_attention_static(_ptr(q_ext), _ptr(k_ext), _ptr(v_ext), _ptr(kv_pool), _ptr(slot_idx),
                                           _ptr(slot_offsets), _ptr(prefix_len), _ptr(ext_len), _ptr(ext_offsets), B, T,
                                           max_kv_len, Hq, Hkv, D, page_size, num_slots, _code(q_ext.dtype, kv8), float(scale),
                                           _ptr(out), _stream(stream)), "pa_extend_attention_static")
    return out


def extend_status(workspace: torch.Tensor, stream=None) -> None:
    """Waits for the stream; raises PrefixAttnError (code -5) if the last bf16 extend_attention launch that used
    `workspace` was given a T or max_kv_len too small for the batch on the device (it then wrote no output)."""
    _check(_lib.pa_extend_status(_ptr(workspace), _stream(stream)), "pa_extend_status")


def extend_set_row_sharing(on: bool) -> None:
    """Process-wide: False gives every request row tiles of its own (for slot lists that do not come from one prefix tree)."""
    _check(_lib.pa_extend_set_row_sharing(1 if on else 0), "pa_extend_set_row_sharing")


def append_kv(kv_pool: torch.Tensor, new_slots: torch.Tensor, k_ext: torch.Tensor, v_ext: torch.Tensor, *,
              page_size: int, num_slots: int, stream=None, kv8: bool = False) -> None:
    T, Hkv, D = k_ext.shape
    _dev_i32(new_slots, "new_slots")
    if new_slots.numel() != T or v_ext.shape != k_ext.shape or v_ext.dtype != k_ext.dtype:
        raise ValueError("append_kv: shape mismatch")
    if not (k_ext.is_cuda and v_ext.is_cuda and k_ext.is_contiguous() and v_ext.is_contiguous()):
        raise TypeError("k_ext / v_ext must be contiguous CUDA tensors")
    if kv_pool.numel() * kv_pool.element_size() < kv_pool_bytes(num_slots, Hkv, D, k_ext.dtype, page_size, kv8):
        raise ValueError("kv_pool smaller than pa_kv_pool_bytes")
    _check(_lib.pa_append_kv(_ptr(kv_pool), _ptr(new_slots), _ptr(k_ext), _ptr(v_ext), T, Hkv, D, page_size,
                             num_slots, _code(k_ext.dtype, kv8), _stream(stream)), "pa_append_kv")


def gather_kv(kv_pool: torch.Tensor, slots: torch.Tensor, *, Hkv: int, D: int, dtype: torch.dtype, page_size: int,
              num_slots: int, stream=None, kv8: bool = False):
    """Test/debug helper: dense (k, v) [n, Hkv, D] of the given slots."""
    _dev_i32(slots, "slots")
    n = slots.numel()
    k = torch.empty((n, Hkv, D), dtype=dtype, device=slots.device)
    v = torch.empty_like(k)
    _check(_lib.pa_gather_kv(_ptr(kv_pool), _ptr(slots), n, Hkv, D, page_size, num_slots, _code(dtype, kv8), _ptr(k),
                             _ptr(v), _stream(stream)), "pa_gather_kv")
    return k, v


def profile_enable(on: bool, clock_probe: bool = False) -> None:
    _check(_lib.pa_profile_enable((2 if clock_probe else 1) if on else 0), "pa_profile_enable")


def profile_clock(workspace: torch.Tensor, reset: bool = False) -> float:
    """Shader clock in MHz seen by the bf16 extend-attention launches that used `workspace` while the clock probe was on."""
    mhz = C.c_double(0.0)
    _check(_lib.pa_profile_clock(_ptr(workspace), 1 if reset else 0, C.byref(mhz)), "pa_profile_clock")
    return float(mhz.value)


def calib_copy(dst: torch.Tensor, src: torch.Tensor, stream=None) -> None:
    """dst = src by the library's plain streaming-copy kernel (uint8 tensors of equal size).  Asynchronous."""
    assert dst.dtype == torch.uint8 and src.dtype == torch.uint8 and dst.numel() == src.numel()
    _check(_lib.pa_calib_copy(_ptr(dst), _ptr(src), dst.numel(), _stream(stream)), "pa_calib_copy")


def calib_mfma(out: torch.Tensor, iters: int, stream=None) -> int:
    """One launch of the MFMA-only loop; -> its flops.  out: uint8 device tensor of >= 16,400 bytes whose first two
    int64 receive (shader cycles, 100 MHz ticks) of one wave's loop.  Asynchronous."""
    flops = _i64(0)
    _check(_lib.pa_calib_mfma(_ptr(out), out.numel() * out.element_size(), int(iters), C.byref(flops), _stream(stream)),
           "pa_calib_mfma")
    return int(flops.value)


def profile_read(kernel: str) -> Tuple[float, int]:
    """-> (summed device time in ms, launches) of one library kernel since profile_enable(True)."""
    ms, n = C.c_double(0.0), _i64(0)
    _check(_lib.pa_profile_read(kernel.encode(), C.byref(ms), C.byref(n)), "pa_profile_read")
    return float(ms.value), int(n.value)
