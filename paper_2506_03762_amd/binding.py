"""Thin ctypes binding of libaha.so: argument marshalling only.

Every step of the eviction path runs in the HIP kernels behind the C ABI of
``include/aha.h``; the functions here take torch tensors (device memory owned
by the caller), pass their pointers and the current HIP stream, and raise
``AhaError`` on a non-zero status.  There is no fallback: if the library has
not been built, loading fails loudly.
"""
from __future__ import annotations

import ctypes
import math
import os
from dataclasses import dataclass
from typing import Optional

import torch  # must be imported before libaha.so so that both share one HIP runtime

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libaha.so")

AHA_OK = 0
AHA_ERR_INVALID_ARG = -1
AHA_ERR_UNSUPPORTED = -2
AHA_ERR_WORKSPACE = -3
AHA_ERR_HIP = -4
AHA_F32, AHA_BF16 = 0, 1
AHA_SCALE_FIXED, AHA_SCALE_ADAPTIVE = 0, 1

# entry points returning an int32 status first, then the two that return strings
EXPORTS = ("aha_workspace_bytes", "aha_prefill_scores", "aha_prefill_scores_lse",
           "aha_prefill_scores_rows",
           "aha_prefill_row_stats", "aha_window_attention_workspace_bytes",
           "aha_prefill_window_attention", "aha_select_topk",
           "aha_compact_kv", "aha_decode_step", "aha_decode_step_static", "aha_profile_events",
           "aha_last_error",
           "aha_version")


class AhaError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__("aha error %d: %s" % (code, msg))
        self.code = code


class aha_params(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("seq_len", ctypes.c_int32), ("window", ctypes.c_int32),
        ("budget", ctypes.c_int32), ("recent", ctypes.c_int32), ("dtype", ctypes.c_int32),
        ("scale_mode", ctypes.c_int32), ("fixed_scale", ctypes.c_float),
        ("lambda_floor", ctypes.c_float), ("value_prior", ctypes.c_int32),
        ("pool_kernel", ctypes.c_int32),
        ("q_stride", ctypes.c_int64 * 3), ("k_stride", ctypes.c_int64 * 3),
        ("v_stride", ctypes.c_int64 * 3),
        ("score_pool", ctypes.c_int32), ("sink", ctypes.c_int32),
        ("decode_value_prior", ctypes.c_int32), ("reserved", ctypes.c_int32),
    ]


_lib = None


def load() -> ctypes.CDLL:
    """Load libaha.so (built in-tree by ``build.py``); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            "libaha.so is not built: run `python -m paper_2506_03762_amd.build` "
            "(or __graft_entry__.build()); there is no fallback path")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    pp = ctypes.POINTER(aha_params)
    lib.aha_workspace_bytes.argtypes = [pp, ctypes.POINTER(sz)]
    lib.aha_prefill_scores.argtypes = [pp, vp, vp, vp, vp, vp, sz, vp]
    lib.aha_prefill_scores_lse.argtypes = [pp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.aha_prefill_scores_rows.argtypes = [pp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.aha_prefill_row_stats.argtypes = [pp, vp, vp, vp, vp, vp, sz, vp]
    lib.aha_window_attention_workspace_bytes.argtypes = [pp, ctypes.POINTER(sz)]
    lib.aha_prefill_window_attention.argtypes = [pp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.aha_select_topk.argtypes = [pp, vp, vp, vp, sz, vp]
    lib.aha_compact_kv.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp]
    lib.aha_decode_step.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, vp, vp, sz, vp]
    lib.aha_decode_step_static.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, vp, vp]
    lib.aha_profile_events.argtypes = [ctypes.POINTER(vp), i32]
    for name in EXPORTS[:-2]:
        getattr(lib, name).restype = i32
    lib.aha_last_error.restype = ctypes.c_char_p
    lib.aha_version.restype = ctypes.c_char_p
    _lib = lib
    return lib


def _check(rc: int):
    if rc != AHA_OK:
        raise AhaError(rc, load().aha_last_error().decode())


def version() -> str:
    return load().aha_version().decode()


@dataclass
class Params:
    """Python mirror of ``aha_params`` (see include/aha.h for the meaning)."""
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    seq_len: int
    window: int
    budget: int
    recent: int
    dtype: int = AHA_BF16
    scale_mode: int = AHA_SCALE_ADAPTIVE
    fixed_scale: float = 0.0
    lambda_floor: float = -1.0
    value_prior: int = 1
    pool_kernel: int = 7
    q_stride: tuple = (0, 0, 0)
    k_stride: tuple = (0, 0, 0)
    v_stride: tuple = (0, 0, 0)
    score_pool: int = 0
    sink: int = 0
    decode_value_prior: int = 0

    def c(self) -> aha_params:
        """The C struct (built once per distinct set of field values: calls in a loop reuse it)."""
        key = (self.batch, self.n_q_heads, self.n_kv_heads, self.head_dim, self.seq_len,
               self.window, self.budget, self.recent, self.dtype, self.scale_mode,
               self.fixed_scale, self.lambda_floor, self.value_prior, self.pool_kernel,
               tuple(self.q_stride), tuple(self.k_stride), tuple(self.v_stride), self.score_pool,
               self.sink, self.decode_value_prior)
        cached = self.__dict__.get("_c")
        if cached is not None and cached[0] == key:
            return aha_params.from_buffer_copy(cached[1])   # a copy: callers may edit theirs
        p = aha_params()
        for f in ("batch", "n_q_heads", "n_kv_heads", "head_dim", "seq_len", "window", "budget",
                  "recent", "dtype", "scale_mode", "value_prior", "pool_kernel", "score_pool",
                  "sink", "decode_value_prior"):
            setattr(p, f, int(getattr(self, f)))
        p.fixed_scale = float(self.fixed_scale)
        p.lambda_floor = float(self.lambda_floor)
        p.q_stride = (ctypes.c_int64 * 3)(*self.q_stride)
        p.k_stride = (ctypes.c_int64 * 3)(*self.k_stride)
        p.v_stride = (ctypes.c_int64 * 3)(*self.v_stride)
        self.__dict__["_c"] = (key, bytes(p))
        return p

    def with_strides(self, q: torch.Tensor, k: torch.Tensor, v: torch.Tensor) -> "Params":
        """Strides (batch, head, token) of [b, h, n, d] views; the d axis must be contiguous."""
        for t in (q, k, v):
            assert t.dim() == 4 and t.stride(3) == 1
        from dataclasses import replace
        return replace(self, q_stride=tuple(q.stride()[:3]), k_stride=tuple(k.stride()[:3]),
                       v_stride=tuple(v.stride()[:3]))


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def torch_dtype(dtype: int):
    return torch.bfloat16 if dtype == AHA_BF16 else torch.float32


def workspace_bytes(p: Params) -> int:
    out = ctypes.c_size_t(0)
    _check(load().aha_workspace_bytes(ctypes.byref(p.c()), ctypes.byref(out)))
    return out.value


def alloc_workspace(p: Params, device="cuda") -> torch.Tensor:
    return torch.empty(max(workspace_bytes(p), 256), dtype=torch.uint8, device=device)


def aha_prefill_scores(p: Params, q, k, v, scores, workspace):
    """scores[b, Hkv, n] (fp32) <- refined eviction scores of q, k, v ([b, h, n, d] views)."""
    cp = p.c()
    _check(load().aha_prefill_scores(ctypes.byref(cp), _ptr(q), _ptr(k), _ptr(v), _ptr(scores),
                                     _ptr(workspace), workspace.numel() if workspace is not None else 0,
                                     _stream()))


def aha_prefill_scores_lse(p: Params, q, k, v, lse, scores, workspace):
    """As aha_prefill_scores, with the rows' natural-log softmax denominators lse[b, Hq, window]
    (fp32) given, e.g. by the attention forward pass: the row-statistics pass is skipped."""
    cp = p.c()
    _check(load().aha_prefill_scores_lse(ctypes.byref(cp), _ptr(q), _ptr(k), _ptr(v), _ptr(lse),
                                         _ptr(scores), _ptr(workspace),
                                         workspace.numel() if workspace is not None else 0,
                                         _stream()))


def aha_prefill_scores_rows(p: Params, q, k, v, rows, scores, workspace):
    """As aha_prefill_scores, accumulated over the query rows at positions rows[b, Hq, window]
    (int32) instead of the most recent ones."""
    cp = p.c()
    _check(load().aha_prefill_scores_rows(ctypes.byref(cp), _ptr(q), _ptr(k), _ptr(v), _ptr(rows),
                                          _ptr(scores), _ptr(workspace),
                                          workspace.numel() if workspace is not None else 0,
                                          _stream()))


def window_attention_workspace_bytes(p: Params) -> int:
    out = ctypes.c_size_t(0)
    _check(load().aha_window_attention_workspace_bytes(ctypes.byref(p.c()), ctypes.byref(out)))
    return out.value


def aha_prefill_window_attention(p: Params, q, k, v, out, lse, workspace):
    """out [b, Hq, window, d] <- causal attention output (standard scale) of the observed rows;
    lse [b, Hq, window] fp32 (or None) <- their natural-log softmax denominators."""
    cp = p.c()
    _check(load().aha_prefill_window_attention(ctypes.byref(cp), _ptr(q), _ptr(k), _ptr(v),
                                               _ptr(out), _ptr(lse), _ptr(workspace),
                                               workspace.numel() if workspace is not None else 0,
                                               _stream()))


def aha_prefill_row_stats(p: Params, q, k, lse, entropy, workspace):
    """lse / entropy [b, Hq, window] (fp32, either may be None) <- natural-log normaliser and
    entropy (nats) of the observed softmax rows."""
    cp = p.c()
    _check(load().aha_prefill_row_stats(ctypes.byref(cp), _ptr(q), _ptr(k), _ptr(lse),
                                        _ptr(entropy), _ptr(workspace),
                                        workspace.numel() if workspace is not None else 0,
                                        _stream()))


def aha_select_topk(p: Params, scores, idx, workspace=None):
    """idx[b, Hkv, budget] (int32) <- ascending retained token positions."""
    cp = p.c()
    _check(load().aha_select_topk(ctypes.byref(cp), _ptr(scores), _ptr(idx), _ptr(workspace),
                                  workspace.numel() if workspace is not None else 0, _stream()))


def aha_compact_kv(p: Params, k, v, scores, idx, k_cache, v_cache, scores_c, pos_c, free_slot):
    cp = p.c()
    _check(load().aha_compact_kv(ctypes.byref(cp), _ptr(k), _ptr(v), _ptr(scores), _ptr(idx),
                                 _ptr(k_cache), _ptr(v_cache), _ptr(scores_c), _ptr(pos_c),
                                 _ptr(free_slot), int(k_cache.shape[2]), _stream()))


def aha_decode_step(p: Params, q_new, k_new, v_new, k_cache, v_cache, scores_c, pos_c, free_slot,
                    logical_pos: int, out, workspace=None):
    cp = p.c()
    _check(load().aha_decode_step(ctypes.byref(cp), _ptr(q_new), _ptr(k_new), _ptr(v_new),
                                  _ptr(k_cache), _ptr(v_cache), _ptr(scores_c), _ptr(pos_c),
                                  _ptr(free_slot), int(k_cache.shape[2]), int(logical_pos),
                                  _ptr(out), _ptr(workspace),
                                  workspace.numel() if workspace is not None else 0, _stream()))


def aha_decode_step_static(p: Params, q_new, k_new, v_new, k_cache, v_cache, scores_c, pos_c,
                           free_slot, logical_pos: int, out):
    """aha_decode_step on the library's built-in scratch buffer (allocates nothing)."""
    cp = p.c()
    _check(load().aha_decode_step_static(ctypes.byref(cp), _ptr(q_new), _ptr(k_new), _ptr(v_new),
                                         _ptr(k_cache), _ptr(v_cache), _ptr(scores_c),
                                         _ptr(pos_c), _ptr(free_slot), int(k_cache.shape[2]),
                                         int(logical_pos), _ptr(out), _stream()))


def profile_events(events=None):
    """Stage events for aha_prefill_scores: four recorded torch.cuda.Event objects
    (enable_timing=True) or None to switch the hook off."""
    if events is None:
        _check(load().aha_profile_events(None, 0))
        return
    arr = (ctypes.c_void_p * 4)(*[ctypes.c_void_p(e.cuda_event) for e in events])
    _check(load().aha_profile_events(arr, 4))


@dataclass
class CompactCache:
    """Caller-owned device buffers of the compact cache of one layer."""
    k: torch.Tensor          # [b, Hkv, slots, d]
    v: torch.Tensor          # [b, Hkv, slots, d]
    scores: torch.Tensor     # [b, Hkv, slots] fp32
    pos: torch.Tensor        # [b, Hkv, slots] int32
    free_slot: torch.Tensor  # [b, Hkv] int32

    @staticmethod
    def empty(p: Params, slots: Optional[int] = None, device="cuda") -> "CompactCache":
        slots = p.budget + 1 if slots is None else slots
        dt = torch_dtype(p.dtype)
        shp = (p.batch, p.n_kv_heads, slots)
        return CompactCache(
            torch.empty(shp + (p.head_dim,), dtype=dt, device=device),
            torch.empty(shp + (p.head_dim,), dtype=dt, device=device),
            torch.empty(shp, dtype=torch.float32, device=device),
            torch.empty(shp, dtype=torch.int32, device=device),
            torch.empty(shp[:2], dtype=torch.int32, device=device))


def default_fixed_scale(head_dim: int) -> float:
    return 1.0 / math.sqrt(head_dim)
