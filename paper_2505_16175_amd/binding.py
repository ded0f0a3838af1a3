"""Thin ctypes binding of libqp_hip.so: argument marshalling only.

Every function has the name and argument order of its C-ABI counterpart in include/qp.h
and takes torch tensors on the GPU (device memory and streams are all torch is used for).
There is no CPU fallback: if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

from .build import LIB_PATH

QP_OK, QP_ERR_INVALID_ARG, QP_ERR_UNSUPPORTED, QP_ERR_CAPACITY, QP_ERR_HIP = range(5)
QP_F32, QP_BF16 = 0, 1
QP_SCORE_KEY_NORM_SMALL, QP_SCORE_VALUE_NORM, QP_SCORE_WINDOW_ATTN = 0, 1, 2
QP_ATTEND_AUTO, QP_ATTEND_SCALAR, QP_ATTEND_MFMA, QP_ATTEND_MFMA_DECODE = 0, 1, 2, 3
QP_SCORE_WINDOW_LOGIT, QP_SCORE_SHARED_HEADS = 3, 0x100
RULES = {"key_norm_small": QP_SCORE_KEY_NORM_SMALL, "value_norm": QP_SCORE_VALUE_NORM,
         "window_attn": QP_SCORE_WINDOW_ATTN, "window_logit": QP_SCORE_WINDOW_LOGIT}
RULES.update({name + "+shared": code | QP_SCORE_SHARED_HEADS for name, code in list(RULES.items())})
QP_MAX_GROUP_TOKENS = 32768


class qp_layout(ctypes.Structure):
    _fields_ = [("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("softmax_scale", ctypes.c_float)]


class qp_cache(ctypes.Structure):
    _fields_ = [("k", ctypes.c_void_p), ("v", ctypes.c_void_p), ("pos", ctypes.c_void_p),
                ("capacity", ctypes.c_int32), ("len", ctypes.c_int32)]


class qp_attend_plan_info(ctypes.Structure):
    _fields_ = [("kernel", ctypes.c_int32), ("workgroups", ctypes.c_int32), ("key_chunks", ctypes.c_int32),
                ("tiles_per_chunk", ctypes.c_int32), ("mirrored_rows", ctypes.c_int32),
                ("scratch_bytes", ctypes.c_size_t)]


class QPError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status}, hip error {last_hip_error()})")


_lib = None
_vp, _i32, _i64, _f64, _sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_double, ctypes.c_size_t
_LP, _CP = ctypes.POINTER(qp_layout), ctypes.POINTER(qp_cache)

SIGNATURES = {
    "qp_keep_count": (_i64, [_i64, _f64]),
    "qp_cache_capacity": (_i64, [_i32, _i32, _i32, _f64]),
    "qp_workspace_bytes": (_sz, [_LP, _i32, _i32]),
    "qp_group_attend": (_i32, [_LP, _vp, _vp, _vp, _i32, _CP, _vp, _vp, _vp, _sz, _vp]),
    "qp_score_kv": (_i32, [_LP, _i32, _vp, _vp, _i32, _vp, _i32, _vp, _vp, _sz, _vp]),
    "qp_topk_compact": (_i32, [_LP, _vp, _vp, _vp, _i32, _i32, _i32, _CP, _vp, _vp, _sz, _vp]),
    "qp_prefill_video": (_i32, [_LP, _i32, _i32, _i32, _f64, _i32, _vp, _vp, _vp, _vp, _i32, _CP, _vp, _vp, _sz, _vp]),
    "qp_attend_plan": (_i32, [_LP, _i32, _i32, _sz, ctypes.POINTER(qp_attend_plan_info)]),
    "qp_select_attend_kernel": (_i32, [_i32]),
    "qp_status_string": (ctypes.c_char_p, [_i32]),
    "qp_last_hip_error": (ctypes.c_int, []),
    "qp_version": (ctypes.c_char_p, []),
}


def lib():
    """The loaded C-ABI library; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2505_16175_amd.build` "
                               "(or __graft_entry__.build()); there is no CPU fallback")
        handle = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype, fn.argtypes = res, args
        _lib = handle
    return _lib


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous GPU tensor")
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(status, where):
    if status != QP_OK:
        raise QPError(status, where)


def make_layout(n_q_heads, n_kv_heads, head_dim, dtype, softmax_scale=0.0) -> qp_layout:
    code = {torch.float32: QP_F32, torch.bfloat16: QP_BF16, "f32": QP_F32, "bf16": QP_BF16}[dtype]
    return qp_layout(n_q_heads, n_kv_heads, head_dim, code, softmax_scale)


class Cache:
    """Owner of the device buffers behind a qp_cache (torch allocates; the library only fills)."""

    def __init__(self, layout: qp_layout, capacity: int, device="cuda"):
        dt = torch.float32 if layout.dtype == QP_F32 else torch.bfloat16
        self.k = torch.zeros(layout.n_kv_heads, capacity, layout.head_dim, dtype=dt, device=device)
        self.v = torch.zeros_like(self.k)
        self.pos = torch.full((layout.n_kv_heads, capacity), -1, dtype=torch.int32, device=device)
        self.c = qp_cache(self.k.data_ptr(), self.v.data_ptr(), self.pos.data_ptr(), capacity, 0)

    @property
    def len(self):
        return self.c.len

    def reset(self):
        self.c.len = 0

    def nbytes(self):
        """Bytes of K and V actually held (2 * H_kv * len * d * sizeof)."""
        return 2 * self.k.shape[0] * self.c.len * self.k.shape[2] * self.k.element_size()


def status_string(status) -> str:
    return lib().qp_status_string(int(status)).decode()


def last_hip_error() -> int:
    return lib().qp_last_hip_error()


def version() -> str:
    return lib().qp_version().decode()


def keep_count(n_group_tokens, retention) -> int:
    return lib().qp_keep_count(n_group_tokens, retention)


def cache_capacity(n_frames, tokens_per_frame, group_frames, retention) -> int:
    return lib().qp_cache_capacity(n_frames, tokens_per_frame, group_frames, retention)


def workspace_bytes(layout, max_group_tokens, n_window) -> int:
    return lib().qp_workspace_bytes(ctypes.byref(layout), max_group_tokens, n_window)


def make_workspace(layout, max_group_tokens, n_window, device="cuda") -> torch.Tensor:
    n = workspace_bytes(layout, max_group_tokens, n_window)
    if n == 0:
        raise QPError(QP_ERR_INVALID_ARG, "qp_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def attend_plan(layout, n_group_tokens, cache_len, workspace_bytes=0) -> dict:
    info = qp_attend_plan_info()
    _check(lib().qp_attend_plan(ctypes.byref(layout), n_group_tokens, cache_len, workspace_bytes, ctypes.byref(info)),
           "qp_attend_plan")
    return {name: getattr(info, name) for name, _ in qp_attend_plan_info._fields_}


def select_attend_kernel(which: int):
    _check(lib().qp_select_attend_kernel(which), "qp_select_attend_kernel")


def _ws(workspace):
    if workspace is None:
        return None, 0
    return _ptr(workspace), workspace.numel() * workspace.element_size()


def group_attend(layout, q_g, k_g, v_g, cache: Optional[Cache], out_g, lse=None, workspace=None):
    wp, wb = _ws(workspace)
    st = lib().qp_group_attend(ctypes.byref(layout), _ptr(q_g), _ptr(k_g), _ptr(v_g), q_g.shape[0],
                               ctypes.byref(cache.c) if cache is not None else None, _ptr(out_g), _ptr(lse),
                               wp, wb, _stream())
    _check(st, "qp_group_attend")


def score_kv(layout, rule, k_g, v_g, q_win, scores, workspace=None):
    wp, wb = _ws(workspace)
    n_g = (k_g if k_g is not None else v_g).shape[0]
    st = lib().qp_score_kv(ctypes.byref(layout), RULES.get(rule, rule), _ptr(k_g), _ptr(v_g), n_g, _ptr(q_win),
                           0 if q_win is None else q_win.shape[0], _ptr(scores), wp, wb, _stream())
    _check(st, "qp_score_kv")


def topk_compact(layout, scores, k_g, v_g, keep, group_token_base, cache: Cache, kept_idx=None, workspace=None):
    wp, wb = _ws(workspace)
    st = lib().qp_topk_compact(ctypes.byref(layout), _ptr(scores), _ptr(k_g), _ptr(v_g), k_g.shape[0], keep,
                               group_token_base, ctypes.byref(cache.c), _ptr(kept_idx), wp, wb, _stream())
    _check(st, "qp_topk_compact")


def prefill_video(layout, n_frames, tokens_per_frame, group_frames, retention, rule, q, k, v, q_win, cache: Cache,
                  out, workspace):
    wp, wb = _ws(workspace)
    st = lib().qp_prefill_video(ctypes.byref(layout), n_frames, tokens_per_frame, group_frames, retention,
                                RULES.get(rule, rule), _ptr(q), _ptr(k), _ptr(v), _ptr(q_win),
                                0 if q_win is None else q_win.shape[0], ctypes.byref(cache.c), _ptr(out), wp, wb,
                                _stream())
    _check(st, "qp_prefill_video")
