"""Thin ctypes binding of libqp_hip.so: argument marshalling only.

Every function has the name and argument order of its C-ABI counterpart in include/qp.h
(the path) or include/qp_layer.h (the decoder layer around it) and takes torch tensors on the GPU (device memory and streams are all torch is used for).
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
                ("capacity", ctypes.c_int32), ("len", ctypes.c_int32), ("format", ctypes.c_int32)]


QP_CACHE_SAME, QP_CACHE_FP8_E4M3 = 0, 1


class qp_attend_plan_info(ctypes.Structure):
    _fields_ = [("kernel", ctypes.c_int32), ("workgroups", ctypes.c_int32), ("key_chunks", ctypes.c_int32),
                ("tiles_per_chunk", ctypes.c_int32), ("mirrored_rows", ctypes.c_int32),
                ("scratch_bytes", ctypes.c_size_t), ("split_row_blocks", ctypes.c_int32)]


class qp_layer_shape(ctypes.Structure):
    _fields_ = [("d_model", ctypes.c_int32), ("d_ff", ctypes.c_int32), ("rms_eps", ctypes.c_float),
                ("rope_theta", ctypes.c_float), ("mrope_section", ctypes.c_int32 * 3)]


class qp_layer_weights(ctypes.Structure):
    _fields_ = [(name, ctypes.c_void_p) for name in
                ("ln1_w", "w_qkv", "b_qkv", "w_o", "ln2_w", "w_gate_up", "w_down")]


class qp_feed_stats(ctypes.Structure):
    _fields_ = [("groups", ctypes.c_int32), ("total_ms", ctypes.c_double), ("waited_ms", ctypes.c_double),
                ("first_group_wait_ms", ctypes.c_double)]


# qp_group_fn of include/qp_feed.h: (user, group, device_input, bytes, hip_stream) -> qp_status
GROUP_FN = ctypes.CFUNCTYPE(ctypes.c_int32, ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_size_t,
                            ctypes.c_void_p)
QP_FEED_PAGEABLE, QP_FEED_END, QP_FEED_TIMEOUT = 1, 100, 101


class qp_linear_plan_info(ctypes.Structure):
    _fields_ = [("token_rows_per_tile", ctypes.c_int32), ("workgroups", ctypes.c_int32), ("k_chunks", ctypes.c_int32),
                ("k_steps_per_chunk", ctypes.c_int32), ("scratch_bytes", ctypes.c_size_t)]


class QPError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status}, hip error {last_hip_error()})")


_lib = None
_vp, _i32, _i64, _f64, _sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_double, ctypes.c_size_t
_LP, _CP = ctypes.POINTER(qp_layout), ctypes.POINTER(qp_cache)
_SP, _WP, _f32 = ctypes.POINTER(qp_layer_shape), ctypes.POINTER(qp_layer_weights), ctypes.c_float

SIGNATURES = {
    "qp_keep_count": (_i64, [_i64, _f64]),
    "qp_cache_capacity": (_i64, [_i32, _i32, _i32, _f64]),
    "qp_debug_fail_after": (_i32, [_i32]),
    "qp_e4m3_from_bf16": (ctypes.c_uint8, [ctypes.c_uint16]),
    "qp_bf16_from_e4m3": (ctypes.c_uint16, [ctypes.c_uint8]),
    "qp_group_attend_noalloc": (_i32, [_LP, _vp, _vp, _vp, _i32, _CP, _vp, _vp, _vp]),
    "qp_group_bounds": (_i32, [_i32, _i32, _i32, ctypes.POINTER(_i32), ctypes.POINTER(_i32), _i32]),
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
    # include/qp_layer.h
    "qp_rms_norm": (_i32, [_vp, _vp, _vp, _i32, _i32, _f32, _vp]),
    "qp_linear": (_i32, [_vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _vp, _sz, _vp]),
    "qp_rope_table": (_i32, [_vp, _i64, _i32, _f32, ctypes.POINTER(ctypes.c_int32), _vp, _vp]),
    "qp_qkv_rope": (_i32, [_LP, _vp, _vp, _vp, _vp, _i32, _i32, _vp, _vp, _vp, _vp, _sz, _vp]),
    "qp_swiglu_gate_up": (_i32, [_vp, _vp, _vp, _i32, _i32, _i32, _vp]),
    "qp_select_linear_tile": (_i32, [_i32]),
    "qp_linear_plan": (_i32, [_i32, _i32, _i32, _sz, ctypes.POINTER(qp_linear_plan_info)]),
    "qp_layer_workspace_bytes": (_sz, [_LP, _SP, _i32, _i32]),
    "qp_layer_group": (_i32, [_LP, _SP, _WP, _vp, _vp, _i64, _i32, _i32, _vp, _i32, _i32, _i32, _CP, _vp, _vp, _vp,
                              _sz, _vp]),
    "qp_layer_window_queries": (_i32, [_LP, _SP, _WP, _vp, _vp, _i64, _i32, _vp, _vp, _sz, _vp]),
    # include/qp_feed.h
    "qp_feed_create": (_i32, [_i32, _sz, _i32, ctypes.POINTER(_vp)]),
    "qp_feed_destroy": (None, [_vp]),
    "qp_feed_stop": (_i32, [_vp]),
    "qp_feed_begin_write": (_i32, [_vp, ctypes.POINTER(_vp)]),
    "qp_feed_publish": (_i32, [_vp, _sz]),
    "qp_feed_close": (_i32, [_vp]),
    "qp_feed_next": (_i32, [_vp, _i32, ctypes.POINTER(_vp), ctypes.POINTER(_sz), ctypes.POINTER(_i32)]),
    "qp_feed_release": (_i32, [_vp, _i32]),
    "qp_feed_consume": (_i32, [_vp, _vp, _vp, _sz, GROUP_FN, _vp, _vp, ctypes.POINTER(qp_feed_stats)]),
    "qp_feed_stub_producer": (_i32, [_vp, _vp, ctypes.POINTER(_sz), _i32, _i64, _i64]),
    "qp_feed_stub_join": (_i32, [_vp, ctypes.POINTER(_f64)]),
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

    def __init__(self, layout: qp_layout, capacity: int, device="cuda", fmt=QP_CACHE_SAME):
        """fmt = QP_CACHE_FP8_E4M3: K~ and V~ hold one E4M3 byte per element (torch.float8_e4m3fn is that format)."""
        dt = torch.float32 if layout.dtype == QP_F32 else torch.bfloat16
        if fmt == QP_CACHE_FP8_E4M3:
            dt = torch.float8_e4m3fn
        self.k = torch.zeros(layout.n_kv_heads, capacity, layout.head_dim, dtype=dt, device=device)
        self.v = torch.zeros_like(self.k)
        self.pos = torch.full((layout.n_kv_heads, capacity), -1, dtype=torch.int32, device=device)
        self.c = qp_cache(self.k.data_ptr(), self.v.data_ptr(), self.pos.data_ptr(), capacity, 0, fmt)

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


def group_bounds(n_frames, tokens_per_frame, group_frames):
    """[(first_token, n_tokens)] of every frame-aligned group, from qp_group_bounds."""
    n = lib().qp_group_bounds(n_frames, tokens_per_frame, group_frames, None, None, 0)
    if n < 0:
        raise QPError(QP_ERR_INVALID_ARG, "qp_group_bounds")
    first, count = (ctypes.c_int32 * n)(), (ctypes.c_int32 * n)()
    lib().qp_group_bounds(n_frames, tokens_per_frame, group_frames, first, count, n)
    return [(int(f), int(c)) for f, c in zip(first, count)]


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


NOALLOC_SCRATCH_BYTES = 8 << 20
NOALLOC_MAX_ROWS = 2048


def group_attend_noalloc(layout, q_g, k_g, v_g, cache: Optional[Cache], out_g, lse=None):
    st = lib().qp_group_attend_noalloc(ctypes.byref(layout), _ptr(q_g), _ptr(k_g), _ptr(v_g), q_g.shape[0],
                                       ctypes.byref(cache.c) if cache is not None else None, _ptr(out_g), _ptr(lse),
                                       _stream())
    _check(st, "qp_group_attend_noalloc")


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


# ---- include/qp_layer.h: the decoder layer around the path -------------------------------------------------
def make_layer_shape(d_model, d_ff, rms_eps=1e-6, rope_theta=1e6, mrope_section=(16, 24, 24)) -> qp_layer_shape:
    return qp_layer_shape(d_model, d_ff, rms_eps, rope_theta, (ctypes.c_int32 * 3)(*mrope_section))


class LayerWeights:
    """Keeps a layer's weight tensors alive next to the qp_layer_weights struct that points at them."""

    def __init__(self, ln1_w, w_qkv, b_qkv, w_o, ln2_w, w_gate_up, w_down):
        self.tensors = dict(ln1_w=ln1_w, w_qkv=w_qkv, b_qkv=b_qkv, w_o=w_o, ln2_w=ln2_w, w_gate_up=w_gate_up,
                            w_down=w_down)
        self.c = qp_layer_weights(**{name: _ptr(t).value for name, t in self.tensors.items()})


def rms_norm(x, w, out, eps):
    _check(lib().qp_rms_norm(_ptr(x), _ptr(w), _ptr(out), x.shape[0], x.shape[1], eps, _stream()), "qp_rms_norm")


def linear(x, w, bias, residual, out, workspace=None):
    wp, wb = _ws(workspace)
    _check(lib().qp_linear(_ptr(x), _ptr(w), _ptr(bias), _ptr(residual), _ptr(out), x.shape[0], w.shape[0], x.shape[1],
                           wp, wb, _stream()), "qp_linear")


def _pos_ptr(pos, first, axis_stride):
    """pos: int32 [3][N] on the GPU; the group starts at token `first`."""
    if pos.dtype != torch.int32 or not pos.is_cuda or not pos.is_contiguous() or pos.shape[0] != 3:
        raise ValueError("expected a contiguous int32 [3][N] GPU tensor of position indices")
    return ctypes.c_void_p(pos.data_ptr() + 4 * first), (pos.shape[1] if axis_stride is None else axis_stride)


def rope_table(pos, first, n_tokens, theta, mrope_section, cos_sin):
    pp, stride = _pos_ptr(pos, first, None)
    _check(lib().qp_rope_table(pp, stride, n_tokens, theta, (ctypes.c_int32 * 3)(*mrope_section), _ptr(cos_sin),
                               _stream()), "qp_rope_table")


def qkv_rope(layout, h, w_qkv, b_qkv, cos_sin, q, k, v, workspace=None):
    wp, wb = _ws(workspace)
    _check(lib().qp_qkv_rope(ctypes.byref(layout), _ptr(h), _ptr(w_qkv), _ptr(b_qkv), _ptr(cos_sin), h.shape[0],
                             h.shape[1], _ptr(q), _ptr(k), _ptr(v), wp, wb, _stream()), "qp_qkv_rope")


def swiglu_gate_up(h, w_gate_up, act):
    _check(lib().qp_swiglu_gate_up(_ptr(h), _ptr(w_gate_up), _ptr(act), h.shape[0], h.shape[1],
                                   w_gate_up.shape[0] // 2, _stream()), "qp_swiglu_gate_up")


def linear_plan(m, n, k, workspace_bytes=0) -> dict:
    info = qp_linear_plan_info()
    _check(lib().qp_linear_plan(m, n, k, workspace_bytes, ctypes.byref(info)), "qp_linear_plan")
    return {name: getattr(info, name) for name, _ in qp_linear_plan_info._fields_}


def select_linear_tile(token_rows: int):
    _check(lib().qp_select_linear_tile(token_rows), "qp_select_linear_tile")


def layer_workspace_bytes(layout, shape, max_group_tokens, n_window) -> int:
    return lib().qp_layer_workspace_bytes(ctypes.byref(layout), ctypes.byref(shape), max_group_tokens, n_window)


def make_layer_workspace(layout, shape, max_group_tokens, n_window, device="cuda") -> torch.Tensor:
    n = layer_workspace_bytes(layout, shape, max_group_tokens, n_window)
    if n == 0:
        raise QPError(QP_ERR_INVALID_ARG, "qp_layer_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def layer_group(layout, shape, weights: LayerWeights, x_g, pos, first, group_token_base, q_win, rule, keep,
                cache: Cache, x_out, kept_idx, workspace):
    wp, wb = _ws(workspace)
    pp, stride = _pos_ptr(pos, first, None)
    st = lib().qp_layer_group(ctypes.byref(layout), ctypes.byref(shape), ctypes.byref(weights.c), _ptr(x_g), pp, stride,
                              x_g.shape[0], group_token_base, _ptr(q_win), 0 if q_win is None else q_win.shape[0],
                              RULES.get(rule, rule), keep, ctypes.byref(cache.c), _ptr(x_out), _ptr(kept_idx), wp, wb,
                              _stream())
    _check(st, "qp_layer_group")


def layer_window_queries(layout, shape, weights: LayerWeights, x_win, pos_win, q_win_out, workspace):
    wp, wb = _ws(workspace)
    pp, stride = _pos_ptr(pos_win, 0, None)
    st = lib().qp_layer_window_queries(ctypes.byref(layout), ctypes.byref(shape), ctypes.byref(weights.c), _ptr(x_win),
                                       pp, stride, x_win.shape[0], _ptr(q_win_out), wp, wb, _stream())
    _check(st, "qp_layer_window_queries")


# ---- include/qp_feed.h: the consumer side of the loader / prefill pipeline ----------------------------------
class Feed:
    """Owner of a qp_feed handle. Producer calls may come from any Python thread (ctypes drops the GIL while a
    call blocks); consume() runs the consumer loop on the calling thread."""

    def __init__(self, n_slots, slot_bytes, flags=0):
        self.h = ctypes.c_void_p()
        _check(lib().qp_feed_create(n_slots, slot_bytes, flags, ctypes.byref(self.h)), "qp_feed_create")
        self.slot_bytes = slot_bytes
        self._keep = []

    def destroy(self):
        if self.h:
            lib().qp_feed_destroy(self.h)
            self.h = ctypes.c_void_p()

    def begin_write(self) -> int:
        p = ctypes.c_void_p()
        _check(lib().qp_feed_begin_write(self.h, ctypes.byref(p)), "qp_feed_begin_write")
        return p.value

    def publish(self, nbytes):
        _check(lib().qp_feed_publish(self.h, nbytes), "qp_feed_publish")

    def close(self):
        _check(lib().qp_feed_close(self.h), "qp_feed_close")

    def stop(self):
        _check(lib().qp_feed_stop(self.h), "qp_feed_stop")

    def next(self, timeout_ms=-1):
        """(status, host_pointer, bytes, group); status is QP_OK, QP_FEED_END or QP_FEED_TIMEOUT."""
        p, n, g = ctypes.c_void_p(), ctypes.c_size_t(), ctypes.c_int32()
        st = lib().qp_feed_next(self.h, timeout_ms, ctypes.byref(p), ctypes.byref(n), ctypes.byref(g))
        if st not in (QP_OK, QP_FEED_END, QP_FEED_TIMEOUT):
            raise QPError(st, "qp_feed_next")
        return st, p.value, n.value, g.value

    def release(self, group):
        _check(lib().qp_feed_release(self.h, group), "qp_feed_release")

    def consume(self, buf0, buf1, group_fn) -> dict:
        """group_fn(group, device_pointer, nbytes) enqueues the group's work on torch's current stream."""
        failure = []

        def tramp(_user, group, dev, nbytes, _stream):
            # an exception cannot cross the C frames of qp_feed_consume: stop the run and re-raise it afterwards
            try:
                group_fn(group, dev, nbytes)
                return QP_OK
            except QPError as e:
                failure.append(e)
                return e.status
            except BaseException as e:  # noqa: BLE001
                failure.append(e)
                return QP_ERR_INVALID_ARG
        cb = GROUP_FN(tramp)
        stats = qp_feed_stats()
        st = lib().qp_feed_consume(self.h, _ptr(buf0), _ptr(buf1), buf0.numel() * buf0.element_size(), cb, None,
                                   _stream(), ctypes.byref(stats))
        if failure:
            raise failure[0]
        _check(st, "qp_feed_consume")
        return {name: getattr(stats, name) for name, _ in qp_feed_stats._fields_}

    def stub_producer(self, host_src: torch.Tensor, bytes_per_group, first_latency_us, per_group_latency_us):
        """host_src: contiguous CPU tensor holding the groups back to back."""
        arr = (ctypes.c_size_t * len(bytes_per_group))(*bytes_per_group)
        self._keep = [host_src, arr]
        _check(lib().qp_feed_stub_producer(self.h, ctypes.c_void_p(host_src.data_ptr()), arr, len(bytes_per_group),
                                           first_latency_us, per_group_latency_us), "qp_feed_stub_producer")

    def stub_join(self) -> float:
        ms = ctypes.c_double()
        _check(lib().qp_feed_stub_join(self.h, ctypes.byref(ms)), "qp_feed_stub_join")
        return ms.value
