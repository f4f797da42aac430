"""Thin ctypes binding over libcrope.so: argument marshalling only.

Every function has the name and argument order of its C declaration in include/crope.h.
Tensors are torch tensors used purely as device-memory handles (data_ptr, strides); all
arithmetic happens in the HIP kernels.  There is no CPU fallback: if the library cannot be
loaded, the call raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional, Sequence, Tuple

HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(HERE, "libcrope.so")
_lib = None


class CropeError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__("crope error %d: %s" % (code, message))
        self.code = code
        self.message = message


class _Desc(ctypes.Structure):
    _fields_ = [("head_dim", ctypes.c_int32), ("dim_t", ctypes.c_int32), ("dim_h", ctypes.c_int32),
                ("dim_w", ctypes.c_int32), ("theta", ctypes.c_double), ("max_t", ctypes.c_int32),
                ("max_h", ctypes.c_int32), ("max_w", ctypes.c_int32)]


class _Strides(ctypes.Structure):
    _fields_ = [("token", ctypes.c_int64), ("head", ctypes.c_int64)]


class _Segment(ctypes.Structure):
    _fields_ = [("start", ctypes.c_int64), ("len", ctypes.c_int64)]


class _Plan(ctypes.Structure):
    _fields_ = [("waves", ctypes.c_int32), ("splits", ctypes.c_int32)]


@dataclass(frozen=True)
class TableDesc:
    """Mirror of crope_table_desc."""
    head_dim: int = 128
    dim_t: int = 44
    dim_h: int = 42
    dim_w: int = 42
    theta: float = 10000.0
    max_t: int = 1024
    max_h: int = 128
    max_w: int = 128

    def _c(self) -> _Desc:
        return _Desc(self.head_dim, self.dim_t, self.dim_h, self.dim_w, float(self.theta),
                     self.max_t, self.max_h, self.max_w)


CROPE_OK, CROPE_EINVAL, CROPE_ESHAPE, CROPE_EALIGN, CROPE_ERANGE, CROPE_EWORKSPACE, CROPE_EHIP = \
    0, -1, -2, -3, -4, -5, -6


def library_path() -> str:
    return _LIB_PATH


def _load():
    global _lib
    if _lib is not None:
        return _lib
    import torch  # noqa: F401  (loads the HIP runtime the library binds to)
    if not os.path.exists(_LIB_PATH):
        from . import build as _build
        _build.build()
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32, i64, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float
    lib.crope_last_error.restype = ctypes.c_char_p
    lib.crope_version.restype = ctypes.c_char_p
    lib.crope_table_bytes.restype = ctypes.c_size_t
    lib.crope_table_bytes.argtypes = [ctypes.POINTER(_Desc)]
    lib.crope_build_table.restype = ctypes.c_int
    lib.crope_build_table.argtypes = [ctypes.POINTER(_Desc), vp, ctypes.c_size_t, vp]
    lib.crope_qk_norm_rotate_append.restype = ctypes.c_int
    lib.crope_qk_norm_rotate_append.argtypes = [
        ctypes.POINTER(_Desc), vp, vp, vp, vp, _Strides, vp, vp, f32, i32, i32, i32, i32, i32,
        i32, i32, vp, _Strides, vp, vp, _Strides, i64, i64, vp]
    lib.crope_qk_norm_rotate_append_qscaled.restype = ctypes.c_int
    lib.crope_qk_norm_rotate_append_qscaled.argtypes = [
        ctypes.POINTER(_Desc), vp, vp, vp, vp, _Strides, vp, vp, f32, i32, i32, i32, i32, i32,
        i32, i32, f32, vp, _Strides, vp, vp, _Strides, i64, i64, vp]
    lib.crope_folded_q_scale.restype = ctypes.c_float
    lib.crope_folded_q_scale.argtypes = [f32]
    lib.chunk_attention_workspace_bytes.restype = ctypes.c_size_t
    lib.chunk_attention_workspace_bytes.argtypes = [i32, i32, i64]
    lib.chunk_attention.restype = ctypes.c_int
    lib.chunk_attention.argtypes = [
        vp, _Strides, i32, i32, vp, vp, _Strides, i64, ctypes.POINTER(_Segment), i32, f32, vp,
        _Strides, vp, vp, ctypes.c_size_t, vp]
    lib.chunk_attention_choose_plan.restype = ctypes.c_int
    lib.chunk_attention_choose_plan.argtypes = [i32, i32, i64, ctypes.POINTER(_Plan)]
    lib.chunk_attention_planned_workspace_bytes.restype = ctypes.c_size_t
    lib.chunk_attention_planned_workspace_bytes.argtypes = [i32, i32, i64, ctypes.POINTER(_Plan)]
    lib.chunk_attention_planned.restype = ctypes.c_int
    lib.chunk_attention_planned.argtypes = [
        vp, _Strides, i32, i32, vp, vp, _Strides, i64, ctypes.POINTER(_Segment), i32, f32,
        ctypes.POINTER(_Plan), vp, _Strides, vp, vp, ctypes.c_size_t, vp]
    lib.chunk_attention_static_capacity.restype = ctypes.c_size_t
    lib.chunk_attention_static_capacity.argtypes = []
    lib.chunk_attention_static.restype = ctypes.c_int
    lib.chunk_attention_static.argtypes = [
        vp, _Strides, i32, i32, vp, vp, _Strides, i64, ctypes.POINTER(_Segment), i32, f32, vp,
        _Strides, vp, vp]
    lib.chunk_attention_limited.restype = ctypes.c_int
    lib.chunk_attention_limited.argtypes = [
        vp, _Strides, i32, i32, vp, vp, _Strides, i64, ctypes.POINTER(_Segment), i32, f32, vp, vp,
        _Strides, vp, vp]
    lib.crope_qkv_project_workspace_bytes.restype = ctypes.c_size_t
    lib.crope_qkv_project_workspace_bytes.argtypes = [i32, i32, i32]
    lib.crope_qkv_project_norm_rotate_append.restype = ctypes.c_int
    lib.crope_qkv_project_norm_rotate_append.argtypes = [
        ctypes.POINTER(_Desc), vp, vp, i64, vp, vp, i32, vp, vp, f32, i32, i32, i32, i32, i32, i32,
        i32, vp, _Strides, vp, vp, _Strides, i64, i64, vp, ctypes.c_size_t, vp]
    _lib = lib
    return lib


def _check(rc: int) -> None:
    if rc != 0:
        raise CropeError(rc, _load().crope_last_error().decode())


def _ptr(t) -> Optional[int]:
    return None if t is None else int(t.data_ptr())


def _strides(t) -> _Strides:
    """[token][head][128] strides in elements; the channel stride must be 1."""
    if t.dim() != 3 or t.stride(2) != 1:
        raise CropeError(CROPE_EINVAL, "expected a [token, head, 128] tensor with contiguous channels")
    return _Strides(int(t.stride(0)), int(t.stride(1)))


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return int(torch.cuda.current_stream().cuda_stream) if torch.cuda.is_available() else None
    return int(getattr(stream, "cuda_stream", stream))


def crope_last_error() -> str:
    return _load().crope_last_error().decode()


def crope_version() -> str:
    return _load().crope_version().decode()


def crope_table_bytes(desc: TableDesc) -> int:
    d = desc._c()
    return int(_load().crope_table_bytes(ctypes.byref(d)))


def crope_build_table(desc: TableDesc, d_table, nbytes: Optional[int] = None, stream=None) -> None:
    d = desc._c()
    if nbytes is None:
        nbytes = d_table.numel() * d_table.element_size()
    _check(_load().crope_build_table(ctypes.byref(d), _ptr(d_table), nbytes, _stream(stream)))


def crope_qk_norm_rotate_append(desc: TableDesc, d_table, q, k, v, gain_q, gain_k, eps: float,
                                norm_group: int, n_tokens: int, n_heads: int, grid_h: int,
                                grid_w: int, start_frame: int, token_offset: int, q_out, k_cache,
                                v_cache, cache_capacity_tokens: int, dst_token: int,
                                stream=None) -> None:
    d = desc._c()
    sin = _strides(q)
    if _strides(k).token != sin.token or _strides(v).token != sin.token or \
            _strides(k).head != sin.head or _strides(v).head != sin.head:
        raise CropeError(CROPE_EINVAL, "q, k, v must share strides")
    sc = _strides(k_cache)
    if _strides(v_cache).token != sc.token or _strides(v_cache).head != sc.head:
        raise CropeError(CROPE_EINVAL, "k_cache and v_cache must share strides")
    _check(_load().crope_qk_norm_rotate_append(
        ctypes.byref(d), _ptr(d_table), _ptr(q), _ptr(k), _ptr(v), sin, _ptr(gain_q),
        _ptr(gain_k), eps, norm_group, n_tokens, n_heads, grid_h, grid_w, start_frame,
        token_offset, _ptr(q_out), _strides(q_out), _ptr(k_cache), _ptr(v_cache), sc,
        cache_capacity_tokens, dst_token, _stream(stream)))


CROPE_SCALE_FOLDED = 0.0


def crope_folded_q_scale(softmax_scale: float) -> float:
    return float(_load().crope_folded_q_scale(softmax_scale))


def crope_qk_norm_rotate_append_qscaled(desc: TableDesc, d_table, q, k, v, gain_q, gain_k, eps: float,
                                        norm_group: int, n_tokens: int, n_heads: int, grid_h: int,
                                        grid_w: int, start_frame: int, token_offset: int, q_scale: float,
                                        q_out, k_cache, v_cache, cache_capacity_tokens: int, dst_token: int,
                                        stream=None) -> None:
    d = desc._c()
    sin = _strides(q)
    if _strides(k).token != sin.token or _strides(v).token != sin.token or \
            _strides(k).head != sin.head or _strides(v).head != sin.head:
        raise CropeError(CROPE_EINVAL, "q, k, v must share strides")
    sc = _strides(k_cache)
    if _strides(v_cache).token != sc.token or _strides(v_cache).head != sc.head:
        raise CropeError(CROPE_EINVAL, "k_cache and v_cache must share strides")
    _check(_load().crope_qk_norm_rotate_append_qscaled(
        ctypes.byref(d), _ptr(d_table), _ptr(q), _ptr(k), _ptr(v), sin, _ptr(gain_q),
        _ptr(gain_k), eps, norm_group, n_tokens, n_heads, grid_h, grid_w, start_frame,
        token_offset, q_scale, _ptr(q_out), _strides(q_out), _ptr(k_cache), _ptr(v_cache), sc,
        cache_capacity_tokens, dst_token, _stream(stream)))


def chunk_attention_workspace_bytes(n_q: int, n_heads: int, n_keys: int) -> int:
    return int(_load().chunk_attention_workspace_bytes(n_q, n_heads, n_keys))


def chunk_attention(q, n_q: int, n_heads: int, k_cache, v_cache, cache_capacity_tokens: int,
                    segs: Sequence[Tuple[int, int]], scale: float, out, lse=None, workspace=None,
                    workspace_bytes: int = 0, stream=None) -> None:
    sc = _strides(k_cache)
    if _strides(v_cache).token != sc.token or _strides(v_cache).head != sc.head:
        raise CropeError(CROPE_EINVAL, "k_cache and v_cache must share strides")
    arr = (_Segment * max(1, len(segs)))()
    for i, (s, n) in enumerate(segs):
        arr[i].start, arr[i].len = int(s), int(n)
    if workspace is not None and workspace_bytes == 0:
        workspace_bytes = workspace.numel() * workspace.element_size()
    _check(_load().chunk_attention(
        _ptr(q), _strides(q), n_q, n_heads, _ptr(k_cache), _ptr(v_cache), sc,
        cache_capacity_tokens, arr, len(segs), scale, _ptr(out), _strides(out), _ptr(lse),
        _ptr(workspace), workspace_bytes, _stream(stream)))


def _plan(plan) -> Optional[_Plan]:
    """plan: None or a (waves, splits) pair; 0 = chosen by the library."""
    return None if plan is None else _Plan(int(plan[0]), int(plan[1]))


def chunk_attention_choose_plan(n_q: int, n_heads: int, n_keys: int, plan=(0, 0)) -> Tuple[int, int]:
    p = _plan(plan)
    _check(_load().chunk_attention_choose_plan(n_q, n_heads, n_keys, ctypes.byref(p)))
    return int(p.waves), int(p.splits)


def chunk_attention_planned_workspace_bytes(n_q: int, n_heads: int, n_keys: int, plan=None) -> int:
    p = _plan(plan)
    return int(_load().chunk_attention_planned_workspace_bytes(n_q, n_heads, n_keys,
                                                               None if p is None else ctypes.byref(p)))


def chunk_attention_planned(q, n_q: int, n_heads: int, k_cache, v_cache, cache_capacity_tokens: int,
                            segs: Sequence[Tuple[int, int]], scale: float, plan, out, lse=None,
                            workspace=None, workspace_bytes: int = 0, stream=None) -> None:
    sc = _strides(k_cache)
    if _strides(v_cache).token != sc.token or _strides(v_cache).head != sc.head:
        raise CropeError(CROPE_EINVAL, "k_cache and v_cache must share strides")
    arr = (_Segment * max(1, len(segs)))()
    for i, (s, n) in enumerate(segs):
        arr[i].start, arr[i].len = int(s), int(n)
    if workspace is not None and workspace_bytes == 0:
        workspace_bytes = workspace.numel() * workspace.element_size()
    p = _plan(plan)
    _check(_load().chunk_attention_planned(
        _ptr(q), _strides(q), n_q, n_heads, _ptr(k_cache), _ptr(v_cache), sc,
        cache_capacity_tokens, arr, len(segs), scale, None if p is None else ctypes.byref(p),
        _ptr(out), _strides(out), _ptr(lse), _ptr(workspace), workspace_bytes, _stream(stream)))


def chunk_attention_static_capacity() -> int:
    return int(_load().chunk_attention_static_capacity())


def chunk_attention_static(q, n_q: int, n_heads: int, k_cache, v_cache, cache_capacity_tokens: int,
                           segs: Sequence[Tuple[int, int]], scale: float, out, lse=None, stream=None) -> None:
    sc = _strides(k_cache)
    if _strides(v_cache).token != sc.token or _strides(v_cache).head != sc.head:
        raise CropeError(CROPE_EINVAL, "k_cache and v_cache must share strides")
    arr = (_Segment * max(1, len(segs)))()
    for i, (s, n) in enumerate(segs):
        arr[i].start, arr[i].len = int(s), int(n)
    _check(_load().chunk_attention_static(
        _ptr(q), _strides(q), n_q, n_heads, _ptr(k_cache), _ptr(v_cache), sc, cache_capacity_tokens,
        arr, len(segs), scale, _ptr(out), _strides(out), _ptr(lse), _stream(stream)))


def chunk_attention_limited(q, n_q: int, n_heads: int, k_cache, v_cache, cache_capacity_tokens: int,
                            segs: Sequence[Tuple[int, int]], scale: float, q_limit, out, lse=None,
                            stream=None) -> None:
    sc = _strides(k_cache)
    if _strides(v_cache).token != sc.token or _strides(v_cache).head != sc.head:
        raise CropeError(CROPE_EINVAL, "k_cache and v_cache must share strides")
    arr = (_Segment * max(1, len(segs)))()
    for i, (s, n) in enumerate(segs):
        arr[i].start, arr[i].len = int(s), int(n)
    _check(_load().chunk_attention_limited(
        _ptr(q), _strides(q), n_q, n_heads, _ptr(k_cache), _ptr(v_cache), sc, cache_capacity_tokens,
        arr, len(segs), scale, _ptr(q_limit), _ptr(out), _strides(out), _ptr(lse), _stream(stream)))


def crope_qkv_project_workspace_bytes(n_tokens: int, n_heads: int, norm_group: int) -> int:
    return int(_load().crope_qkv_project_workspace_bytes(n_tokens, n_heads, norm_group))


def crope_qkv_project_norm_rotate_append(desc: TableDesc, d_table, x, w_qkv, bias, c_in: int, gain_q,
                                         gain_k, eps: float, norm_group: int, n_tokens: int,
                                         n_heads: int, grid_h: int, grid_w: int, start_frame: int,
                                         token_offset: int, q_out, k_cache, v_cache,
                                         cache_capacity_tokens: int, dst_token: int, workspace=None,
                                         workspace_bytes: int = 0, stream=None) -> None:
    d = desc._c()
    if x.dim() != 2 or x.stride(1) != 1:
        raise CropeError(CROPE_EINVAL, "expected x as [token, c_in] with contiguous channels")
    if w_qkv.dim() != 2 or not w_qkv.is_contiguous():
        raise CropeError(CROPE_EINVAL, "expected w_qkv as a contiguous [3*H*128, c_in] tensor")
    sc = _strides(k_cache)
    if _strides(v_cache).token != sc.token or _strides(v_cache).head != sc.head:
        raise CropeError(CROPE_EINVAL, "k_cache and v_cache must share strides")
    if workspace is not None and workspace_bytes == 0:
        workspace_bytes = workspace.numel() * workspace.element_size()
    _check(_load().crope_qkv_project_norm_rotate_append(
        ctypes.byref(d), _ptr(d_table), _ptr(x), int(x.stride(0)), _ptr(w_qkv), _ptr(bias), c_in,
        _ptr(gain_q), _ptr(gain_k), eps, norm_group, n_tokens, n_heads, grid_h, grid_w, start_frame,
        token_offset, _ptr(q_out), _strides(q_out), _ptr(k_cache), _ptr(v_cache), sc,
        cache_capacity_tokens, dst_token, _ptr(workspace), workspace_bytes, _stream(stream)))
