"""CPU oracle (fp64) — TEST INFRASTRUCTURE ONLY.

numpy-facing wrappers around ``oracle.cpp`` plus the few lines of bookkeeping that the
method's problem statement needs (cache rows written at a destination, visible segments).
Nothing here may be imported by the product package; only tests, ``smoke()`` and the
bench's ``cpu_baseline`` leg use it.
"""
from __future__ import annotations

import ctypes
from typing import Optional, Sequence, Tuple

import numpy as np

from . import build as _build

_lib = None

_D = ctypes.POINTER(ctypes.c_double)
_I = ctypes.POINTER(ctypes.c_int32)


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(_build.build())
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_axis_table.argtypes = [ctypes.c_int, ctypes.c_double, ctypes.c_int, _D]
        lib.oracle_decode.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int, ctypes.c_int,
                                      ctypes.c_int, _I, _I, _I]
        lib.oracle_rmsnorm.argtypes = [_D, _D, ctypes.c_double, ctypes.c_int64, ctypes.c_int,
                                       ctypes.c_int, _D]
        lib.oracle_rotate.argtypes = [_D, ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                      ctypes.c_int, ctypes.c_double, ctypes.c_int, ctypes.c_int,
                                      ctypes.c_int, ctypes.c_int64, _D]
        lib.oracle_attention.argtypes = [_D, _D, _D, ctypes.c_int64, ctypes.c_int64, ctypes.c_int,
                                         ctypes.c_int, ctypes.c_double, _I, _I, _D, _D, _D]
        lib.oracle_project.argtypes = [_D, _D, _D, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, _D]
        for f in (lib.oracle_axis_table, lib.oracle_decode, lib.oracle_rmsnorm, lib.oracle_rotate,
                  lib.oracle_attention, lib.oracle_project):
            f.restype = None
        _lib = lib
    return _lib


def _dp(a: np.ndarray):
    return a.ctypes.data_as(_D)


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def axis_table(dim_a: int, theta: float, n_pos: int) -> np.ndarray:
    """[n_pos, dim_a/2, 2] (cos, sin) of pos * theta^(-2j/dim_a)."""
    out = np.empty((n_pos, dim_a // 2, 2), dtype=np.float64)
    _load().oracle_axis_table(dim_a, float(theta), n_pos, _dp(out))
    return out


def decode(i_local: int, delta: int, s: int, grid_h: int, grid_w: int) -> Tuple[int, int, int]:
    t, h, w = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32()
    _load().oracle_decode(i_local, delta, s, grid_h, grid_w, ctypes.byref(t), ctypes.byref(h),
                          ctypes.byref(w))
    return t.value, h.value, w.value


def rmsnorm(x, gain, eps: float, group: int) -> np.ndarray:
    """x: [n, H, D] (or [n, H*D]); gain: [H*D]; group: H*D or D."""
    x = _f64(x)
    shape = x.shape
    n = shape[0]
    hd = int(np.prod(shape[1:]))
    gain = _f64(gain).reshape(-1)
    assert gain.size == hd and hd % group == 0
    y = np.empty_like(x)
    _load().oracle_rmsnorm(_dp(x), _dp(gain), float(eps), n, hd, int(group), _dp(y))
    return y


def rotate(x, dims: Sequence[int], theta: float, grid_h: int, grid_w: int, s: int,
           delta: int = 0) -> np.ndarray:
    """x: [n, H, D] with D = sum(dims); rows are tokens delta..delta+n-1 of the chunk."""
    x = _f64(x)
    n, H, D = x.shape
    dt, dh, dw = (int(d) for d in dims)
    assert dt + dh + dw == D and dt % 2 == 0 and dh % 2 == 0 and dw % 2 == 0
    out = np.empty_like(x)
    _load().oracle_rotate(_dp(x), n, H, dt, dh, dw, float(theta), grid_h, grid_w, int(s),
                          int(delta), _dp(out))
    return out


def qk_norm_rotate(x, gain, eps, group, dims, theta, grid_h, grid_w, s, delta=0) -> np.ndarray:
    """RMSNorm then rotation, no rounding in between."""
    return rotate(rmsnorm(x, gain, eps, group), dims, theta, grid_h, grid_w, s, delta)


def project(x, w, bias=None) -> np.ndarray:
    """x: [n, C]; w: [O, C] (a linear layer's [out][in] weights); bias: [O] or None -> [n, O]."""
    x, w = _f64(x), _f64(w)
    n, c_in = x.shape
    n_out = w.shape[0]
    assert w.shape == (n_out, c_in)
    b = None if bias is None else _f64(bias).reshape(-1)
    assert b is None or b.size == n_out
    y = np.empty((n, n_out), dtype=np.float64)
    _load().oracle_project(_dp(x), _dp(w), _dp(b) if b is not None else None, n, c_in, n_out, _dp(y))
    return y


def qkv_project_norm_rotate(x, w, bias, gain_q, gain_k, eps, group, n_heads, dims, theta, grid_h,
                            grid_w, s, delta=0):
    """Algorithm 3 steps 1-3 with nothing rounded in between: project, split the output
    columns into q | k | v, RMS-normalise and rotate q and k.  Returns (q~, k~, v), each
    [n, H, D]."""
    y = project(x, w, bias)
    n = y.shape[0]
    hd = y.shape[1] // 3
    D = hd // n_heads
    q = y[:, :hd].reshape(n, n_heads, D)
    k = y[:, hd:2 * hd].reshape(n, n_heads, D)
    v = y[:, 2 * hd:].reshape(n, n_heads, D).copy()
    return (qk_norm_rotate(q, gain_q, eps, group, dims, theta, grid_h, grid_w, s, delta),
            qk_norm_rotate(k, gain_k, eps, group, dims, theta, grid_h, grid_w, s, delta), v)


def attention(q, k, v, scale: float, q_block: Optional[np.ndarray] = None,
              k_block: Optional[np.ndarray] = None, return_p: bool = False):
    """q: [Lq,H,D]; k, v: [Lk,H,D].  Returns (o [Lq,H,D], lse [H,Lq][, P [H,Lq,Lk]])."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    Lq, H, D = q.shape
    Lk = k.shape[0]
    assert k.shape == (Lk, H, D) and v.shape == (Lk, H, D)
    o = np.empty_like(q)
    lse = np.empty((H, Lq), dtype=np.float64)
    P = np.empty((H, Lq, Lk), dtype=np.float64) if return_p else None
    qb = kb = None
    if q_block is not None or k_block is not None:
        qb = np.ascontiguousarray(q_block, dtype=np.int32)
        kb = np.ascontiguousarray(k_block, dtype=np.int32)
        assert qb.shape == (Lq,) and kb.shape == (Lk,)
    _load().oracle_attention(
        _dp(q), _dp(k), _dp(v), Lq, Lk, H, D, float(scale),
        qb.ctypes.data_as(_I) if qb is not None else None,
        kb.ctypes.data_as(_I) if kb is not None else None,
        _dp(o), _dp(lse), _dp(P) if P is not None else None)
    return (o, lse, P) if return_p else (o, lse)


class Cache:
    """Rolling KV cache as the problem statement has it (Algorithm 3 step 5): rotated keys
    and untouched values are *assigned* into rows [dst, dst+n); attention later reads a
    list of (start, len) row segments."""

    def __init__(self, capacity_tokens: int, n_heads: int, head_dim: int):
        self.k = np.zeros((capacity_tokens, n_heads, head_dim), dtype=np.float64)
        self.v = np.zeros_like(self.k)

    def write(self, dst: int, k_rot: np.ndarray, v: np.ndarray) -> None:
        n = k_rot.shape[0]
        assert dst >= 0 and dst + n <= self.k.shape[0]
        self.k[dst:dst + n] = k_rot
        self.v[dst:dst + n] = v

    def gather(self, segments: Sequence[Tuple[int, int]]):
        ks = [self.k[s:s + n] for s, n in segments]
        vs = [self.v[s:s + n] for s, n in segments]
        return np.concatenate(ks, axis=0), np.concatenate(vs, axis=0)
