"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol
the header declares, and rejects bad arguments before anything is launched."""
import ctypes
import os
import re

import pytest

import paper_2603_06664_amd as P
from paper_2603_06664_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    return B._load()


def test_exports_every_declared_symbol(lib):
    hdr = open(os.path.join(ROOT, "include", "crope.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b((?:crope_|chunk_attention)\w*)\s*\(", hdr))
    assert {"crope_build_table", "crope_qk_norm_rotate_append", "chunk_attention",
            "crope_table_bytes", "chunk_attention_workspace_bytes", "crope_last_error",
            "crope_version"} <= names
    for n in names:
        assert hasattr(lib, n), n


def test_version_and_table_bytes():
    assert "gfx950" in P.crope_version()
    d = P.TableDesc()
    assert P.crope_table_bytes(d) == 4 * 2 * (1024 * 22 + 128 * 21 + 128 * 21)
    assert P.crope_table_bytes(P.TableDesc(head_dim=64)) == 0
    assert P.crope_table_bytes(P.TableDesc(dim_t=43, dim_h=43)) == 0
    assert P.crope_table_bytes(P.TableDesc(dim_t=40)) == 0          # does not sum to 128


class _FakeTensor:
    """Stands in for a device tensor: only the address and strides are marshalled, and the
    calls under test must fail validation before touching memory."""
    def __init__(self, addr, shape, strides=None, esize=2):
        self._addr, self._shape, self._esize = addr, shape, esize
        if strides is None:
            strides, acc = [], 1
            for s in reversed(shape):
                strides.insert(0, acc)
                acc *= s
        self._strides = strides
    def data_ptr(self): return self._addr
    def dim(self): return len(self._shape)
    def stride(self, i): return self._strides[i]
    def numel(self):
        n = 1
        for s in self._shape: n *= s
        return n
    def element_size(self): return self._esize


A = 0x10000  # a 16-byte aligned fake address


def _append(desc=None, q_addr=A, n=24, H=2, gh=4, gw=6, s=5, off=0, cap=72, dst=48,
            group=256, strides=None, tab_addr=A, heads_arg=None):
    desc = desc or P.TableDesc()
    t = _FakeTensor(q_addr, (n, H, 128), strides)
    c = _FakeTensor(A, (cap, H, 128))
    tab = _FakeTensor(tab_addr, (1,), esize=4)
    g = _FakeTensor(A, (H * 128,), esize=4)
    P.crope_qk_norm_rotate_append(desc, tab, t, t, t, g, g, 1e-6, group, n,
                                  H if heads_arg is None else heads_arg, gh, gw, s, off, t, c, c,
                                  cap, dst)


@pytest.mark.parametrize("kwargs,code", [
    (dict(q_addr=A + 2), B.CROPE_EALIGN),
    (dict(strides=[2 * 128 + 4, 128, 1]), B.CROPE_EALIGN),
    (dict(desc=P.TableDesc(head_dim=64)), B.CROPE_ESHAPE),
    (dict(desc=P.TableDesc(max_t=5)), B.CROPE_ERANGE),          # frame 5 needs max_t >= 6
    (dict(desc=P.TableDesc(max_w=5)), B.CROPE_ERANGE),          # grid_w 6 > 5
    (dict(dst=49), B.CROPE_ERANGE),                             # rows 49..72 exceed capacity 72
    (dict(dst=-1), B.CROPE_ERANGE),
    (dict(group=64), B.CROPE_EINVAL),
    (dict(n=-1), B.CROPE_EINVAL),
    (dict(heads_arg=0), B.CROPE_EINVAL),
    (dict(heads_arg=65), B.CROPE_ESHAPE),
    (dict(gh=0), B.CROPE_EINVAL),
    (dict(s=-1), B.CROPE_EINVAL),
    (dict(tab_addr=0), B.CROPE_EINVAL),
    (dict(off=24, desc=P.TableDesc(max_t=6)), B.CROPE_ERANGE),  # offset pushes rows into frame 6
    (dict(off=2**31 - 10, desc=P.TableDesc(max_t=1 << 20, max_h=1 << 10, max_w=1 << 11), gh=1 << 10,
          gw=1 << 11, s=0), B.CROPE_ERANGE),                    # 32-bit token index would wrap
    (dict(desc=P.TableDesc(max_h=1 << 16, max_w=1 << 16), gh=1 << 16, gw=1 << 15),
     B.CROPE_ERANGE),                                           # tokens per frame would not fit 32 bits
])
def test_append_rejects_bad_arguments(kwargs, code):
    with pytest.raises(P.CropeError) as ei:
        _append(**kwargs)
    assert ei.value.code == code
    assert ei.value.message and P.crope_last_error() == ei.value.message


@pytest.mark.parametrize("q_scale", [0.0, -0.5, float("nan"), float("inf")])
def test_qscaled_append_rejects_bad_scale(q_scale):
    t = _FakeTensor(A, (24, 2, 128))
    c = _FakeTensor(A, (72, 2, 128))
    g = _FakeTensor(A, (256,), esize=4)
    with pytest.raises(P.CropeError) as ei:
        P.crope_qk_norm_rotate_append_qscaled(P.TableDesc(), _FakeTensor(A, (1,), esize=4), t, t, t, g, g, 1e-6,
                                              256, 24, 2, 4, 6, 5, 0, q_scale, t, c, c, 72, 48)
    assert ei.value.code == B.CROPE_EINVAL


def test_folded_q_scale_value():
    assert abs(P.crope_folded_q_scale(128 ** -0.5) - 128 ** -0.5 * 1.4426950408889634) < 1e-7
    assert P.CROPE_SCALE_FOLDED == 0.0


def test_append_zero_tokens_is_a_noop():
    _append(n=0, dst=72)   # valid: writes rows [72, 72)


def _attn(n_q=24, H=2, cap=72, segs=((0, 72),), scale=128 ** -0.5, q_addr=A, ws=None, ws_bytes=0,
          q_strides=None, c_strides=None, plan=None):
    q = _FakeTensor(q_addr, (max(n_q, 1), H, 128), q_strides)
    c = _FakeTensor(A, (cap, H, 128), c_strides)
    if plan is None:
        P.chunk_attention(q, n_q, H, c, c, cap, list(segs), scale, q, None, ws, ws_bytes)
    else:
        P.chunk_attention_planned(q, n_q, H, c, c, cap, list(segs), scale, plan, q, None, ws, ws_bytes)


@pytest.mark.parametrize("kwargs,code", [
    (dict(segs=((0, 73),)), B.CROPE_ERANGE),
    (dict(segs=((-1, 5),)), B.CROPE_ERANGE),
    (dict(segs=((0, 0),)), B.CROPE_EINVAL),
    (dict(segs=()), B.CROPE_EINVAL),
    (dict(segs=((0, 1),) * 5), B.CROPE_EINVAL),
    (dict(scale=-1.0), B.CROPE_EINVAL),              # 0 is CROPE_SCALE_FOLDED; negative is not a scale
    (dict(scale=float("inf")), B.CROPE_EINVAL),
    (dict(scale=float("nan")), B.CROPE_EINVAL),
    (dict(q_addr=A + 8), B.CROPE_EALIGN),
    (dict(n_q=-3), B.CROPE_EINVAL),
    (dict(H=0), B.CROPE_EINVAL),
    (dict(q_strides=[128, 64, 1]), B.CROPE_EINVAL),      # heads would overlap
    (dict(c_strides=[256, 120, 1]), B.CROPE_EINVAL),
    (dict(plan=(3, 0)), B.CROPE_EINVAL),                 # 4 or 8 waves
    (dict(plan=(8, 17)), B.CROPE_EINVAL),
    (dict(plan=(0, -1)), B.CROPE_EINVAL),
    (dict(n_q=4680, cap=32760, segs=((0, 32760),), H=12, plan=(4, 2)), B.CROPE_EWORKSPACE),
])
def test_attention_rejects_bad_arguments(kwargs, code):
    with pytest.raises(P.CropeError) as ei:
        _attn(**kwargs)
    assert ei.value.code == code


def test_attention_zero_queries_is_a_noop():
    _attn(n_q=0)


def test_workspace_size_query():
    assert P.chunk_attention_workspace_bytes(0, 12, 100) == 0
    assert P.chunk_attention_workspace_bytes(4680, 12, 32760) >= 0


def test_plan_queries_are_pure_functions_of_their_arguments(monkeypatch):
    # no environment variable or earlier call changes a plan
    monkeypatch.setenv("CROPE_ATTN_SPLITS", "7")
    monkeypatch.setenv("CROPE_ATTN_WAVES", "4")
    auto = P.chunk_attention_choose_plan(4680, 12, 32760)
    assert auto == P.chunk_attention_choose_plan(4680, 12, 32760, (0, 0))
    assert auto[0] in (4, 8) and 1 <= auto[1] <= 16
    assert P.chunk_attention_workspace_bytes(4680, 12, 32760) == \
        P.chunk_attention_planned_workspace_bytes(4680, 12, 32760, auto) == \
        P.chunk_attention_planned_workspace_bytes(4680, 12, 32760, None)
    # a pinned field is kept, the other one chosen
    assert P.chunk_attention_choose_plan(4680, 12, 32760, (4, 0))[0] == 4
    assert P.chunk_attention_choose_plan(4680, 12, 32760, (0, 3))[1] == 3
    # fp32 partial O (128) plus reference maximum and denominator per query, head and split
    assert P.chunk_attention_planned_workspace_bytes(100, 3, 1000, (4, 3)) == 3 * 3 * 100 * 130 * 4
    # more splits than key tiles: lowered until no split is empty (130 keys = 3 tiles)
    assert P.chunk_attention_choose_plan(50, 2, 130, (4, 16)) == (4, 3)
    assert P.chunk_attention_choose_plan(50, 2, 64 * 5, (8, 4)) == (8, 3)   # 5 tiles in 4 splits of 2 leaves one empty
    with pytest.raises(P.CropeError):
        P.chunk_attention_choose_plan(0, 2, 130)
    assert P.chunk_attention_planned_workspace_bytes(100, 3, 1000, (5, 3)) == 0   # invalid plan


def test_build_table_rejects_small_buffer():
    d = P.TableDesc()
    with pytest.raises(P.CropeError) as ei:
        P.crope_build_table(d, _FakeTensor(A, (16,), esize=4))
    assert ei.value.code == B.CROPE_EWORKSPACE
    with pytest.raises(P.CropeError) as ei:
        P.crope_build_table(d, _FakeTensor(A + 4, (1 << 20,), esize=4))
    assert ei.value.code == B.CROPE_EALIGN


class _FakeMatrix(_FakeTensor):
    def is_contiguous(self): return True


def _project(n=24, H=2, c_in=256, x_addr=A, w_addr=A, x_stride=None, cap=72, dst=48, group=256, ws=A,
             ws_bytes=1 << 26, desc=None, gh=4, gw=6, s=5):
    desc = desc or P.TableDesc()
    x = _FakeMatrix(x_addr, (n, c_in), [c_in if x_stride is None else x_stride, 1])
    w = _FakeMatrix(w_addr, (3 * H * 128, c_in))
    out = _FakeTensor(A, (max(n, 1), H, 128))
    c = _FakeTensor(A, (cap, H, 128))
    tab = _FakeTensor(A, (1,), esize=4)
    g = _FakeTensor(A, (H * 128,), esize=4)
    wsp = None if ws is None else _FakeTensor(ws, (ws_bytes,), esize=1)
    P.crope_qkv_project_norm_rotate_append(desc, tab, x, w, None, c_in, g, g, 1e-6, group, n, H, gh, gw, s, 0,
                                           out, c, c, cap, dst, wsp, ws_bytes if ws is not None else 0)


@pytest.mark.parametrize("kwargs,code", [
    (dict(c_in=96), B.CROPE_ESHAPE),                 # not a multiple of 64
    (dict(c_in=0), B.CROPE_ESHAPE),
    (dict(x_addr=A + 8), B.CROPE_EALIGN),
    (dict(w_addr=0), B.CROPE_EINVAL),
    (dict(x_stride=128), B.CROPE_EINVAL),            # row stride smaller than c_in
    (dict(x_stride=260), B.CROPE_EALIGN),            # rows not 16-byte aligned
    (dict(x_stride=(1 << 22) + 8), B.CROPE_ERANGE),  # 32-bit byte offsets inside a tile would wrap
    (dict(dst=49), B.CROPE_ERANGE),
    (dict(group=64), B.CROPE_EINVAL),
    (dict(ws=None), B.CROPE_EWORKSPACE),             # the row-wide norm needs its scratch
    (dict(ws_bytes=16), B.CROPE_EWORKSPACE),
    (dict(desc=P.TableDesc(max_t=5)), B.CROPE_ERANGE),
    (dict(n=-1), B.CROPE_EINVAL),
])
def test_project_rejects_bad_arguments(kwargs, code):
    with pytest.raises(P.CropeError) as ei:
        _project(**kwargs)
    assert ei.value.code == code
    assert ei.value.message


def test_project_zero_tokens_is_a_noop_and_workspace_sizes():
    _project(n=0, dst=72)
    assert P.crope_qkv_project_workspace_bytes(4680, 12, 128) == 0
    # sums of squares (rounded up to 256 B) + the bf16 low parts of q and k
    assert P.crope_qkv_project_workspace_bytes(4680, 12, 1536) == 2 * 4680 * 12 * 4 + 2 * 4680 * 12 * 128 * 2
    assert P.crope_qkv_project_workspace_bytes(3, 3, 384) == 256 + 2 * 3 * 3 * 128 * 2
    assert P.crope_qkv_project_workspace_bytes(0, 12, 1536) == 0
