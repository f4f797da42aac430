"""Parity of the fused QKV projection + norm + RoPE + cache update (through the C ABI)
against the fp64 oracle chain, element by element.

Tolerances: v and, with the per-head norm, q and k are rounded once: max-abs <= 2e-2, relative
L2 <= 1e-2.  With the row-wide norm q and k are rounded twice (stored as rotate(gain*y), then
scaled by 1/rms in place): each rounding is at most 2^-9 relative, so the element bound is
2e-2 + 2^-8*|oracle| (and the same relative L2)."""
import numpy as np
import pytest

from paper_2603_06664_amd import workloads as W

import harness as Hn

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2603_06664_amd as pkg
    from paper_2603_06664_amd import binding
    binding._load()
    return pkg


def _say(msg):
    print(msg, flush=True)


def _check(cfg, got, ref, per_head):
    q, k, v = ref
    eq = Hn.assert_close("q", got["q"], q)
    ek = Hn.assert_close("k", got["k"], k)
    ev = Hn.assert_close("v", got["v"], v)
    assert got["untouched_ok"], "rows outside [dst, dst+n) were written"
    return eq, ek, ev


# (config, c_in): token counts ragged against the 256-token tile, reduction lengths of 1, 2, 3,
# 5 and 7 steps of 64 (prologue only, tail only, steady loop once, steady loop + 4-step tail)
SMALL = [
    (W.ChunkConfig("Q1", 31, 2, 4, 6, start_frame=5, n_frames=1, first_kv_frame=5), 256),
    (W.ChunkConfig("Q2", 32, 3, 5, 7, start_frame=6, n_frames=3, first_kv_frame=6), 64),
    (W.ChunkConfig("Q3", 33, 5, 10, 15, start_frame=4, n_frames=1, first_kv_frame=4), 128),
    (W.ChunkConfig("Q4", 34, 40, 4, 5, start_frame=3, n_frames=3, first_kv_frame=3, token_offset=15, n_local=15), 192),
    (W.ChunkConfig("Q5", 35, 1, 10, 10, start_frame=0, n_frames=3, first_kv_frame=0), 320),
    (W.ChunkConfig("Q6", 36, 4, 19, 9, start_frame=2, n_frames=3, first_kv_frame=2, k_head_scale=True), 448),
]


@pytest.mark.parametrize("cfg,c_in", SMALL, ids=[c.name for c, _ in SMALL])
@pytest.mark.parametrize("per_head", [False, True], ids=["normHD", "normD"])
def test_small_every_element(P, cfg, c_in, per_head):
    _say("projection case %s c_in=%d per_head=%s n=%d" % (cfg.name, c_in, per_head, cfg.n_q))
    group = cfg.head_dim if per_head else cfg.n_heads * cfg.head_dim
    inp = W.make_inputs(cfg)
    pin = W.make_projection_inputs(cfg, c_in=c_in)
    ref = Hn.oracle_projected(cfg, pin, inp, norm_group=group)
    got = Hn.hip_projected(cfg, pin, inp, norm_group=group)
    _check(cfg, got, ref, per_head)


def test_no_bias_and_padded_input_rows(P):
    cfg, c_in = SMALL[2]
    _say("projection no-bias / strided x")
    inp = W.make_inputs(cfg)
    pin = W.make_projection_inputs(cfg, c_in=c_in)
    ref = Hn.oracle_projected(cfg, pin, inp, use_bias=False)
    got = Hn.hip_projected(cfg, pin, inp, use_bias=False, x_pad=24)
    _check(cfg, got, ref, per_head=False)


def test_deterministic(P):
    cfg, c_in = SMALL[5]
    inp = W.make_inputs(cfg)
    pin = W.make_projection_inputs(cfg, c_in=c_in)
    a = Hn.hip_projected(cfg, pin, inp)
    b = Hn.hip_projected(cfg, pin, inp)
    for key in ("q", "k", "v"):
        np.testing.assert_array_equal(a[key], b[key])


def test_matches_unfused_path_on_identity_weights(P):
    """W_q = W_k = W_v = I, no bias: the projection returns x itself (exactly, in fp32), so the
    fused call must agree with crope_qk_norm_rotate_append on q = k = v = x to rounding."""
    import torch
    cfg = W.ChunkConfig("Q7", 37, 2, 6, 7, start_frame=1, n_frames=2, first_kv_frame=1)
    H, D, n = cfg.n_heads, cfg.head_dim, cfg.n_q
    hd = H * D
    inp = W.make_inputs(cfg)
    x = inp.q.reshape(n, hd)
    eye = W.f32_to_bf16_bits(np.concatenate([np.eye(hd, dtype=np.float32)] * 3, axis=0))
    pin = W.ProjectionInputs(x, eye, np.zeros(3 * hd, dtype=np.float32))
    got = Hn.hip_projected(cfg, pin, inp, norm_group=D, use_bias=False, dst=0, cap_extra=0)
    desc, tab = Hn.make_table(P.TableDesc())
    xq = Hn.to_dev_bf16(inp.q)
    q_out = torch.empty_like(xq)
    kc = torch.zeros_like(xq)
    vc = torch.zeros_like(xq)
    P.crope_qk_norm_rotate_append(desc, tab, xq, xq, xq, torch.from_numpy(inp.gain_q).cuda(),
                                  torch.from_numpy(inp.gain_k).cuda(), cfg.eps, D, n, H, cfg.grid_h,
                                  cfg.grid_w, cfg.start_frame, 0, q_out, kc, vc, n, 0)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(got["v"], Hn.bits_to_f64(Hn.dev_bits(vc)))   # v = x, bit-exact
    # same fp32 inputs, same formula; only the summation order of the statistics differs
    assert np.max(np.abs(got["q"] - Hn.bits_to_f64(Hn.dev_bits(q_out)))) <= 2 ** -6
    assert np.mean(got["q"] != Hn.bits_to_f64(Hn.dev_bits(q_out))) < 0.01
    assert np.mean(got["k"] != Hn.bits_to_f64(Hn.dev_bits(kc))) < 0.01


FULL = [("C4", None), ("C5", None)]


@pytest.mark.parametrize("name,c_in", FULL, ids=[n for n, _ in FULL])
@pytest.mark.parametrize("per_head", [False, True], ids=["normHD", "normD"])
def test_full_size_every_element(P, name, c_in, per_head):
    cfg = W.CONFIGS[name]
    _say("projection full size %s per_head=%s: %d tokens, %d heads" % (name, per_head, cfg.n_q, cfg.n_heads))
    group = cfg.head_dim if per_head else cfg.n_heads * cfg.head_dim
    inp = W.make_inputs(cfg)
    pin = W.make_projection_inputs(cfg, c_in=c_in)
    ref = Hn.oracle_projected(cfg, pin, inp, norm_group=group)
    got = Hn.hip_projected(cfg, pin, inp, norm_group=group)
    eq, ek, ev = _check(cfg, got, ref, per_head)
    _say("  q %.3e/%.3e  k %.3e/%.3e  v %.3e/%.3e (max-abs / rel-L2)" % (eq + ek + ev))


def test_errors(P):
    import torch
    cfg, c_in = SMALL[0]
    inp = W.make_inputs(cfg)
    pin = W.make_projection_inputs(cfg, c_in=c_in)
    H, D, n = cfg.n_heads, cfg.head_dim, cfg.n_q
    desc, tab = Hn.make_table(P.TableDesc())
    x = Hn.to_dev_bf16(pin.x)
    w = Hn.to_dev_bf16(pin.w)
    g = torch.ones(H * D, device="cuda")
    q_out = torch.empty((n, H, D), dtype=torch.bfloat16, device="cuda")
    kc = torch.zeros((n, H, D), dtype=torch.bfloat16, device="cuda")
    vc = torch.zeros_like(kc)
    args = lambda c, ws, wsb, cap=n: (desc, tab, x, w, None, c, g, g, cfg.eps, H * D, n, H, cfg.grid_h,
                                      cfg.grid_w, cfg.start_frame, 0, q_out, kc, vc, cap, 0, ws, wsb)
    with pytest.raises(P.CropeError) as e:
        P.crope_qkv_project_norm_rotate_append(*args(96, None, 0))
    assert e.value.code == -2
    with pytest.raises(P.CropeError) as e:
        P.crope_qkv_project_norm_rotate_append(*args(c_in, None, 0))
    assert e.value.code == -5
    ws = torch.empty(P.crope_qkv_project_workspace_bytes(n, H, H * D), dtype=torch.uint8, device="cuda")
    with pytest.raises(P.CropeError) as e:
        P.crope_qkv_project_norm_rotate_append(*args(c_in, ws, 0, cap=n - 1))
    assert e.value.code == -4
    P.crope_qkv_project_norm_rotate_append(*args(c_in, ws, 0))   # and the valid call goes through
    torch.cuda.synchronize()


def test_strided_outputs(P):
    """q_out and the caches as views into wider buffers (token and head strides larger than the
    dense ones): results equal the dense call bit for bit and nothing else is written."""
    import torch
    cfg, c_in = SMALL[2]
    H, D, n = cfg.n_heads, cfg.head_dim, cfg.n_q
    inp = W.make_inputs(cfg)
    pin = W.make_projection_inputs(cfg, c_in=c_in)
    dense = Hn.hip_projected(cfg, pin, inp, dst=0, cap_extra=0)
    desc, tab = Hn.make_table(P.TableDesc())
    x, w = Hn.to_dev_bf16(pin.x), Hn.to_dev_bf16(pin.w)
    bias = torch.from_numpy(pin.bias).cuda()
    gq, gk = torch.from_numpy(inp.gain_q).cuda(), torch.from_numpy(inp.gain_k).cuda()
    canary = 0x7FC1
    def wide():
        return torch.zeros((n, H + 1, D + 64), dtype=torch.int16, device="cuda").fill_(canary).view(torch.bfloat16)
    qb, kb, vb = wide(), wide(), wide()
    q_out, kc, vc = qb[:, :H, :D], kb[:, :H, :D], vb[:, :H, :D]
    ws_bytes = P.crope_qkv_project_workspace_bytes(n, H, H * D)
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device="cuda")
    P.crope_qkv_project_norm_rotate_append(desc, tab, x, w, bias, c_in, gq, gk, cfg.eps, H * D, n, H, cfg.grid_h,
                                           cfg.grid_w, cfg.start_frame, cfg.token_offset, q_out, kc, vc, n, 0,
                                           ws, ws_bytes)
    torch.cuda.synchronize()
    for name, buf in (("q", qb), ("k", kb), ("v", vb)):
        bits = Hn.dev_bits(buf)
        np.testing.assert_array_equal(Hn.bits_to_f64(bits[:, :H, :D]), dense[name])
        assert np.all(bits[:, H:, :] == canary) and np.all(bits[:, :, D:] == canary), name
