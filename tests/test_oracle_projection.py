"""Pins of the oracle's QKV projection (Algorithm 3 step 1) and of the projected chain
(steps 1-3), against things other than itself."""
import numpy as np
import pytest

import oracle
from paper_2603_06664_amd import workloads as W


def test_project_matches_library_matmul():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((37, 96))
    w = rng.standard_normal((50, 96))
    b = rng.standard_normal(50)
    got = oracle.project(x, w, b)
    assert got.shape == (37, 50)
    np.testing.assert_allclose(got, x @ w.T + b, rtol=0, atol=1e-12)
    np.testing.assert_allclose(oracle.project(x, w), x @ w.T, rtol=0, atol=1e-12)


def test_project_matches_torch_linear():
    import torch
    rng = np.random.default_rng(1)
    x = rng.standard_normal((9, 64))
    w = rng.standard_normal((24, 64))
    b = rng.standard_normal(24)
    ref = torch.nn.functional.linear(torch.from_numpy(x), torch.from_numpy(w), torch.from_numpy(b)).numpy()
    np.testing.assert_allclose(oracle.project(x, w, b), ref, rtol=0, atol=1e-12)


def test_project_weight_orientation_is_out_by_in():
    # one-hot weights: output o picks input column sel[o]; a transposed operand would not
    x = np.arange(12, dtype=np.float64).reshape(3, 4)
    sel = [2, 0, 3, 3, 1, 0]
    w = np.zeros((6, 4))
    for o, c in enumerate(sel):
        w[o, c] = 1.0
    np.testing.assert_array_equal(oracle.project(x, w), x[:, sel])


def test_project_special_cases():
    rng = np.random.default_rng(2)
    w = rng.standard_normal((10, 8))
    b = rng.standard_normal(10)
    np.testing.assert_array_equal(oracle.project(np.zeros((4, 8)), w, b), np.tile(b, (4, 1)))
    x = rng.standard_normal((5, 8))
    np.testing.assert_allclose(oracle.project(2.5 * x, w), 2.5 * oracle.project(x, w), rtol=1e-14)
    np.testing.assert_allclose(oracle.project(x, w, b) - oracle.project(x, w), np.tile(b, (5, 1)), atol=1e-13)


@pytest.mark.parametrize("group_per_head", [False, True])
def test_identity_weights_reduce_to_unprojected_chain(group_per_head):
    # W_q = W_k = W_v = I, no bias: the projected chain must equal norm+rotate of x itself
    cfg = W.ChunkConfig("P0", 21, 3, 4, 5, start_frame=2, n_frames=2, first_kv_frame=0)
    H, D = cfg.n_heads, cfg.head_dim
    hd = H * D
    rng = np.random.default_rng(3)
    n = cfg.n_q
    x = rng.standard_normal((n, hd))
    w = np.concatenate([np.eye(hd)] * 3, axis=0)
    gq = 1 + 0.1 * rng.standard_normal(hd)
    gk = 1 + 0.1 * rng.standard_normal(hd)
    group = D if group_per_head else hd
    q, k, v = oracle.qkv_project_norm_rotate(x, w, None, gq, gk, cfg.eps, group, H, cfg.dims, cfg.theta,
                                             cfg.grid_h, cfg.grid_w, cfg.start_frame, 0)
    xr = x.reshape(n, H, D)
    np.testing.assert_array_equal(v, xr)
    np.testing.assert_array_equal(q, oracle.qk_norm_rotate(xr, gq, cfg.eps, group, cfg.dims, cfg.theta,
                                                           cfg.grid_h, cfg.grid_w, cfg.start_frame, 0))
    np.testing.assert_array_equal(k, oracle.qk_norm_rotate(xr, gk, cfg.eps, group, cfg.dims, cfg.theta,
                                                           cfg.grid_h, cfg.grid_w, cfg.start_frame, 0))


def test_column_blocks_are_q_k_v_in_that_order():
    # distinct constant weight blocks: q sees only W_q, k only W_k, v only W_v
    cfg = W.ChunkConfig("P1", 22, 1, 2, 3, start_frame=0, n_frames=1, first_kv_frame=0)
    hd = cfg.head_dim
    rng = np.random.default_rng(4)
    x = rng.standard_normal((cfg.n_q, 16))
    wq, wk, wv = (rng.standard_normal((hd, 16)) for _ in range(3))
    b = rng.standard_normal(3 * hd)
    ones = np.ones(hd)
    q, k, v = oracle.qkv_project_norm_rotate(x, np.concatenate([wq, wk, wv]), b, ones, ones, cfg.eps, hd, 1,
                                             cfg.dims, cfg.theta, cfg.grid_h, cfg.grid_w, 0, 0)
    np.testing.assert_allclose(v[:, 0], x @ wv.T + b[2 * hd:], atol=1e-12)
    # token 0 of frame 0 sits at the origin: rotation is the identity there, so q~[0] is the
    # RMS-normalised projection itself
    yq = x[0] @ wq.T + b[:hd]
    np.testing.assert_allclose(q[0, 0], yq / np.sqrt((yq ** 2).mean() + cfg.eps), atol=1e-12)
    yk = x[0] @ wk.T + b[hd:2 * hd]
    np.testing.assert_allclose(k[0, 0], yk / np.sqrt((yk ** 2).mean() + cfg.eps), atol=1e-12)


def test_projection_inputs_are_seeded_and_bf16():
    cfg = W.CONFIGS["C1"]
    a = W.make_projection_inputs(cfg)
    b = W.make_projection_inputs(cfg)
    assert a.x.shape == (cfg.n_q, 256) and a.w.shape == (768, 256) and a.bias.shape == (768,)
    np.testing.assert_array_equal(a.x, b.x)
    np.testing.assert_array_equal(a.w, b.w)
    np.testing.assert_array_equal(W.round_to_bf16(a.bias), a.bias)
    y = oracle.project(W.bf16_bits_to_f32(a.x), W.bf16_bits_to_f32(a.w), a.bias)
    assert 0.7 < y.std() < 1.3
