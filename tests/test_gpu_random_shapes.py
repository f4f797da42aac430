"""Seeded random shapes: head counts, grids, chunk lengths, history lengths, ring capacities,
shard offsets and reduction lengths drawn at random (fixed seeds), every output element
compared with the oracle.  Complements the hand-picked edge cases."""
import numpy as np
import pytest

from paper_2603_06664_amd import workloads as W

import harness as Hn

pytestmark = pytest.mark.gpu


def _random_config(seed: int) -> W.ChunkConfig:
    rng = np.random.default_rng(1000 + seed)
    H = int(rng.choice([1, 2, 3, 5, 8, 12, 17, 40]))
    gh, gw = int(rng.integers(1, 13)), int(rng.integers(1, 17))
    nf = int(rng.integers(1, 4))
    hist = int(rng.integers(0, 5)) * nf
    first = int(rng.integers(0, 4)) * nf
    start = first + hist
    cache_frames = None
    if rng.random() < 0.4 and hist > 0:
        cache_frames = hist + nf          # a ring exactly as long as the visible window
    kwargs = {}
    chunk = nf * gh * gw
    if rng.random() < 0.3 and chunk >= 4:  # a shard of the chunk
        parts = int(rng.choice([2, 4]))
        n_local = -(-chunk // parts)
        r = int(rng.integers(0, parts))
        if r * n_local < chunk and (r + 1) * n_local <= chunk:
            kwargs = dict(token_offset=r * n_local, n_local=n_local)
    return W.ChunkConfig("RND%d" % seed, 2000 + seed, H, gh, gw, start_frame=start, n_frames=nf,
                         first_kv_frame=first, cache_frames=cache_frames,
                         k_head_scale=bool(rng.random() < 0.3), **kwargs)


@pytest.mark.parametrize("seed", range(32))
def test_random_chunk(seed):
    cfg = _random_config(seed)
    print("random chunk %d: H=%d grid %dx%d frames %d..%d chunk %d q=%d keys=%d ring=%s off=%d"
          % (seed, cfg.n_heads, cfg.grid_h, cfg.grid_w, cfg.first_kv_frame, cfg.start_frame, cfg.n_frames,
             cfg.n_q, cfg.n_keys, cfg.cache_frames, cfg.token_offset), flush=True)
    per_head = seed % 2 == 1
    group = cfg.head_dim if per_head else cfg.n_heads * cfg.head_dim
    inp = W.make_inputs(cfg)
    ref = Hn.oracle_chain(cfg, inp, norm_group=group)
    got = Hn.hip_chain(cfg, inp, norm_group=group)
    assert got["segs"] == ref["segs"]
    Hn.assert_close("q_rot", got["q_rot"], ref["q_rot"])
    Hn.assert_close("k_cache", got["k_cache"], ref["k_cache"])
    np.testing.assert_array_equal(got["v_cache_bits"], W.f32_to_bf16_bits(ref["v_cache"].astype(np.float32)))
    Hn.assert_close("o", got["o"], ref["o"])
    assert np.max(np.abs(got["lse"] - ref["lse"])) <= 2e-2


@pytest.mark.parametrize("seed", range(20))
def test_random_projection(seed):
    cfg = _random_config(100 + seed)
    rng = np.random.default_rng(5000 + seed)
    c_in = 64 * int(rng.integers(1, 10))
    per_head = seed % 2 == 0
    print("random projection %d: H=%d tokens=%d c_in=%d per_head=%s off=%d" %
          (seed, cfg.n_heads, cfg.n_q, c_in, per_head, cfg.token_offset), flush=True)
    group = cfg.head_dim if per_head else cfg.n_heads * cfg.head_dim
    inp = W.make_inputs(cfg)
    pin = W.make_projection_inputs(cfg, c_in=c_in)
    use_bias = seed % 3 != 0
    q, k, v = Hn.oracle_projected(cfg, pin, inp, norm_group=group, use_bias=use_bias)
    got = Hn.hip_projected(cfg, pin, inp, norm_group=group, use_bias=use_bias, dst=int(rng.integers(0, 9)),
                           cap_extra=11)
    Hn.assert_close("q", got["q"], q)
    Hn.assert_close("k", got["k"], k)
    Hn.assert_close("v", got["v"], v)
    assert got["untouched_ok"]


@pytest.mark.parametrize("seed", range(10))
def test_random_limited_attention(seed):
    """Random per-query prefix limits (sorted, blocky or arbitrary) against the oracle's mask."""
    import torch
    import oracle
    import paper_2603_06664_amd as P
    rng = np.random.default_rng(9000 + seed)
    H = int(rng.choice([1, 2, 5, 12]))
    n_q = int(rng.integers(1, 700))
    n_k = int(rng.integers(1, 1500))
    kind = seed % 3
    if kind == 0:
        limits = np.sort(rng.integers(1, n_k + 1, size=n_q))
    elif kind == 1:
        blk = int(rng.integers(1, max(2, n_k // 3)))
        limits = np.minimum(n_k, (np.arange(n_q) * n_k // max(n_q, 1) // blk + 1) * blk)
    else:
        limits = rng.integers(1, n_k + 1, size=n_q)
    print("random limited %d: H=%d n_q=%d n_k=%d kind=%d" % (seed, H, n_q, n_k, kind), flush=True)
    qb = W.f32_to_bf16_bits(rng.standard_normal((n_q, H, 128), dtype=np.float32))
    kb = W.f32_to_bf16_bits(rng.standard_normal((n_k, H, 128), dtype=np.float32))
    vb = W.f32_to_bf16_bits(rng.standard_normal((n_k, H, 128), dtype=np.float32))
    q, k, v = Hn.to_dev_bf16(qb), Hn.to_dev_bf16(kb), Hn.to_dev_bf16(vb)
    out = torch.empty_like(q)
    lse = torch.empty((H, n_q), dtype=torch.float32, device="cuda")
    lim = torch.from_numpy(limits.astype(np.int32)).cuda()
    P.chunk_attention_limited(q, n_q, H, k, v, n_k, [(0, n_k)], Hn.SCALE, lim, out, lse)
    torch.cuda.synchronize()
    o_ref, lse_ref = oracle.attention(Hn.bits_to_f64(qb), Hn.bits_to_f64(kb), Hn.bits_to_f64(vb), Hn.SCALE,
                                      q_block=(limits - 1).astype(np.int32), k_block=np.arange(n_k, dtype=np.int32))
    Hn.assert_close("o", Hn.bits_to_f64(Hn.dev_bits(out)), o_ref)
    assert np.max(np.abs(lse.cpu().numpy().astype(np.float64) - lse_ref)) <= 2e-2


@pytest.mark.parametrize("seed", range(24))
def test_random_attention_segments_and_plans(seed):
    """Random query/key counts, 1..4 disjoint cache segments in random order, a random work
    division forced through chunk_attention_planned and either scale convention, against the
    oracle over the concatenated segments."""
    import torch
    import oracle
    import paper_2603_06664_amd as P
    rng = np.random.default_rng(70000 + seed)
    H = int(rng.choice([1, 2, 3, 5, 8]))
    n_q = int(rng.integers(1, 1300))
    cap = int(rng.integers(8, 5000))
    n_segs = int(rng.integers(1, 5))
    cuts = np.sort(rng.choice(np.arange(1, cap), size=min(2 * n_segs - 1, cap - 1), replace=False))
    bounds = np.concatenate([[0], cuts, [cap]])
    pieces = [(int(bounds[i]), int(bounds[i + 1] - bounds[i])) for i in range(0, len(bounds) - 1, 2)][:n_segs]
    segs = [pieces[i] for i in rng.permutation(len(pieces))]
    plan = (int(rng.choice([0, 4, 8])), int(rng.choice([0, 0, 1, 2, 3, 5, 8, 16])))
    folded = bool(rng.integers(0, 2))
    n_keys = sum(m for _, m in segs)
    print("random attention %d: H=%d n_q=%d cap=%d segs=%s plan=%s folded=%d" % (seed, H, n_q, cap, segs, plan, folded),
          flush=True)
    bits = lambda shape: W.f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32))
    qb, kb, vb = bits((n_q, H, 128)), bits((cap, H, 128)), bits((cap, H, 128))
    q_ref, scale = Hn.bits_to_f64(qb), Hn.SCALE
    if folded:   # q as crope_qk_norm_rotate_append_qscaled would have written it
        c = np.float32(P.crope_folded_q_scale(Hn.SCALE))
        qb = W.f32_to_bf16_bits(W.bf16_bits_to_f32(qb) * c)
        q_ref, scale = Hn.bits_to_f64(qb) / float(c), P.CROPE_SCALE_FOLDED
    q, k, v = Hn.to_dev_bf16(qb), Hn.to_dev_bf16(kb), Hn.to_dev_bf16(vb)
    out = torch.empty_like(q)
    lse = torch.empty((H, n_q), dtype=torch.float32, device="cuda")
    wsb = P.chunk_attention_planned_workspace_bytes(n_q, H, n_keys, plan)
    ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device="cuda")
    P.chunk_attention_planned(q, n_q, H, k, v, cap, segs, scale, plan, out, lse, ws, wsb)
    torch.cuda.synchronize()
    kf, vf = Hn.bits_to_f64(kb), Hn.bits_to_f64(vb)
    o_ref, lse_ref = oracle.attention(q_ref, np.concatenate([kf[s:s + m] for s, m in segs]),
                                      np.concatenate([vf[s:s + m] for s, m in segs]), Hn.SCALE)
    Hn.assert_close("o", Hn.bits_to_f64(Hn.dev_bits(out)), o_ref)
    assert np.max(np.abs(lse.cpu().numpy().astype(np.float64) - lse_ref)) <= 2e-2
