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


@pytest.mark.parametrize("seed", range(14))
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
    strict = not cfg.k_head_scale
    Hn.assert_close("q_rot", got["q_rot"], ref["q_rot"], strict_abs=strict)
    Hn.assert_close("k_cache", got["k_cache"], ref["k_cache"], strict_abs=strict)
    np.testing.assert_array_equal(got["v_cache_bits"], W.f32_to_bf16_bits(ref["v_cache"].astype(np.float32)))
    Hn.assert_close("o", got["o"], ref["o"])
    assert np.max(np.abs(got["lse"] - ref["lse"])) <= 2e-2


@pytest.mark.parametrize("seed", range(10))
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
    Hn.assert_close("q", got["q"], q, strict_abs=per_head)
    Hn.assert_close("k", got["k"], k, strict_abs=per_head and not cfg.k_head_scale)
    Hn.assert_close("v", got["v"], v, strict_abs=True)
    assert got["untouched_ok"]
