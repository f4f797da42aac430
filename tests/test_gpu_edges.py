"""Edge cases of the HIP path against the fp64 oracle: many segments, ragged tiles, extreme
logits, head counts at the limits, far time positions, and the non-default work-group shapes."""
import os

import numpy as np
import pytest

from paper_2603_06664_amd import workloads as W

import harness as Hn

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def P():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2603_06664_amd as pkg
    from paper_2603_06664_amd import binding
    binding._load()
    return pkg


def _rand_bits(rng, shape, scale=1.0):
    return W.f32_to_bf16_bits((rng.standard_normal(shape) * scale).astype(np.float32))


def _folded_q(P, qb):
    """bf16 queries carrying the factor scale*log2(e), as crope_qk_norm_rotate_append_qscaled would
    have written them, and the fp64 queries the oracle must see for the same softmax."""
    c = np.float32(P.crope_folded_q_scale(Hn.SCALE))
    bits = W.f32_to_bf16_bits(W.bf16_bits_to_f32(qb) * c)
    return bits, Hn.bits_to_f64(bits) / float(c)


FOLDED = pytest.mark.parametrize("folded", [False, True], ids=["scale", "folded"])


def _attn_case(P, n_q, H, cap, segs, seed, q_scale=1.0, want_lse=True, folded=False):
    import torch
    import oracle
    rng = np.random.default_rng(seed)
    qb, kb, vb = _rand_bits(rng, (n_q, H, 128), q_scale), _rand_bits(rng, (cap, H, 128)), _rand_bits(rng, (cap, H, 128))
    q_ref = Hn.bits_to_f64(qb)
    if folded:
        qb, q_ref = _folded_q(P, qb)
    q, k, v = Hn.to_dev_bf16(qb), Hn.to_dev_bf16(kb), Hn.to_dev_bf16(vb)
    out = torch.empty_like(q)
    lse = torch.empty((H, n_q), dtype=torch.float32, device="cuda") if want_lse else None
    n_keys = sum(n for _, n in segs)
    wsb = P.chunk_attention_workspace_bytes(n_q, H, n_keys)
    ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device="cuda")
    P.chunk_attention(q, n_q, H, k, v, cap, segs, P.CROPE_SCALE_FOLDED if folded else Hn.SCALE, out, lse, ws, wsb)
    torch.cuda.synchronize()
    kf, vf = Hn.bits_to_f64(kb), Hn.bits_to_f64(vb)
    kk = np.concatenate([kf[s:s + n] for s, n in segs])
    vv = np.concatenate([vf[s:s + n] for s, n in segs])
    o_ref, lse_ref = oracle.attention(q_ref, kk, vv, Hn.SCALE)
    got = Hn.bits_to_f64(Hn.dev_bits(out))
    return got, o_ref, (lse.cpu().numpy().astype(np.float64) if want_lse else None), lse_ref


@pytest.mark.parametrize("segs", [
    [(300, 70), (0, 33), (100, 129), (250, 5)],     # four segments, all ragged, out of order
    [(10, 63), (200, 1)],                           # 64 keys split 63 + 1 across a tile
    [(5, 64), (100, 64), (300, 64)],                # tile-aligned lengths, unaligned starts
    [(0, 1), (1, 1), (2, 1), (3, 1)],               # four one-key segments
    # key 0 -> row 100 and key 63 -> row 163 are 63 rows apart, but the rows between them are
    # not consecutive (keys 32..47 live in rows 0..15): the tile must not be copied as one run
    [(100, 32), (0, 16), (148, 16)],
    [(64, 16), (0, 32), (112, 16), (200, 70)],      # the same trap with a fourth segment behind it
])
@FOLDED
def test_attention_segment_shapes(P, segs, folded):
    print("case segs", segs, "folded", folded, flush=True)
    got, ref, lse, lse_ref = _attn_case(P, 77, 3, 400, segs, seed=31, folded=folded)
    Hn.assert_close("o", got, ref)
    assert np.max(np.abs(lse - lse_ref)) <= 2e-2


@pytest.mark.parametrize("n_q", [1, 31, 32, 33, 127, 129, 255, 257])
@FOLDED
def test_attention_query_counts(P, n_q, folded):
    print("case n_q", n_q, "folded", folded, flush=True)
    got, ref, lse, lse_ref = _attn_case(P, n_q, 2, 333, [(3, 330)], seed=32 + n_q, folded=folded)
    Hn.assert_close("o", got, ref)
    assert np.max(np.abs(lse - lse_ref)) <= 2e-2


@FOLDED
def test_attention_extreme_logits(P, folded):
    """Scores spanning hundreds of powers of two: the reference maximum is raised again and
    again (also by far more than one step), and the softmax saturates.  Scores are exact in
    fp32 (bf16 inputs, fp32 accumulation), so even here only the bf16 rounding of P and O
    separates the kernel from the oracle."""
    for q_scale, seed in ((40.0, 40), (6.0, 42)):
        got, ref, lse, lse_ref = _attn_case(P, 70, 2, 1000, [(0, 1000)], seed=seed, q_scale=q_scale, folded=folded)
        assert np.all(np.isfinite(got)) and np.all(np.isfinite(lse))
        max_abs, rel_l2, _ = Hn.errors(got, ref)
        print("q_scale %g: max_abs %.3e rel_l2 %.3e" % (q_scale, max_abs, rel_l2), flush=True)
        Hn.assert_close("o", got, ref)
        assert np.max(np.abs(lse - lse_ref) / np.maximum(1.0, np.abs(lse_ref))) <= 2e-3


@FOLDED
def test_attention_increasing_scores(P, folded):
    """Keys ordered so that later blocks always beat earlier ones (worst case for a lazily
    raised reference)."""
    import torch
    import oracle
    rng = np.random.default_rng(41)
    H, n_q, n_k = 1, 40, 640
    base = rng.standard_normal((1, H, 128)).astype(np.float32)
    qb = W.f32_to_bf16_bits(np.repeat(base, n_q, axis=0) * 3.0)
    ramp = np.linspace(-4.0, 4.0, n_k, dtype=np.float32)[:, None, None]
    kb = W.f32_to_bf16_bits(base * ramp + 0.05 * rng.standard_normal((n_k, H, 128)).astype(np.float32))
    vb = _rand_bits(rng, (n_k, H, 128))
    q_ref = Hn.bits_to_f64(qb)
    if folded:
        qb, q_ref = _folded_q(P, qb)
    q, k, v = Hn.to_dev_bf16(qb), Hn.to_dev_bf16(kb), Hn.to_dev_bf16(vb)
    out = torch.empty_like(q)
    wsb = P.chunk_attention_workspace_bytes(n_q, H, n_k)
    ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device="cuda")
    P.chunk_attention(q, n_q, H, k, v, n_k, [(0, n_k)], P.CROPE_SCALE_FOLDED if folded else Hn.SCALE, out, None,
                      ws, wsb)
    torch.cuda.synchronize()
    o_ref, _ = oracle.attention(q_ref, Hn.bits_to_f64(kb), Hn.bits_to_f64(vb), Hn.SCALE)
    Hn.assert_close("o", Hn.bits_to_f64(Hn.dev_bits(out)), o_ref)


@pytest.mark.parametrize("H", [1, 7, 16, 24, 33, 64])
def test_rope_head_counts(P, H):
    print("case heads", H, flush=True)
    cfg = W.ChunkConfig("RH%d" % H, 50 + H, H, 3, 5, start_frame=2, n_frames=2, first_kv_frame=2)
    inp = W.make_inputs(cfg)
    for group in (H * 128, 128):
        ref = Hn.oracle_chain(cfg, inp, norm_group=group)
        got = Hn.hip_chain(cfg, inp, norm_group=group)
        Hn.assert_close("q_rot", got["q_rot"], ref["q_rot"])
        Hn.assert_close("k_cache", got["k_cache"], ref["k_cache"])
        assert np.array_equal(got["v_cache_bits"], inp.v)
        Hn.assert_close("o", got["o"], ref["o"])


@pytest.mark.parametrize("H", [16, 21, 40, 64])
def test_rope_many_tokens_of_many_heads(P, H):
    """More than 2048 tokens of 16..64 heads: one wave walks a whole row in up to 16 rounds
    (below that token count such head counts take the four-waves-per-row kernel)."""
    print("case heads", H, "tokens 2100", flush=True)
    cfg = W.ChunkConfig("RM%d" % H, 80 + H, H, 30, 35, start_frame=1, n_frames=2, first_kv_frame=1)
    assert cfg.n_q == 2100
    inp = W.make_inputs(cfg)
    rows = [0, 1049, 1050, 2099]
    for group in (H * 128, 128):
        ref = Hn.oracle_chain(cfg, inp, norm_group=group, q_rows=rows)
        got = Hn.hip_chain(cfg, inp, norm_group=group)
        Hn.assert_close("q_rot", got["q_rot"], ref["q_rot"])
        Hn.assert_close("k_cache", got["k_cache"], ref["k_cache"])
        assert np.array_equal(got["v_cache_bits"], inp.v)
        Hn.assert_close("o", got["o"][rows], ref["o"])


@pytest.mark.parametrize("grid,frames,label", [((30, 52), 3, "three tokens per wave, streaming stores"),
                                               ((40, 60), 1, "two tokens per wave"),
                                               ((60, 104), 3, "one token per wave, write-back stores (172 MB)")])
@pytest.mark.parametrize("per_head", [False, True], ids=["normHD", "normD"])
def test_rope_launch_shapes_both_norms(P, grid, frames, label, per_head):
    """The append kernel picks tokens per wave and the store policy from the launch size; every
    such shape with both norm readings, every element of q~ and of the written cache rows."""
    print("case", grid, frames, label, "per_head", per_head, flush=True)
    cfg = W.ChunkConfig("RL%dx%d" % grid, 95 + grid[0], 12, grid[0], grid[1], start_frame=0, n_frames=frames,
                        first_kv_frame=0)
    group = 128 if per_head else 12 * 128
    inp = W.make_inputs(cfg)
    got = Hn.hip_chain(cfg, inp, norm_group=group, want_lse=False, folded=True)
    import oracle
    q_ref = oracle.qk_norm_rotate(Hn.bits_to_f64(inp.q), inp.gain_q, cfg.eps, group, cfg.dims, cfg.theta,
                                  cfg.grid_h, cfg.grid_w, 0, 0)
    k_ref = oracle.qk_norm_rotate(Hn.bits_to_f64(inp.k), inp.gain_k, cfg.eps, group, cfg.dims, cfg.theta,
                                  cfg.grid_h, cfg.grid_w, 0, 0)
    Hn.assert_close("q_rot", got["q_rot"], q_ref)
    Hn.assert_close("k_cache", got["k_cache"], k_ref)
    assert np.array_equal(got["v_cache_bits"], inp.v)


def test_rope_far_time_positions(P):
    """Frames near the end of a 1024-entry time table: angles of ~1000 rad must still be
    accurate (they are formed in fp64 when the table is built)."""
    cfg = W.ChunkConfig("FAR", 61, 2, 4, 6, start_frame=1020, n_frames=3, first_kv_frame=1020)
    inp = W.make_inputs(cfg)
    ref = Hn.oracle_chain(cfg, inp)
    got = Hn.hip_chain(cfg, inp)
    Hn.assert_close("q_rot", got["q_rot"], ref["q_rot"])
    Hn.assert_close("k_cache", got["k_cache"], ref["k_cache"])


def test_rope_rejects_frame_beyond_table(P):
    import paper_2603_06664_amd as pkg
    cfg = W.ChunkConfig("OOR", 62, 2, 4, 6, start_frame=1022, n_frames=3, first_kv_frame=1022)
    inp = W.make_inputs(cfg)
    with pytest.raises(pkg.CropeError) as ei:
        Hn.hip_chain(cfg, inp)
    assert ei.value.code == -4


@pytest.mark.parametrize("plan", [(4, 0), (8, 0), (4, 3), (8, 7), (0, 2), (4, 16)])
@FOLDED
def test_forced_plans(P, plan, folded):
    """The work-group shape and the key split are normally chosen by the library; reach the
    other shapes through chunk_attention_planned and compare each with the oracle."""
    import torch
    for cfg in (W.ChunkConfig("V1", 71, 3, 9, 11, start_frame=6, n_frames=3, first_kv_frame=0),
                W.ChunkConfig("V2", 72, 2, 4, 6, start_frame=7, n_frames=1, first_kv_frame=5, cache_frames=3)):
        print("case", cfg.name, "plan", plan, "folded", folded, flush=True)
        inp = W.make_inputs(cfg)
        ref = Hn.oracle_chain(cfg, inp)
        from paper_2603_06664_amd.devutil import StepBuffers
        sb = StepBuffers(cfg, inp, folded=folded)
        scale = P.CROPE_SCALE_FOLDED if folded else Hn.SCALE
        sb.append()
        resolved = P.chunk_attention_choose_plan(cfg.n_q, cfg.n_heads, sb.n_keys, plan)
        assert resolved[0] in (4, 8) and 1 <= resolved[1] <= 16
        if plan[0]:
            assert resolved[0] == plan[0]
        n_tiles = (sb.n_keys + 63) // 64
        if plan[1]:
            assert resolved[1] == plan[1] or plan[1] > n_tiles or (plan[1] - 1) * -(-n_tiles // plan[1]) >= n_tiles
        wsb = P.chunk_attention_planned_workspace_bytes(cfg.n_q, cfg.n_heads, sb.n_keys, plan)
        assert (wsb == 0) == (resolved[1] == 1)
        ws = torch.empty(max(wsb, 16), dtype=torch.uint8, device="cuda")
        P.chunk_attention_planned(sb.q_rot, cfg.n_q, cfg.n_heads, sb.k_cache, sb.v_cache, sb.cap, sb.segs,
                                  scale, plan, sb.out, sb.lse, ws, wsb)
        torch.cuda.synchronize()
        Hn.assert_close("o", Hn.bits_to_f64(Hn.dev_bits(sb.out)), ref["o"])
        assert np.max(np.abs(sb.lse.cpu().numpy().astype(np.float64) - ref["lse"])) <= 2e-2
        if wsb:   # a split plan with too little workspace is refused
            with pytest.raises(P.CropeError) as ei:
                P.chunk_attention_planned(sb.q_rot, cfg.n_q, cfg.n_heads, sb.k_cache, sb.v_cache, sb.cap,
                                          sb.segs, scale, plan, sb.out, sb.lse, ws, wsb - 16)
            assert ei.value.code == -5


def _limited_case(P, n_q, H, n_k, limits, seed, folded=False):
    import torch
    import oracle
    rng = np.random.default_rng(seed)
    qb, kb, vb = _rand_bits(rng, (n_q, H, 128)), _rand_bits(rng, (n_k, H, 128)), _rand_bits(rng, (n_k, H, 128))
    q_ref = Hn.bits_to_f64(qb)
    if folded:
        qb, q_ref = _folded_q(P, qb)
    q, k, v = Hn.to_dev_bf16(qb), Hn.to_dev_bf16(kb), Hn.to_dev_bf16(vb)
    out = torch.empty_like(q)
    lse = torch.empty((H, n_q), dtype=torch.float32, device="cuda")
    lim = torch.from_numpy(np.asarray(limits, dtype=np.int32)).cuda()
    P.chunk_attention_limited(q, n_q, H, k, v, n_k, [(0, n_k)], P.CROPE_SCALE_FOLDED if folded else Hn.SCALE, lim,
                              out, lse)
    torch.cuda.synchronize()
    # oracle: key m visible to query i iff m < limit_i  <=>  k_block[m] = m <= q_block[i] = limit_i - 1
    lim_c = np.clip(np.asarray(limits), 1, n_k)
    o_ref, lse_ref = oracle.attention(q_ref, Hn.bits_to_f64(kb), Hn.bits_to_f64(vb), Hn.SCALE,
                                      q_block=(lim_c - 1).astype(np.int32), k_block=np.arange(n_k, dtype=np.int32))
    return Hn.bits_to_f64(Hn.dev_bits(out)), o_ref, lse.cpu().numpy().astype(np.float64), lse_ref


@pytest.mark.parametrize("kind", ["block_causal", "token_causal", "ragged", "clamped", "block_causal_long"])
@FOLDED
def test_attention_with_per_query_limits(P, kind, folded):
    """One pass over a whole sequence with the generator's block-causal rule (and other prefix
    masks) against the oracle's masked attention."""
    print("case", kind, flush=True)
    n = 1500 if kind == "block_causal_long" else 600
    i = np.arange(n)
    if kind == "block_causal_long":
        limits = (i // 333 + 1) * 333          # block ends inside key tiles; many unmasked tiles below them
    elif kind == "block_causal":
        limits = (i // 150 + 1) * 150          # blocks of 150 tokens: query sees up to the end of its block
    elif kind == "token_causal":
        limits = i + 1
    elif kind == "ragged":
        limits = np.random.default_rng(7).integers(1, n + 1, size=n)
    else:
        limits = np.where(i % 2 == 0, 0, 10 * n)   # out-of-range values are clamped to [1, n]
    got, ref, lse, lse_ref = _limited_case(P, n, 3, n, limits, seed=80, folded=folded)
    Hn.assert_close("o", got, ref)
    assert np.max(np.abs(lse - lse_ref)) <= 2e-2


def test_one_shot_block_causal_equals_streaming_on_gpu(P):
    """Streaming == one-shot on the device: generating three blocks one at a time with the
    cache gives the same outputs as ONE limited call over the whole sequence."""
    import torch
    cfg_blocks = [W.ChunkConfig("OS%d" % b, 90, 3, 6, 8, start_frame=3 * b, n_frames=3, first_kv_frame=0)
                  for b in range(3)]
    last = cfg_blocks[-1]
    inp = W.make_inputs(last)                   # k, v for all 9 frames; q for the last block only
    rng = np.random.default_rng(91)
    hw, H = last.hw, last.n_heads
    q_all = W.f32_to_bf16_bits(rng.standard_normal((9 * hw, H, 128), dtype=np.float32))
    streamed = []
    for b, cfg in enumerate(cfg_blocks):
        sub = W.ChunkInputs(cfg, q_all[3 * b * hw:3 * (b + 1) * hw], inp.k[:3 * (b + 1) * hw],
                            inp.v[:3 * (b + 1) * hw], inp.gain_q, inp.gain_k)
        streamed.append(Hn.hip_chain(cfg, sub)["o"])
    streamed = np.concatenate(streamed, axis=0)
    # one shot: rotate everything with s = 0, then one limited attention call
    desc, tab = Hn.make_table()
    n = 9 * hw
    q, k, v = Hn.to_dev_bf16(q_all), Hn.to_dev_bf16(inp.k), Hn.to_dev_bf16(inp.v)
    gq, gk = torch.from_numpy(inp.gain_q).cuda(), torch.from_numpy(inp.gain_k).cuda()
    qo, kc, vc = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    P.crope_qk_norm_rotate_append(desc, tab, q, k, v, gq, gk, 1e-6, H * 128, n, H, last.grid_h, last.grid_w,
                                  0, 0, qo, kc, vc, n, 0)
    limits = torch.from_numpy(((np.arange(n) // (3 * hw) + 1) * 3 * hw).astype(np.int32)).cuda()
    out = torch.empty_like(qo)
    P.chunk_attention_limited(qo, n, H, kc, vc, n, [(0, n)], Hn.SCALE, limits, out)
    torch.cuda.synchronize()
    one_shot = Hn.bits_to_f64(Hn.dev_bits(out))
    # both sides are bf16 results of the same exact scores; they differ by rounding order only
    Hn.assert_close("one-shot vs streamed", one_shot, streamed)
