"""Parity of the HIP path (through the C ABI) against the fp64 CPU oracle.

Small shapes are compared element by element on every output; so are the full-size
benchmark configurations (rotated q, rotated-k cache, v cache, attention output and LSE of
every query row), except the 960x1664 workload, whose attention output is compared on a
sample of query rows that covers tile edges (the oracle would need minutes for all of it).
"""
import dataclasses

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
    binding._load()   # fail loudly if the HIP library is missing
    return pkg


def _say(msg):
    print(msg, flush=True)


# ------------------------------------------------------------------ tables
def test_tables_match_oracle(P):
    import oracle
    desc, tab = Hn.make_table(P.TableDesc(max_t=1024, max_h=128, max_w=128))
    t = tab.cpu().numpy().astype(np.float64)
    off = 0
    for dim_a, n_pos in ((44, 1024), (42, 128), (42, 128)):
        ref = oracle.axis_table(dim_a, 10000.0, n_pos)
        got = t[off:off + ref.size].reshape(ref.shape)
        off += ref.size
        assert np.max(np.abs(got - ref)) <= 1e-5
        assert np.sqrt(((got - ref) ** 2).sum() / (ref ** 2).sum()) <= 1e-5
        assert np.all(got[0, :, 0] == 1.0) and np.all(got[0, :, 1] == 0.0)   # exact at position 0
    assert off == t.size


# ------------------------------------------------------------------ small shapes, every element
SMALL = [
    W.CONFIGS["C1"],
    # three 3-frame blocks on a 5x7 grid: 105 queries, 315 keys (ragged in both tile sizes)
    W.ChunkConfig("S1", 11, 3, 5, 7, start_frame=6, n_frames=3, first_kv_frame=0),
    # one-frame chunks on a 10x15 grid: 150 queries (two query tiles), 5 frames of keys
    W.ChunkConfig("S2", 12, 5, 10, 15, start_frame=4, n_frames=1, first_kv_frame=0),
    # ring of 3 frames that has wrapped: frames 5,6,7 sit in slots 2,0,1 -> two segments
    W.ChunkConfig("S3", 13, 4, 6, 9, start_frame=7, n_frames=1, first_kv_frame=5, cache_frames=3),
    # first chunk, single head, key count == one tile exactly (64)
    W.ChunkConfig("S4", 14, 1, 8, 8, start_frame=0, n_frames=1, first_kv_frame=0),
    # 65 keys: one full tile plus one key
    W.ChunkConfig("S5", 15, 2, 5, 13, start_frame=0, n_frames=1, first_kv_frame=0),
    # a sharded call: rank 1 of 4 with a shard that straddles a frame boundary, 40 heads
    W.ChunkConfig("S6", 16, 40, 4, 5, start_frame=3, n_frames=3, first_kv_frame=0,
                  token_offset=15, n_local=15),
    # k gain scaled per head (wide logit range)
    W.ChunkConfig("S7", 17, 6, 6, 6, start_frame=3, n_frames=3, first_kv_frame=0, k_head_scale=True),
]


@pytest.mark.parametrize("cfg", SMALL, ids=[c.name for c in SMALL])
@pytest.mark.parametrize("per_head", [False, True], ids=["normHD", "normD"])
@pytest.mark.parametrize("folded", [False, True], ids=["scale", "folded"])
def test_small_config_every_element(P, cfg, per_head, folded):
    _say("case %s per_head=%s folded=%s" % (cfg.name, per_head, folded))
    group = cfg.head_dim if per_head else cfg.n_heads * cfg.head_dim
    inp = W.make_inputs(cfg)
    ref = Hn.oracle_chain(cfg, inp, norm_group=group)
    got = Hn.hip_chain(cfg, inp, norm_group=group, folded=folded)
    assert got["segs"] == ref["segs"]
    Hn.assert_close("q_rot", got["q_rot"], ref["q_rot"])
    Hn.assert_close("k_cache", got["k_cache"], ref["k_cache"])
    # v is a copy: bit-exact
    v_ref = np.zeros_like(got["v_cache_bits"])
    for (s, nf, row0, n, off, _) in W.chunk_schedule(cfg):
        d = Hn.dst_row(cfg, s, off)
        v_ref[d:d + n] = inp.v[row0:row0 + n]
    assert np.array_equal(got["v_cache_bits"], v_ref)
    Hn.assert_close("o", got["o"], ref["o"])
    assert np.max(np.abs(got["lse"] - ref["lse"])) <= 2e-2


# ------------------------------------------------------------------ full-size configurations
def _sample_rows(n_q, rng, count=40):
    edges = [0, 1, 31, 32, 63, 64, 127, 128, 129, 255, 256, n_q - 1, n_q - 2,
             (n_q // 128) * 128 - 1, (n_q // 128) * 128, n_q // 2]
    rows = sorted({r for r in edges if 0 <= r < n_q} |
                  {int(r) for r in rng.integers(0, n_q, size=count)})
    return rows


# the benchmark's pairing (q written with the softmax factor folded in) at every workload; the
# plain pairing (explicit scale) at the headline workload and the split-key one
@pytest.mark.parametrize("name,folded", [("C2", True), ("C3", True), ("C4", True), ("C5", True), ("R288", True),
                                         ("C5P", True), ("C4R", True), ("R960", True), ("C4", False),
                                         ("C5", False)])
def test_full_size_config(P, name, folded):
    cfg = W.CONFIGS[name]
    _say("case %s folded=%s: n_q=%d n_keys=%d heads=%d" % (name, folded, cfg.n_q, cfg.n_keys, cfg.n_heads))
    inp = W.make_inputs(cfg)
    # every query row; only the largest workload is sampled
    rows = _sample_rows(cfg.n_q, np.random.default_rng(100 + cfg.seed)) if name == "R960" else list(range(cfg.n_q))
    got = Hn.hip_chain(cfg, inp, folded=folded)
    _say("  hip path done")
    ref = Hn.oracle_chain(cfg, inp, q_rows=rows)
    _say("  oracle done (%d of %d query rows)" % (len(rows), cfg.n_q))
    e = Hn.assert_close("q_rot", got["q_rot"], ref["q_rot"])
    _say("  q_rot   max_abs %.3e rel_l2 %.3e" % e)
    e = Hn.assert_close("k_cache", got["k_cache"], ref["k_cache"])
    _say("  k_cache max_abs %.3e rel_l2 %.3e" % e)
    v_ref = np.zeros_like(got["v_cache_bits"])
    for (s_, nf, row0, n, off, _) in W.chunk_schedule(cfg):
        for f in range(nf):      # frame by frame: a ring slot holds one frame
            lo = max(off, f * cfg.hw)
            hi = min(off + n, (f + 1) * cfg.hw)
            if lo < hi:
                d = W.cache_slot(cfg, s_ + f) * cfg.hw + (lo - f * cfg.hw)
                v_ref[d:d + hi - lo] = inp.v[row0 + lo - off:row0 + hi - off]
    assert np.array_equal(got["v_cache_bits"], v_ref)
    e = Hn.assert_close("o", got["o"][rows], ref["o"])
    _say("  o       max_abs %.3e rel_l2 %.3e" % e)
    lse_err = np.max(np.abs(got["lse"][:, rows] - ref["lse"]))
    _say("  lse     max_abs %.3e" % lse_err)
    assert lse_err <= 2e-2
    # property that holds at any size: outputs are convex combinations of the values
    v = Hn.bits_to_f64(inp.v)
    lo, hi = v.min(axis=0), v.max(axis=0)
    assert np.all(got["o"] >= lo[None] - 1e-2) and np.all(got["o"] <= hi[None] + 1e-2)


# ------------------------------------------------------------------ method properties on the GPU
def test_shard_equals_slice_bitwise(P):
    """Section 3.3.3 on the device: every rank's local call reproduces its rows of the
    whole-chunk call exactly (P = 8, shard size 75 straddles frame and row boundaries)."""
    import torch
    cfg = W.ChunkConfig("T1", 21, 4, 10, 20, start_frame=9, n_frames=3, first_kv_frame=9)
    inp = W.make_inputs(cfg)
    desc, tab = Hn.make_table()
    H, D, n = cfg.n_heads, 128, cfg.chunk_tokens
    q, k, v = (Hn.to_dev_bf16(a) for a in (inp.q, inp.k, inp.v))
    gq, gk = torch.from_numpy(inp.gain_q).cuda(), torch.from_numpy(inp.gain_k).cuda()

    def run(shards):
        qo = torch.zeros_like(q)
        kc = torch.zeros_like(k)
        vc = torch.zeros_like(v)
        n_loc = n // shards
        for r in range(shards):
            d = r * n_loc
            P.crope_qk_norm_rotate_append(desc, tab, q[d:d + n_loc], k[d:d + n_loc], v[d:d + n_loc],
                                          gq, gk, 1e-6, H * D, n_loc, H, cfg.grid_h, cfg.grid_w,
                                          cfg.start_frame, d, qo[d:d + n_loc], kc, vc, n, d)
        torch.cuda.synchronize()
        return Hn.dev_bits(qo), Hn.dev_bits(kc), Hn.dev_bits(vc)

    whole = run(1)
    for shards in (2, 4, 8):
        part = run(shards)
        for a, b in zip(whole, part):
            assert np.array_equal(a, b)


def test_frame_shift_invariance_on_gpu(P):
    """Shifting every global frame index by a constant changes no attention output beyond
    bf16 rounding (rotated keys stay valid in a rolling cache)."""
    base = W.ChunkConfig("T4", 22, 3, 6, 8, start_frame=3, n_frames=3, first_kv_frame=0)
    inp = W.make_inputs(base)
    a = Hn.hip_chain(base, inp)
    shifted = dataclasses.replace(base, start_frame=3 + 30, first_kv_frame=30)
    inp2 = dataclasses.replace(inp, cfg=shifted)
    b = Hn.hip_chain(shifted, inp2)
    Hn.assert_close("o shifted", b["o"], a["o"])


def test_runs_are_bitwise_deterministic(P):
    cfg = SMALL[1]
    inp = W.make_inputs(cfg)
    a = Hn.hip_chain(cfg, inp)
    b = Hn.hip_chain(cfg, inp)
    for key in ("q_rot", "k_cache", "o", "lse"):
        assert np.array_equal(a[key], b[key]), key


def test_strided_inputs_and_outputs(P):
    """q, k, v as slices of one fused [token][3][head][128] projection buffer, and caches
    with a padded head stride."""
    import torch
    import oracle
    cfg = W.ChunkConfig("ST", 23, 3, 4, 6, start_frame=2, n_frames=1, first_kv_frame=2)
    inp = W.make_inputs(cfg)
    n, H, D = cfg.n_q, cfg.n_heads, 128
    fused = torch.empty((n, 3, H, D), dtype=torch.bfloat16, device="cuda")
    fused[:, 0] = Hn.to_dev_bf16(inp.q)
    fused[:, 1] = Hn.to_dev_bf16(inp.k)
    fused[:, 2] = Hn.to_dev_bf16(inp.v)
    desc, tab = Hn.make_table()
    gq, gk = torch.from_numpy(inp.gain_q).cuda(), torch.from_numpy(inp.gain_k).cuda()
    cache = torch.zeros((2, n + 8, H, D + 64), dtype=torch.bfloat16, device="cuda")
    kc, vc = cache[0, :, :, :D], cache[1, :, :, :D]
    qo = torch.empty((n, H, D), dtype=torch.bfloat16, device="cuda")
    P.crope_qk_norm_rotate_append(desc, tab, fused[:, 0], fused[:, 1], fused[:, 2], gq, gk, 1e-6,
                                  H * D, n, H, cfg.grid_h, cfg.grid_w, 2, 0, qo, kc, vc, n + 8, 8)
    out = torch.empty((n, H, D + 16), dtype=torch.bfloat16, device="cuda")[:, :, :D]
    P.chunk_attention(qo, n, H, kc, vc, n + 8, [(8, n)], Hn.SCALE, out)
    torch.cuda.synchronize()
    q_ref = oracle.qk_norm_rotate(Hn.bits_to_f64(inp.q), inp.gain_q, 1e-6, H * D, cfg.dims, cfg.theta,
                                  4, 6, 2)
    k_ref = oracle.qk_norm_rotate(Hn.bits_to_f64(inp.k), inp.gain_k, 1e-6, H * D, cfg.dims, cfg.theta,
                                  4, 6, 2)
    o_ref, _ = oracle.attention(q_ref, k_ref, Hn.bits_to_f64(inp.v), Hn.SCALE)
    Hn.assert_close("k strided", Hn.bits_to_f64(Hn.dev_bits(kc[8:])), k_ref)
    assert np.array_equal(Hn.dev_bits(vc[8:]), inp.v)
    assert float(cache[:, :8].abs().max()) == 0.0 and float(cache[..., D:].abs().max()) == 0.0
    Hn.assert_close("o strided", Hn.bits_to_f64(Hn.dev_bits(out)), o_ref)


def test_single_key_and_single_query(P):
    import torch
    import oracle
    rng = np.random.default_rng(5)
    H, D = 2, 128
    qb = W.f32_to_bf16_bits(rng.standard_normal((1, H, D), dtype=np.float32))
    kb = W.f32_to_bf16_bits(rng.standard_normal((130, H, D), dtype=np.float32))
    vb = W.f32_to_bf16_bits(rng.standard_normal((130, H, D), dtype=np.float32))
    q, k, v = Hn.to_dev_bf16(qb), Hn.to_dev_bf16(kb), Hn.to_dev_bf16(vb)
    out = torch.empty_like(q)
    P.chunk_attention(q, 1, H, k, v, 130, [(7, 1)], Hn.SCALE, out)      # one visible key
    torch.cuda.synchronize()
    assert np.array_equal(Hn.dev_bits(out), vb[7:8])                     # o == v exactly
    P.chunk_attention(q, 1, H, k, v, 130, [(0, 130)], Hn.SCALE, out)
    torch.cuda.synchronize()
    o_ref, _ = oracle.attention(Hn.bits_to_f64(qb), Hn.bits_to_f64(kb), Hn.bits_to_f64(vb), Hn.SCALE)
    Hn.assert_close("o 1 query", Hn.bits_to_f64(Hn.dev_bits(out)), o_ref)


def test_canaries_around_outputs_survive(P):
    """Nothing is written outside [dst, dst+n) of the caches or past the end of out."""
    import torch
    cfg = W.ChunkConfig("CN", 24, 3, 5, 7, start_frame=0, n_frames=1, first_kv_frame=0)
    inp = W.make_inputs(cfg)
    n, H, D = cfg.n_q, cfg.n_heads, 128
    desc, tab = Hn.make_table()
    q, k, v = (Hn.to_dev_bf16(a) for a in (inp.q, inp.k, inp.v))
    gq, gk = torch.from_numpy(inp.gain_q).cuda(), torch.from_numpy(inp.gain_k).cuda()
    cap = n + 20
    kc = torch.full((cap, H, D), 7.0, dtype=torch.bfloat16, device="cuda")
    vc = torch.full((cap, H, D), 7.0, dtype=torch.bfloat16, device="cuda")
    qo = torch.full((n + 10, H, D), 7.0, dtype=torch.bfloat16, device="cuda")
    P.crope_qk_norm_rotate_append(desc, tab, q, k, v, gq, gk, 1e-6, H * D, n, H, 5, 7, 0, 0,
                                  qo[:n], kc, vc, cap, 10)
    out = torch.full((n + 10, H, D), 7.0, dtype=torch.bfloat16, device="cuda")
    P.chunk_attention(qo[:n], n, H, kc, vc, cap, [(10, n)], Hn.SCALE, out[:n])
    torch.cuda.synchronize()
    for t in (kc[:10], kc[10 + n:], vc[:10], vc[10 + n:], qo[n:], out[n:]):
        assert bool((t == 7.0).all())
