"""Pins for the oracle's softmax attention and cache semantics (CPU only)."""
import numpy as np
import pytest
from scipy.special import softmax as scipy_softmax

import oracle

DIMS = (44, 42, 42)
THETA = 10000.0
SCALE = 128 ** -0.5


def _rng(seed):
    return np.random.default_rng(seed)


def test_rows_of_p_sum_to_one_and_lse():
    q = _rng(0).standard_normal((24, 2, 128))
    k = _rng(1).standard_normal((72, 2, 128)) * 2.0
    v = _rng(2).standard_normal((72, 2, 128))
    o, lse, P = oracle.attention(q, k, v, SCALE, return_p=True)
    assert np.max(np.abs(P.sum(-1) - 1.0)) < 1e-14
    assert np.all(P >= 0)
    s = SCALE * np.einsum("ihd,jhd->hij", q, k)
    assert np.allclose(lse, np.log(np.exp(s).sum(-1)), rtol=1e-13)
    # explicit-P brute force for the output
    assert np.max(np.abs(o - np.einsum("hij,jhd->ihd", P, v))) < 1e-13


def test_matches_scipy_softmax_one_liner():
    q = _rng(3).standard_normal((17, 3, 128))
    k = _rng(4).standard_normal((53, 3, 128))
    v = _rng(5).standard_normal((53, 3, 128))
    o, _ = oracle.attention(q, k, v, SCALE)
    ref = np.einsum("hij,jhd->ihd",
                    scipy_softmax(SCALE * np.einsum("ihd,jhd->hij", q, k), axis=-1), v)
    assert np.max(np.abs(o - ref)) < 1e-13


def test_matches_torch_sdpa_fp64():
    torch = pytest.importorskip("torch")
    q = _rng(6).standard_normal((20, 2, 128))
    k = _rng(7).standard_normal((45, 2, 128))
    v = _rng(8).standard_normal((45, 2, 128))
    tq, tk, tv = (torch.from_numpy(a).permute(1, 0, 2)[None] for a in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)[0].permute(1, 0, 2).numpy()
    o, _ = oracle.attention(q, k, v, SCALE)   # torch's default scale is 1/sqrt(D) too
    assert np.max(np.abs(o - ref)) < 1e-12


def test_single_key_returns_its_value():
    q = _rng(9).standard_normal((5, 2, 128))
    k = _rng(10).standard_normal((1, 2, 128))
    v = _rng(11).standard_normal((1, 2, 128))
    o, lse = oracle.attention(q, k, v, SCALE)
    assert np.array_equal(o, np.broadcast_to(v, o.shape))
    assert np.allclose(lse, SCALE * np.einsum("ihd,jhd->hi", q, k), rtol=1e-14)


def test_identical_keys_give_mean_of_values():
    q = _rng(12).standard_normal((4, 2, 128))
    k = np.broadcast_to(_rng(13).standard_normal((1, 2, 128)), (9, 2, 128))
    v = _rng(14).standard_normal((9, 2, 128))
    o, _ = oracle.attention(q, k, v, SCALE)
    assert np.allclose(o, np.broadcast_to(v.mean(0), o.shape), atol=1e-14)


def test_key_permutation_invariance():
    q = _rng(15).standard_normal((6, 2, 128))
    k = _rng(16).standard_normal((31, 2, 128))
    v = _rng(17).standard_normal((31, 2, 128))
    perm = _rng(18).permutation(31)
    o1, l1 = oracle.attention(q, k, v, SCALE)
    o2, l2 = oracle.attention(q, k[perm], v[perm], SCALE)
    assert np.max(np.abs(o1 - o2)) < 1e-14 and np.max(np.abs(l1 - l2)) < 1e-13


def test_heads_are_independent_and_not_transposed():
    # head 1 of k and v is garbage: head 0's output must not change
    q = _rng(19).standard_normal((6, 2, 128))
    k = _rng(20).standard_normal((11, 2, 128))
    v = _rng(21).standard_normal((11, 2, 128))
    o1, _ = oracle.attention(q, k, v, SCALE)
    k2, v2 = k.copy(), v.copy()
    k2[:, 1] = 7.0
    v2[:, 1] = -3.0
    o2, _ = oracle.attention(q, k2, v2, SCALE)
    assert np.array_equal(o1[:, 0], o2[:, 0])
    assert np.allclose(o2[:, 1], -3.0)


def test_large_logits_are_stable():
    q = _rng(22).standard_normal((3, 1, 128)) * 40
    k = _rng(23).standard_normal((50, 1, 128)) * 40
    v = _rng(24).standard_normal((50, 1, 128))
    o, lse = oracle.attention(q, k, v, 1.0)
    assert np.all(np.isfinite(o)) and np.all(np.isfinite(lse))
    # softmax saturates: output equals the value of the arg-max key
    s = np.einsum("ihd,jhd->hij", q, k)[0]
    assert np.allclose(o[:, 0], v[np.argmax(s, -1), 0], atol=1e-9)


def test_block_mask_matches_torch_masked_sdpa():
    torch = pytest.importorskip("torch")
    q = _rng(25).standard_normal((12, 2, 128))
    k = _rng(26).standard_normal((12, 2, 128))
    v = _rng(27).standard_normal((12, 2, 128))
    blk = np.repeat(np.arange(4), 3).astype(np.int32)
    o, _ = oracle.attention(q, k, v, SCALE, q_block=blk, k_block=blk)
    mask = torch.from_numpy(blk[None, :] <= blk[:, None])
    tq, tk, tv = (torch.from_numpy(a).permute(1, 0, 2)[None] for a in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask)[0]
    assert np.max(np.abs(o - ref.permute(1, 0, 2).numpy())) < 1e-12


def _stream(q_raw, k_raw, v, gh, gw, tau, n_blocks, capacity_frames=None, frame_shift=0):
    """Block-by-block generation with a rolling cache: rotate with s = k*tau (+shift),
    assign into the ring slot of each frame, attend over whatever the cache holds."""
    hw = gh * gw
    H, D = q_raw.shape[1:]
    cap = n_blocks * tau if capacity_frames is None else capacity_frames
    cache = oracle.Cache(cap * hw, H, D)
    held = []
    outs = []
    for b in range(n_blocks):
        s = b * tau + frame_shift
        rows = slice(b * tau * hw, (b + 1) * tau * hw)
        qr = oracle.rotate(q_raw[rows], DIMS, THETA, gh, gw, s=s)
        kr = oracle.rotate(k_raw[rows], DIMS, THETA, gh, gw, s=s)
        for f in range(tau):
            frame = b * tau + f
            slot = frame % cap
            cache.write(slot * hw, kr[f * hw:(f + 1) * hw], v[rows][f * hw:(f + 1) * hw])
            held = [g for g in held if g % cap != slot] + [frame]
        segs = [((g % cap) * hw, hw) for g in held]
        kk, vv = cache.gather(segs)
        o, _ = oracle.attention(qr, kk, vv, SCALE)
        outs.append(o)
    return np.concatenate(outs, axis=0)


def test_streaming_equals_one_shot_block_causal():
    # Generating block by block with the cache == masked attention over the whole
    # sequence with a block-causal mask of block size tau (Sections 2.1, 3.2, 3.3.2).
    gh, gw, tau, n_blocks = 2, 3, 2, 3
    hw = gh * gw
    n = n_blocks * tau * hw
    q = _rng(28).standard_normal((n, 2, 128))
    k = _rng(29).standard_normal((n, 2, 128))
    v = _rng(30).standard_normal((n, 2, 128))
    streamed = _stream(q, k, v, gh, gw, tau, n_blocks)
    qr = oracle.rotate(q, DIMS, THETA, gh, gw, s=0)
    kr = oracle.rotate(k, DIMS, THETA, gh, gw, s=0)
    blk = (np.arange(n) // (tau * hw)).astype(np.int32)
    one_shot, _ = oracle.attention(qr, kr, v, SCALE, q_block=blk, k_block=blk)
    assert np.max(np.abs(streamed - one_shot)) < 1e-12


def test_frame_shift_leaves_attention_unchanged():
    # System-level relative-position identity: shifting every global frame index by a
    # constant (current and cached alike) does not change the outputs.
    gh, gw, tau, n_blocks = 2, 3, 3, 2
    n = n_blocks * tau * gh * gw
    q = _rng(31).standard_normal((n, 2, 128))
    k = _rng(32).standard_normal((n, 2, 128))
    v = _rng(33).standard_normal((n, 2, 128))
    a = _stream(q, k, v, gh, gw, tau, n_blocks)
    b = _stream(q, k, v, gh, gw, tau, n_blocks, frame_shift=11)
    assert np.max(np.abs(a - b)) < 1e-11


def test_ring_wrap_equals_sliding_window_reference():
    # capacity 3 frames, stream 8 one-frame blocks: the ring must behave like "attend to
    # the last 3 frames", whatever slot they sit in.
    gh, gw, tau, n_blocks, cap = 2, 3, 1, 8, 3
    hw = gh * gw
    n = n_blocks * hw
    q = _rng(34).standard_normal((n, 2, 128))
    k = _rng(35).standard_normal((n, 2, 128))
    v = _rng(36).standard_normal((n, 2, 128))
    ring = _stream(q, k, v, gh, gw, tau, n_blocks, capacity_frames=cap)
    qr = oracle.rotate(q, DIMS, THETA, gh, gw, s=0)
    kr = oracle.rotate(k, DIMS, THETA, gh, gw, s=0)
    for b in range(n_blocks):
        lo = max(0, b - cap + 1) * hw
        hi = (b + 1) * hw
        ref, _ = oracle.attention(qr[b * hw:hi], kr[lo:hi], v[lo:hi], SCALE)
        assert np.max(np.abs(ring[b * hw:hi] - ref)) < 1e-12


def test_c1_oracle_values_are_stable():
    """Regression pin: sampled oracle outputs for configuration C1 match the stored values
    (written by tests/golden/make_c1_golden.py, which calls only the oracle)."""
    import importlib.util
    import os
    here = os.path.join(os.path.dirname(__file__), "golden")
    spec = importlib.util.spec_from_file_location("make_c1_golden", os.path.join(here, "make_c1_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    q_rot, k_rot, o, lse = mod.c1_outputs()
    arrays = dict(q_rot=q_rot, k_rot=k_rot, o=o, lse=lse)
    n = 0
    for ln in open(os.path.join(here, "c1_oracle_values.txt")):
        if ln.startswith("#") or not ln.strip():
            continue
        parts = ln.split()
        idx = tuple(int(x) for x in parts[1:-1])
        assert arrays[parts[0]][idx] == pytest.approx(float(parts[-1]), rel=1e-12, abs=1e-14)
        n += 1
    assert n == 15
