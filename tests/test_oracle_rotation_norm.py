"""Pins for the oracle's RMSNorm and 3D rotation (CPU only)."""
import numpy as np
import pytest

import oracle

DIMS = (44, 42, 42)
THETA = 10000.0


def _rng(seed=0):
    return np.random.default_rng(seed)


# ------------------------------------------------------------------ rotation
def test_rotation_preserves_pair_norms():
    x = _rng(1).standard_normal((3 * 4 * 6, 2, 128))
    y = oracle.rotate(x, DIMS, THETA, 4, 6, s=17)
    nx = x.reshape(-1, 64, 2)
    ny = y.reshape(-1, 64, 2)
    assert np.allclose((nx ** 2).sum(-1), (ny ** 2).sum(-1), rtol=1e-13, atol=1e-13)


def test_rotation_identity_at_origin():
    x = _rng(2).standard_normal((24, 3, 128))
    y = oracle.rotate(x, DIMS, THETA, 4, 6, s=0)
    assert np.array_equal(y[0], x[0])          # (t,h,w) = (0,0,0): exact identity
    assert not np.allclose(y[1], x[1])         # w = 1 rotates the width block ...
    assert np.array_equal(y[1][:, :86], x[1][:, :86])   # ... and only that block
    assert np.array_equal(y[6][:, 86:], x[6][:, 86:])   # (0,1,0): width block untouched
    assert np.array_equal(y[6][:, :44], x[6][:, :44])   # time block untouched
    assert not np.allclose(y[6][:, 44:86], x[6][:, 44:86])


def test_rotation_known_quarter_turn():
    # One pair, omega_0 = 1: at t = 1 the pair (1, 0) must become (cos 1, sin 1): counter-
    # clockwise, i.e. multiplication by e^{+i theta} (Section 3.3.1).
    x = np.zeros((2, 1, 2))
    x[:, 0, 0] = 1.0
    y = oracle.rotate(x, (2, 0, 0), THETA, 1, 1, s=0)   # two frames of a 1x1 grid
    assert y[1, 0, 0] == pytest.approx(np.cos(1.0), abs=1e-15)
    assert y[1, 0, 1] == pytest.approx(np.sin(1.0), abs=1e-15)
    # and (0, 1) -> (-sin 1, cos 1)
    x2 = np.zeros((2, 1, 2))
    x2[:, 0, 1] = 1.0
    y2 = oracle.rotate(x2, (2, 0, 0), THETA, 1, 1, s=0)
    assert y2[1, 0, 0] == pytest.approx(-np.sin(1.0), abs=1e-15)
    assert y2[1, 0, 1] == pytest.approx(np.cos(1.0), abs=1e-15)


def _algorithm2_bruteforce(x, dims, theta, F, gh, gw, s, max_pos=64):
    """Independent derivation with complex numbers, following Algorithm 2's structure:
    per-axis complex tables, time table sliced at [s, s+F), expanded over the (F,H,W) grid
    and concatenated along the channel axis, then one complex multiply."""
    def table(d):
        j = np.arange(d // 2)
        omega = 1.0 / theta ** (2.0 * j / d)
        return np.exp(1j * np.outer(np.arange(max_pos), omega))     # polar(1, pos*omega)
    ft, fh, fw = (table(d) for d in dims)
    freqs = np.concatenate([
        np.broadcast_to(ft[s:s + F][:, None, None, :], (F, gh, gw, dims[0] // 2)),
        np.broadcast_to(fh[:gh][None, :, None, :], (F, gh, gw, dims[1] // 2)),
        np.broadcast_to(fw[:gw][None, None, :, :], (F, gh, gw, dims[2] // 2)),
    ], axis=-1).reshape(F * gh * gw, 1, -1)
    n, H, D = x.shape
    xc = x.reshape(n, H, D // 2, 2)
    xc = xc[..., 0] + 1j * xc[..., 1]
    yc = xc * freqs
    return np.stack([yc.real, yc.imag], axis=-1).reshape(n, H, D)


@pytest.mark.parametrize("F,gh,gw,s", [(1, 4, 6, 5), (3, 4, 6, 0), (3, 3, 5, 6), (2, 1, 7, 40)])
def test_rotation_matches_algorithm2_bruteforce(F, gh, gw, s):
    x = _rng(3).standard_normal((F * gh * gw, 2, 128))
    ref = _algorithm2_bruteforce(x, DIMS, THETA, F, gh, gw, s)
    got = oracle.rotate(x, DIMS, THETA, gh, gw, s=s)
    assert np.max(np.abs(got - ref)) < 1e-12


def test_rotation_other_split_and_theta():
    x = _rng(4).standard_normal((2 * 3 * 3, 1, 16))
    ref = _algorithm2_bruteforce(x, (8, 4, 4), 100.0, 2, 3, 3, 7)
    got = oracle.rotate(x, (8, 4, 4), 100.0, 3, 3, s=7)
    assert np.max(np.abs(got - ref)) < 1e-13


@pytest.mark.parametrize("P", [1, 2, 4, 8])
def test_local_rotation_equals_slice_of_global(P):
    # Section 3.3.3: rotating a rank's shard with (s, Delta) equals the rows of rotating
    # the whole chunk.  L = 3*5*13 = 195 does not divide by 2, 4 or 8, and shards straddle
    # frame boundaries.
    gh, gw, F, s = 5, 13, 3, 9
    L = F * gh * gw
    x = _rng(5).standard_normal((L, 2, 128))
    whole = oracle.rotate(x, DIMS, THETA, gh, gw, s=s)
    n_loc = -(-L // P)
    for r in range(P):
        d = r * n_loc
        part = oracle.rotate(x[d:d + n_loc], DIMS, THETA, gh, gw, s=s, delta=d)
        assert np.array_equal(part, whole[d:d + n_loc])


def test_global_time_index_t_plus_s():
    # Section 3.3.2 item 1: chunk k rotated with s = k*tau equals frames [k*tau, k*tau+tau)
    # of a long sequence rotated with s = 0.
    gh, gw, tau, n_blocks = 4, 6, 3, 4
    hw = gh * gw
    x = _rng(6).standard_normal((n_blocks * tau * hw, 2, 128))
    whole = oracle.rotate(x, DIMS, THETA, gh, gw, s=0)
    for kblk in range(n_blocks):
        rows = slice(kblk * tau * hw, (kblk + 1) * tau * hw)
        part = oracle.rotate(x[rows], DIMS, THETA, gh, gw, s=kblk * tau)
        assert np.array_equal(part, whole[rows])


def test_relative_position_identity():
    # <rot(q,p1), rot(k,p2)> depends only on p1-p2 per axis: shift all frames by a constant
    # (the property that lets a rolling cache keep rotated keys).
    gh, gw = 4, 6
    q = _rng(7).standard_normal((2 * gh * gw, 2, 128))
    k = _rng(8).standard_normal((2 * gh * gw, 2, 128))

    def scores(sq, sk):
        qr = oracle.rotate(q, DIMS, THETA, gh, gw, s=sq)
        kr = oracle.rotate(k, DIMS, THETA, gh, gw, s=sk)
        return np.einsum("ihd,jhd->hij", qr, kr)

    base = scores(5, 2)
    for shift in (1, 7, 100):
        assert np.max(np.abs(scores(5 + shift, 2 + shift) - base)) < 1e-10
    assert np.max(np.abs(scores(6, 2) - base)) > 1e-3   # a relative shift does matter


def test_relative_position_identity_spatial():
    # same along h and w: compare token pairs with equal (dh, dw) offsets in one frame
    gh, gw = 6, 7
    rng = _rng(9)
    qv = rng.standard_normal(128)
    kv = rng.standard_normal(128)
    q = np.broadcast_to(qv, (gh * gw, 1, 128)).copy()
    k = np.broadcast_to(kv, (gh * gw, 1, 128)).copy()
    qr = oracle.rotate(q, DIMS, THETA, gh, gw, s=3).reshape(gh, gw, 128)
    kr = oracle.rotate(k, DIMS, THETA, gh, gw, s=3).reshape(gh, gw, 128)
    ref = qr[2, 3] @ kr[1, 1]          # offset (+1, +2)
    for (h, w) in [(1, 2), (5, 6), (3, 4)]:
        assert qr[h, w] @ kr[h - 1, w - 2] == pytest.approx(ref, abs=1e-11)


# ------------------------------------------------------------------ RMSNorm
def test_rmsnorm_constant_vector_closed_form():
    c, eps = 3.0, 1e-6
    x = np.full((2, 2, 128), c)
    g = _rng(10).standard_normal(256)
    y = oracle.rmsnorm(x, g, eps, 256)
    assert np.allclose(y, (g * c / np.sqrt(c * c + eps)).reshape(2, 128)[None], rtol=1e-15)


@pytest.mark.parametrize("group", [256, 128])
def test_rmsnorm_unit_rms_and_numpy_formula(group):
    x = _rng(11).standard_normal((7, 2, 128)) * 3.0
    y = oracle.rmsnorm(x, np.ones(256), 0.0, group)
    yg = y.reshape(7, 256 // group, group)
    assert np.allclose(np.sqrt((yg ** 2).mean(-1)), 1.0, rtol=1e-14)
    g = _rng(12).standard_normal(256)
    xg = x.reshape(7, 256 // group, group)
    ref = (xg / np.sqrt((xg ** 2).mean(-1, keepdims=True) + 1e-6)).reshape(7, 256) * g
    got = oracle.rmsnorm(x, g, 1e-6, group).reshape(7, 256)
    assert np.max(np.abs(got - ref)) < 1e-14


def test_rmsnorm_groups_differ_and_scale_invariance():
    x = _rng(13).standard_normal((3, 2, 128))
    x[:, 1] *= 5.0
    g = np.ones(256)
    full = oracle.rmsnorm(x, g, 0.0, 256)
    per_head = oracle.rmsnorm(x, g, 0.0, 128)
    assert not np.allclose(full, per_head)
    assert np.allclose(oracle.rmsnorm(4.0 * x, g, 0.0, 256), full, rtol=1e-14)


def test_rmsnorm_matches_torch_rms_norm():
    torch = pytest.importorskip("torch")
    x = _rng(14).standard_normal((5, 2, 128))
    g = _rng(15).standard_normal(256)
    ref = torch.nn.functional.rms_norm(torch.from_numpy(x.reshape(5, 256)), (256,),
                                       torch.from_numpy(g), eps=1e-6).numpy()
    got = oracle.rmsnorm(x, g, 1e-6, 256).reshape(5, 256)
    assert np.max(np.abs(got - ref)) < 1e-13
