"""Pins for the oracle's frequency tables and global index decode (CPU only).

Each check is independent of the oracle's own formula: closed forms, library routines,
exhaustive enumeration with numpy.unravel_index, and the one worked example the paper
prints (start_frame = 0, 3, 6 for tau = 3 — Section 3.3.2 item 1).
"""
import math
import os

import numpy as np
import pytest

import oracle

THETA = 10000.0


@pytest.mark.parametrize("dim_a", [44, 42, 8, 2])
def test_table_closed_forms(dim_a):
    n_pos = 40
    tab = oracle.axis_table(dim_a, THETA, n_pos)
    assert tab.shape == (n_pos, dim_a // 2, 2)
    # position 0: zero angle, exactly (1, 0)
    assert np.all(tab[0, :, 0] == 1.0) and np.all(tab[0, :, 1] == 0.0)
    # pair 0 has omega = 1, so the angle is the position itself
    for p in range(n_pos):
        assert tab[p, 0, 0] == pytest.approx(math.cos(p), abs=1e-15)
        assert tab[p, 0, 1] == pytest.approx(math.sin(p), abs=1e-15)
    # unit modulus
    assert np.allclose(tab[..., 0] ** 2 + tab[..., 1] ** 2, 1.0, atol=1e-14)
    # last pair: omega = theta^(-(d-2)/d), checked through a different route (exp/log)
    j = dim_a // 2 - 1
    w_last = math.exp(-math.log(THETA) * (dim_a - 2) / dim_a)
    assert tab[7, j, 0] == pytest.approx(math.cos(7 * w_last), abs=1e-13)
    assert tab[7, j, 1] == pytest.approx(math.sin(7 * w_last), abs=1e-13)


def test_table_independent_recomputation():
    # whole table through exp(-ln(theta)*2j/d) and numpy's cos/sin
    for dim_a in (44, 42):
        j = np.arange(dim_a // 2, dtype=np.float64)
        omega = np.exp(-np.log(THETA) * 2.0 * j / dim_a)
        p = np.arange(1024, dtype=np.float64)[:, None]
        ref = np.stack([np.cos(p * omega), np.sin(p * omega)], axis=-1)
        tab = oracle.axis_table(dim_a, THETA, 1024)
        assert np.max(np.abs(tab - ref)) < 2e-12  # omega differs by an ulp -> 1e3 * 1e-16


def test_table_frequencies_decrease_geometrically():
    # ratio of successive angles at p = 1 is theta^(-2/d): recover it from atan2
    tab = oracle.axis_table(44, THETA, 2)
    ang = np.arctan2(tab[1, :, 1], tab[1, :, 0])  # all angles < 1 rad, no wrap
    ratio = ang[1:] / ang[:-1]
    assert np.allclose(ratio, THETA ** (-2.0 / 44), rtol=1e-12)


def test_theta_infinite_limit_is_identity_for_higher_pairs():
    tab = oracle.axis_table(8, 1e300, 5)
    # omega_j -> 0 for j >= 1
    assert np.allclose(tab[:, 1:, 0], 1.0) and np.allclose(tab[:, 1:, 1], 0.0, atol=1e-60)


@pytest.mark.parametrize("grid", [(4, 6), (3, 5), (1, 7), (30, 52)])
def test_decode_matches_unravel_index(grid):
    gh, gw = grid
    F = 3
    s = 6
    n = F * gh * gw
    step = 1 if n < 2000 else 7
    for i in range(0, n, step):
        f, h, w = np.unravel_index(i, (F, gh, gw))
        assert oracle.decode(i, 0, s, gh, gw) == (s + f, h, w)


@pytest.mark.parametrize("P", [1, 2, 4, 8])
def test_decode_shard_equals_slice(P):
    # Section 3.3.3: rank r's token i_local sits at global index r*L/P + i_local.
    gh, gw, F, s = 5, 13, 3, 9     # L = 195; 195/8 is not an integer -> use ceil-sized shards
    L = F * gh * gw
    whole = [oracle.decode(i, 0, s, gh, gw) for i in range(L)]
    n_loc = -(-L // P)
    for r in range(P):
        delta = r * n_loc
        for i in range(min(n_loc, L - delta)):
            assert oracle.decode(i, delta, s, gh, gw) == whole[delta + i]


def test_c5_shard_straddles_frame_boundary():
    # rank 2 of 8 at 480P: rows 1170..1754 cross from frame 0 to frame 1 at row 1560
    assert oracle.decode(0, 1170, 18, 30, 52) == (18, 22, 26)
    assert oracle.decode(1559 - 1170, 1170, 18, 30, 52) == (18, 29, 51)
    assert oracle.decode(1560 - 1170, 1170, 18, 30, 52) == (19, 0, 0)
    assert oracle.decode(584, 1170, 18, 30, 52) == (19, 3, 38)


def test_printed_start_frames():
    path = os.path.join(os.path.dirname(__file__), "golden", "start_frames.txt")
    rows = [tuple(int(x) for x in ln.split()) for ln in open(path)
            if ln.strip() and not ln.startswith("#")]
    assert rows == [(0, 3, 0), (1, 3, 3), (2, 3, 6)]
    for k, tau, s in rows:
        assert s == k * tau
        # first token of block k, local time index t=0..tau-1 -> t_global = t + s
        for t in range(tau):
            tg, h, w = oracle.decode(t * 24, 0, s, 4, 6)
            assert (tg, h, w) == (t + s, 0, 0)
