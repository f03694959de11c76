"""Pins for the prologue oracle (tile-order flattening, decoupled rotary embedding): what the mathematics fixes,
checked without reusing the oracle's own formulas.  CPU only."""
import math

import numpy as np
import pytest

from oracle import isa_oracle_prologue as P


# ---------------------------------------------------------------- tile order
@pytest.mark.parametrize("grid,tile", [((4, 8, 16), (2, 4, 8)), ((5, 7, 9), (2, 4, 4)), ((1, 30, 52), (2, 8, 8)),
                                       ((3, 3, 3), (1, 1, 1)), ((2, 5, 6), (4, 8, 8))])
def test_tile_order_is_a_permutation(grid, tile):
    perm = P.tile_order(grid, tile)
    n = grid[0] * grid[1] * grid[2]
    assert perm.shape == (n,)
    assert np.array_equal(np.sort(perm), np.arange(n))


def test_tile_order_degenerate_shapes_are_the_identity():
    grid = (3, 5, 7)
    n = 3 * 5 * 7
    for tile in ((3, 5, 7), (1, 1, 7), (1, 5, 7), (9, 9, 9), (1, 1, 100)):
        assert np.array_equal(P.tile_order(grid, tile), np.arange(n)), tile


def test_every_run_of_a_divisible_grid_is_one_box():
    grid, tile = (4, 8, 12), (2, 4, 6)
    perm = P.tile_order(grid, tile)
    vol = 2 * 4 * 6
    seen = set()
    for r in range(len(perm) // vol):
        idx = perm[r * vol:(r + 1) * vol]
        ft, rem = np.divmod(idx, 8 * 12)
        fh, fw = np.divmod(rem, 12)
        # the run covers exactly a tt x th x tw box that starts at a multiple of the tile shape
        assert ft.max() - ft.min() == 1 and fh.max() - fh.min() == 3 and fw.max() - fw.min() == 5
        assert ft.min() % 2 == 0 and fh.min() % 4 == 0 and fw.min() % 6 == 0
        assert len(set(idx.tolist())) == vol
        seen.add((int(ft.min()), int(fh.min()), int(fw.min())))
    assert len(seen) == (4 // 2) * (8 // 4) * (12 // 6)


def test_tile_order_by_hand():
    # 1 x 2 x 4 grid, 1 x 2 x 2 tiles: raster indices 0 1 2 3 / 4 5 6 7; left tile first (0 1 4 5), then right (2 3 6 7)
    assert P.tile_order((1, 2, 4), (1, 2, 2)).tolist() == [0, 1, 4, 5, 2, 3, 6, 7]
    # clipped edge: 1 x 1 x 5 grid, tiles of 2 along w -> still the raster order; 1 x 3 x 2 grid with 2 x 1 tiles in (h, w)
    assert P.tile_order((1, 1, 5), (1, 1, 2)).tolist() == [0, 1, 2, 3, 4]
    assert P.tile_order((1, 3, 2), (1, 2, 1)).tolist() == [0, 2, 1, 3, 4, 5]
    # tiles ordered with t slowest: 2 x 1 x 2 grid, 1 x 1 x 1 tiles = raster; 2 x 1 x 2 with (2, 1, 1) tiles pairs frames
    assert P.tile_order((2, 1, 2), (2, 1, 1)).tolist() == [0, 2, 1, 3]


def test_untile_inverts_the_reordering():
    rng = np.random.default_rng(3)
    grids, tile = [(2, 5, 6), (1, 3, 4)], (2, 2, 4)
    S = 60 + 12
    X = rng.standard_normal((S, 4))
    _, _, Xt = P.prologue_head(X, X, X, grids, tile, (0, 0, 0), 10000.0)      # values are only reordered
    assert not np.array_equal(Xt, X)
    assert np.array_equal(P.untile_head(Xt, grids, tile), X)


# ---------------------------------------------------------------- rotary embedding
def rot2(a):
    return np.array([[math.cos(a), -math.sin(a)], [math.sin(a), math.cos(a)]])


def test_rotation_by_hand():
    # one radian on the first pair (frame coordinate 1, first frequency of the axis is theta^0 = 1): (1, 0) -> (cos 1, sin 1)
    X = np.zeros((2, 4)); X[:, 0] = 1.0; X[:, 2] = 1.0
    coords = np.array([[0, 0, 0], [1, 0, 0]])
    ang = P.rope_angles(coords, 4, (4, 0, 0), 100.0)
    Y = P.rope_rotate(X, ang)
    np.testing.assert_allclose(Y[0], X[0], atol=0)                            # origin: untouched
    np.testing.assert_allclose(Y[1, :2], [0.5403023058681398, 0.8414709848078965], atol=1e-15)
    # second pair of a 4-channel axis: frequency theta^(-2/4) = 0.1 -> a tenth of a radian
    np.testing.assert_allclose(Y[1, 2:], [math.cos(0.1), math.sin(0.1)], atol=1e-15)


def test_rotation_matches_explicit_2x2_matrices_and_axis_split():
    rng = np.random.default_rng(4)
    D, dims, theta = 12, (4, 2, 4), 50.0          # pairs: 2 on t, 1 on h, 2 on w, 1 passes through
    coords = np.array([[3, 5, 7], [0, 2, 0]])
    X = rng.standard_normal((2, D))
    Y = P.rope_rotate(X, P.rope_angles(coords, D, dims, theta))
    for n in range(2):
        t, h, w = coords[n]
        expect_angles = [t * 1.0, t * theta ** (-0.5), h * 1.0, w * 1.0, w * theta ** (-0.5), 0.0]
        for i, a in enumerate(expect_angles):
            np.testing.assert_allclose(Y[n, 2 * i:2 * i + 2], rot2(a) @ X[n, 2 * i:2 * i + 2], atol=1e-14)


def test_rotation_preserves_pair_norms_and_scores_depend_on_offsets_only():
    rng = np.random.default_rng(5)
    D, dims, theta = 16, (4, 6, 6), 10000.0
    q, k = rng.standard_normal((1, D)), rng.standard_normal((1, D))
    def score(pq, pk):
        a = P.rope_rotate(q, P.rope_angles(np.array([pq]), D, dims, theta))
        b = P.rope_rotate(k, P.rope_angles(np.array([pk]), D, dims, theta))
        return float((a * b).sum()), a
    s0, a0 = score((2, 3, 4), (1, 1, 6))
    s1, _ = score((7, 10, 5), (6, 8, 7))       # both shifted by (5, 7, 1)
    s2, _ = score((2, 3, 4), (1, 1, 7))
    np.testing.assert_allclose(s0, s1, rtol=1e-12)
    assert abs(s0 - s2) > 1e-3
    np.testing.assert_allclose(a0[0, 0::2] ** 2 + a0[0, 1::2] ** 2, q[0, 0::2] ** 2 + q[0, 1::2] ** 2, rtol=1e-13)


def test_positions_restart_in_every_segment_and_values_are_not_rotated():
    rng = np.random.default_rng(6)
    grids, tile, dims = [(2, 3, 4), (1, 3, 4), (3, 2, 2)], (1, 3, 4), (4, 2, 2)     # tile = one frame: order unchanged
    S = 24 + 12 + 12
    Q, K, V = (rng.standard_normal((S, 8)) for _ in range(3))
    Qo, Ko, Vo = P.prologue_head(Q, K, V, grids, tile, dims, 10000.0)
    assert np.array_equal(Vo, V)
    for first in (0, 24, 36):                    # first token of every segment sits at the origin
        np.testing.assert_allclose(Qo[first], Q[first], atol=1e-15)
        np.testing.assert_allclose(Ko[first], K[first], atol=1e-15)
    assert np.abs(Qo[1] - Q[1]).max() > 1e-3
    # a segment is embedded the same way wherever it stands in the sequence
    Q2o, _, _ = P.prologue_head(Q[24:36], K[24:36], V[24:36], [grids[1]], tile, dims, 10000.0)
    np.testing.assert_allclose(Qo[24:36], Q2o, atol=1e-15)


def test_rotation_and_reordering_commute_as_stated():
    # rotating by the coordinates and then reordering = reordering and rotating by the reordered coordinates
    rng = np.random.default_rng(7)
    grid, tile, dims = (3, 4, 6), (2, 2, 4), (2, 4, 2)
    n = 72
    Q = rng.standard_normal((n, 8))
    Qo, _, _ = P.prologue_head(Q, Q, Q, [grid], tile, dims, 10000.0)
    perm = P.tile_order(grid, tile)
    coords = P.grid_coords(grid)
    for p in (0, 5, 17, 40, 71):
        src = perm[p]
        t, rem = divmod(int(src), 24)
        h, w = divmod(rem, 6)
        assert coords[src].tolist() == [t, h, w]
        expect = Q[src].copy()
        expect[0:2] = rot2(t * 1.0) @ Q[src, 0:2]
        expect[2:4] = rot2(h * 1.0) @ Q[src, 2:4]
        expect[4:6] = rot2(h * 10000.0 ** (-0.5)) @ Q[src, 4:6]
        expect[6:8] = rot2(w * 1.0) @ Q[src, 6:8]
        np.testing.assert_allclose(Qo[p], expect, atol=1e-13)


# ---------------------------------------------------------------- backward of the prologue
def test_backward_is_the_adjoint_and_the_inverse():
    rng = np.random.default_rng(8)
    grids, tile, dims = [(3, 4, 6), (1, 5, 3), (2, 2, 2)], (2, 3, 4), (4, 2, 6)
    S = 72 + 15 + 8
    X = [rng.standard_normal((S, 12)) for _ in range(3)]
    Y = [rng.standard_normal((S, 12)) for _ in range(3)]
    F = P.prologue_head(*X, grids, tile, dims, 10000.0)
    G = P.prologue_bwd_head(*Y, grids, tile, dims, 10000.0)
    for x, y, f, g in zip(X, Y, F, G):
        np.testing.assert_allclose((f * y).sum(), (x * g).sum(), rtol=1e-12)        # <A x, y> = <x, A^T y>
    back = P.prologue_bwd_head(*F, grids, tile, dims, 10000.0)                        # orthogonal map: A^T A = I
    for x, b in zip(X, back):
        np.testing.assert_allclose(b, x, atol=1e-13)


def test_backward_by_hand():
    # 1 x 1 x 2 grid, whole-grid tile (order unchanged), one pair turning with w at frequency 1: token 1 turns by one
    # radian forward, so its gradient turns back by one radian: (1, 0) -> (cos 1, -sin 1)
    g = np.array([[1.0, 0.0], [1.0, 0.0]])
    dq, dk, dv = P.prologue_bwd_head(g, g, g, [(1, 1, 2)], (1, 1, 2), (0, 0, 2), 10000.0)
    np.testing.assert_allclose(dq[0], [1.0, 0.0], atol=1e-15)
    np.testing.assert_allclose(dq[1], [0.5403023058681398, -0.8414709848078965], atol=1e-15)
    np.testing.assert_allclose(dk, dq, atol=0)
    np.testing.assert_allclose(dv, g, atol=0)
    # reordering alone: 1 x 2 x 4 grid with 1 x 2 x 2 tiles; output row p came from input row [0, 1, 4, 5, 2, 3, 6, 7][p]
    y = np.arange(8, dtype=np.float64).reshape(8, 1) * np.ones((1, 2))
    _, _, dv = P.prologue_bwd_head(y, y, y, [(1, 2, 4)], (1, 2, 2), (0, 0, 0), 10000.0)
    assert dv[:, 0].tolist() == [0, 1, 4, 5, 2, 3, 6, 7]      # input row 4 receives the gradient of output row 2, etc.
