"""Pins for the oracle's 84x84 rasteriser (CPU only): the any-overlap rule written out with exact
rational cell edges, max-pooling of a full-resolution raster, fixed paddle columns, lit-pixel bound."""
from fractions import Fraction

import numpy as np

from oracle import oracle as orc


def S(**kw):
    base = dict(bx=79.0, by=104.0, vx=3.0, vy=0.0, pa=97.0, po=97.0, sa=0, so=0, ep_ret=0, ep_len=0)
    base.update(kw)
    return base


def _exact_frame(bx, by, pa, po):
    """Open-interval overlap of each rectangle with each cell, in exact rationals."""
    rects = [(Fraction(140), pa, 4, 16), (Fraction(16), po, 4, 16), (bx, by, 2, 2)]
    out = np.zeros((84, 84), np.uint8)
    for r in range(84):
        y_lo, y_hi = Fraction(210 * r, 84), Fraction(210 * (r + 1), 84)
        for c in range(84):
            x_lo, x_hi = Fraction(160 * c, 84), Fraction(160 * (c + 1), 84)
            for (x0, y0, w, h) in rects:
                if x0 < x_hi and x0 + w > x_lo and y0 < y_hi and y0 + h > y_lo:
                    out[r, c] = 255
    return out


def _maxpool_fullres(bx, by, pa, po):
    """Integer positions only: draw the rectangles on a 160x210 unit raster, then pixel (r,c) is
    lit iff any unit cell overlapping its footprint is lit (unit cell [u,u+1) overlaps
    [160c/84,160(c+1)/84) iff 84u < 160(c+1) and 84(u+1) > 160c)."""
    full = np.zeros((210, 160), bool)
    full[pa:pa + 16, 140:144] = True
    full[po:po + 16, 16:20] = True
    full[by:by + 2, bx:bx + 2] = True
    out = np.zeros((84, 84), np.uint8)
    cols = [[u for u in range(160) if 84 * u < 160 * (c + 1) and 84 * (u + 1) > 160 * c]
            for c in range(84)]
    rows = [[v for v in range(210) if 84 * v < 210 * (r + 1) and 84 * (v + 1) > 210 * r]
            for r in range(84)]
    for r in range(84):
        for c in range(84):
            if full[np.ix_(rows[r], cols[c])].any():
                out[r, c] = 255
    return out


def test_integer_positions_equal_maxpool_of_full_resolution_raster():
    rng = np.random.default_rng(3)
    cases = [(79, 104, 97, 97), (0, 0, 0, 0), (158, 208, 194, 194), (20, 100, 0, 194),
             (138, 50, 44, 60)]
    cases += [(int(rng.integers(0, 159)), int(rng.integers(0, 209)), int(rng.integers(0, 195)),
               int(rng.integers(0, 195))) for _ in range(12)]
    for bx, by, pa, po in cases:
        got = orc.pong_render_one(S(bx=float(bx), by=float(by), pa=float(pa), po=float(po)))
        assert np.array_equal(got, _maxpool_fullres(bx, by, pa, po)), (bx, by, pa, po)


def test_fractional_positions_equal_exact_rational_overlap():
    # positions on a 1/64 grid: every float32 product in the predicate is exact, so the float
    # rule and the rational rule must agree pixel for pixel
    rng = np.random.default_rng(4)
    for _ in range(10):
        bx = Fraction(int(rng.integers(0, 158 * 64)), 64)
        by = Fraction(int(rng.integers(0, 208 * 64)), 64)
        pa = Fraction(int(rng.integers(0, 194 * 64)), 64)
        po = Fraction(int(rng.integers(0, 194 * 64)), 64)
        got = orc.pong_render_one(S(bx=float(bx), by=float(by), pa=float(pa), po=float(po)))
        assert np.array_equal(got, _exact_frame(bx, by, pa, po))


def test_cell_edge_cases():
    # a ball whose left edge sits exactly on a cell edge does not light the cell to its left:
    # cell edge 160*21/84 = 40 -> ball [40,42) lights columns 21 (and 22 if 42 > 160*22/84=41.9)
    f = orc.pong_render_one(S(bx=40.0, by=0.0, pa=194.0, po=194.0))
    ball_cols = np.flatnonzero(f[0])
    assert ball_cols.tolist() == [21, 22]
    # row cell height 2.5: ball rows [0,2) only touch row 0; [5,7) touches rows 2 (5..7.5) only
    assert np.flatnonzero(f[:, 21]).tolist() == [0]
    f = orc.pong_render_one(S(bx=40.0, by=5.0, pa=194.0, po=194.0))
    assert np.flatnonzero(f[:, 21]).tolist() == [2]
    f = orc.pong_render_one(S(bx=40.0, by=4.0, pa=194.0, po=194.0))
    assert np.flatnonzero(f[:, 21]).tolist() == [1, 2]


def test_paddle_columns_and_lit_bound_on_a_rollout():
    p = orc.Pong(32, 6, max_score=2); p.reset()
    stack = np.zeros((32, 4, 84, 84), np.uint8)
    p.fill_stack(stack)
    assert all(np.array_equal(stack[:, 0], stack[:, k]) for k in range(1, 4))
    for t in range(40):
        obs, _, _ = p.step(stack=stack)
        slot = t % 4
        fr = stack[:, slot]
        assert set(np.unique(fr)) <= {0, 255}
        assert (fr == 255).reshape(32, -1).sum(1).max() <= 54
        for i in range(32):
            f = fr[i]
            # paddle pixels: columns 73..75 (agent) and 8..10 (opponent); ball within 3 columns
            pa, po = obs[i, 4], obs[i, 5]
            lit_cols = np.flatnonzero(f.any(axis=0))
            ball_c = int(np.floor(obs[i, 0] * 84 / 160))
            allowed = {8, 9, 10, 73, 74, 75, ball_c, ball_c + 1, ball_c + 2}
            assert set(lit_cols.tolist()) <= allowed
            assert {8, 9, 10, 73, 74, 75} <= set(lit_cols.tolist())
            # with the ball away from the paddle columns each paddle covers 7 or 8 rows whose
            # first row is floor(y * 84 / 210)
            if 12 <= ball_c <= 69:
                ra = np.flatnonzero(f[:, 74]); ro = np.flatnonzero(f[:, 9])
                assert 7 <= len(ra) <= 8 and 7 <= len(ro) <= 8
                assert ra.min() == int(np.floor(float(pa) * 84 / 210))
                assert ro.min() == int(np.floor(float(po) * 84 / 210))
                assert np.array_equal(f[:, 73], f[:, 74]) and np.array_equal(f[:, 74], f[:, 75])
            # the frame equals a fresh render of the state in the observation
            want = orc.pong_render_one(S(bx=float(obs[i, 0]), by=float(obs[i, 1]),
                                         pa=float(pa), po=float(po)))
            assert np.array_equal(f, want)
    # ring: after 40 steps slot k holds the frame of the last step with index = k (mod 4)
    assert not np.array_equal(stack[:, 0], stack[:, 3])
