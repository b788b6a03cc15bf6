"""Pins for the oracle's Fuse/blend: golden ramp, closed forms, brute force.  CPU only."""
import numpy as np
import pytest

import oracle
from synthetic import TileGeometry, CONFIGS


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def brute_force_blend(tile_outs, g):
    """Per output token: enumerate every tile, test coverage, accumulate by hand."""
    heads, d = tile_outs[0].shape[0], tile_outs[0].shape[-1]
    oh, ow = g.tile_h - g.stride_h, g.tile_w - g.stride_w
    out = np.zeros((heads, g.T, g.H, g.W, d))
    for y in range(g.H):
        for x in range(g.W):
            num, den = np.zeros((heads, g.T, d)), 0.0
            for tr in range(g.n_tile_rows):
                for tc in range(g.n_tile_cols):
                    i, j = y - tr * g.stride_h, x - tc * g.stride_w
                    if 0 <= i < g.tile_h and 0 <= j < g.tile_w:
                        w = (min(1.0, (i + 1) / (oh + 1), (g.tile_h - i) / (oh + 1)) *
                             min(1.0, (j + 1) / (ow + 1), (g.tile_w - j) / (ow + 1)))
                        num += w * tile_outs[tr * g.n_tile_cols + tc][:, :, i, j, :]
                        den += w
            out[:, :, y, x, :] = num / den
    return out


def test_ramp_golden(repo_root):
    w = oracle.ramp_weight(10, 4)
    rows = [l.split() for l in open(f"{repo_root}/tests/golden/ramp_o4_L10.txt") if not l.startswith("#")]
    for i, val in rows:
        assert abs(w[int(i)] - float(val)) < 1e-15
    np.testing.assert_array_equal(oracle.ramp_weight(7, 0), np.ones(7))      # o = 0: placement
    assert oracle.ramp_weight(48, 27).min() == pytest.approx(1 / 28)          # >= 1/(o+1) > 0


@pytest.mark.parametrize("geom", [
    CONFIGS["tiny_f32"],
    TileGeometry("triple", 2, 9, 7, 5, 4, 2, 3, 3, 2, 2, 4, "f32", 0),      # rows covered 3 times
])
def test_matches_brute_force(geom):
    tiles = [_rand(geom.tile_shape, 100 + i) for i in range(geom.n_tiles)]
    np.testing.assert_allclose(oracle.blend(tiles, geom), brute_force_blend(tiles, geom),
                               rtol=1e-13, atol=1e-14)


def test_constant_tiles_give_the_constant():
    g = CONFIGS["tiny_f32"]
    tiles = [np.full(g.tile_shape, 2.5) for _ in range(g.n_tiles)]
    np.testing.assert_allclose(oracle.blend(tiles, g), 2.5, rtol=1e-15)


def test_zero_overlap_is_pure_placement():
    g = TileGeometry("p", 2, 8, 6, 4, 3, 4, 3, 2, 2, 2, 4, "f32", 0)
    tiles = [_rand(g.tile_shape, 200 + i) for i in range(4)]
    out = oracle.blend(tiles, g)
    for tr in range(2):
        for tc in range(2):
            np.testing.assert_array_equal(out[:, :, 4 * tr:4 * tr + 4, 3 * tc:3 * tc + 3, :], tiles[2 * tr + tc])


def test_grid_consistent_field_is_reproduced():
    """If every tile carries the same canvas-wide field, blending returns that field."""
    g = TileGeometry("triple", 2, 9, 7, 5, 4, 2, 3, 3, 2, 2, 4, "f32", 0)
    field = _rand(g.grid_shape, 300)
    tiles = [np.ascontiguousarray(oracle.slice_tile(field, g, r, c)) for r in range(3) for c in range(2)]
    np.testing.assert_allclose(oracle.blend(tiles, g), field, rtol=1e-13, atol=1e-14)


def test_two_tile_overlap_closed_form_and_single_coverage_passthrough():
    """One row of two tiles, L = 6, stride 4 (o = 2).  In the overlap, position k = 0..o-1
    gets weights (o-k)/(o+1) from the left tile and (k+1)/(o+1) from the right one (they
    sum to 1); elsewhere a single tile covers the token and passes through exactly."""
    g = TileGeometry("two", 1, 3, 10, 3, 6, 3, 4, 1, 2, 1, 2, "f32", 0)
    a, b = _rand(g.tile_shape, 400), _rand(g.tile_shape, 401)
    out = oracle.blend([a, b], g)
    np.testing.assert_allclose(out[..., 0:4, :], a[..., 0:4, :], rtol=1e-15)
    np.testing.assert_allclose(out[..., 6:10, :], b[..., 2:6, :], rtol=1e-15)
    for k in range(2):
        expect = (2 - k) / 3 * a[..., 4 + k, :] + (k + 1) / 3 * b[..., k, :]
        np.testing.assert_allclose(out[..., 4 + k, :], expect, rtol=1e-13)


def test_tiles_must_cover_canvas():
    g = TileGeometry("gap", 1, 3, 12, 3, 4, 3, 6, 1, 2, 1, 2, "f32", 0)    # stride > tile: a gap
    with pytest.raises(ValueError):
        oracle.blend([np.ones(g.tile_shape)] * 2, g)
