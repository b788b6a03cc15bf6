"""Pins of the oracle's tile shifting (Algorithm 1 "Shift", Section 4.2) and of the scheduler update
fused after Fuse (Algorithm 1 "Model.Denoise")."""
import numpy as np
import pytest

import oracle
from synthetic import TileGeometry

# non-overlapping 2 x 3 partition of a 2 x 6 x 12 canvas (the paper's setting: stride = tile)
GP = TileGeometry("p", 2, 6, 12, 3, 4, 3, 4, 2, 3, 2, 4, "f32", 0)
# overlapping 2 x 2 partition
GO = TileGeometry("o", 1, 5, 7, 3, 4, 2, 3, 2, 2, 2, 4, "f32", 0)


def _canvas(g, seed):
    return np.random.default_rng(seed).normal(size=g.grid_shape)


def _brute_slice(grid, g, tr, tc, dy, dx):
    out = np.empty((grid.shape[0], g.T, g.tile_h, g.tile_w, grid.shape[-1]))
    for i in range(g.tile_h):
        for j in range(g.tile_w):
            out[:, :, i, j, :] = grid[:, :, (tr * g.stride_h + i + dy) % g.H, (tc * g.stride_w + j + dx) % g.W, :]
    return out


@pytest.mark.parametrize("dy,dx", [(0, 0), (1, 0), (0, 3), (2, 5), (5, 11), (3, 4)])
def test_shifted_slice_is_the_wrapped_window(dy, dx):
    c = _canvas(GP, 1)
    for tr in range(GP.n_tile_rows):
        for tc in range(GP.n_tile_cols):
            np.testing.assert_array_equal(oracle.slice_tile_shifted(c, GP, tr, tc, dy, dx), _brute_slice(c, GP, tr, tc, dy, dx))
    if (dy, dx) == (0, 0):
        np.testing.assert_array_equal(oracle.slice_tile_shifted(c, GP, 1, 2, 0, 0), oracle.slice_tile(c, GP, 1, 2))


@pytest.mark.parametrize("dy,dx", [(0, 0), (1, 2), (4, 9), (5, 11)])
def test_slice_then_fuse_is_the_identity_for_non_overlapping_tiles(dy, dx):
    """Every token lies in exactly one tile, so Fuse(SliceTile(L)) = L for any shift."""
    c = _canvas(GP, 2)
    tiles = [oracle.slice_tile_shifted(c, GP, tr, tc, dy, dx) for tr in range(GP.n_tile_rows) for tc in range(GP.n_tile_cols)]
    np.testing.assert_array_equal(oracle.blend_shifted(tiles, GP, dy, dx), c)


@pytest.mark.parametrize("dy,dx", [(1, 2), (4, 6)])
def test_shifted_blend_brute_force_with_overlap(dy, dx):
    rng = np.random.default_rng(3)
    tiles = [rng.normal(size=GO.tile_shape) for _ in range(GO.n_tiles)]
    got = oracle.blend_shifted(tiles, GO, dy, dx)
    wh = oracle.ramp_weight(GO.tile_h, GO.tile_h - GO.stride_h)
    ww = oracle.ramp_weight(GO.tile_w, GO.tile_w - GO.stride_w)
    ref = np.zeros(GO.grid_shape)
    for y in range(GO.H):
        for x in range(GO.W):
            yu, xu = (y - dy) % GO.H, (x - dx) % GO.W          # position in the unshifted partition
            num, den = 0.0, 0.0
            for tr in range(GO.n_tile_rows):
                for tc in range(GO.n_tile_cols):
                    i, j = yu - tr * GO.stride_h, xu - tc * GO.stride_w
                    if 0 <= i < GO.tile_h and 0 <= j < GO.tile_w:
                        w = wh[i] * ww[j]
                        num = num + w * tiles[tr * GO.n_tile_cols + tc][:, :, i, j, :]
                        den += w
            ref[:, :, y, x, :] = num / den
    np.testing.assert_allclose(got, ref, rtol=1e-14, atol=1e-15)
    # a canvas-consistent field sliced with the same shift is reproduced
    c = _canvas(GO, 4)
    tiles = [oracle.slice_tile_shifted(c, GO, tr, tc, dy, dx) for tr in range(2) for tc in range(2)]
    np.testing.assert_allclose(oracle.blend_shifted(tiles, GO, dy, dx), c, rtol=1e-14, atol=1e-15)


def test_fuse_and_denoise_is_the_affine_update():
    rng = np.random.default_rng(5)
    tiles = [rng.normal(size=GO.tile_shape) for _ in range(GO.n_tiles)]
    lat = rng.normal(size=GO.grid_shape)
    n = oracle.blend(tiles, GO)
    np.testing.assert_array_equal(oracle.fuse_and_denoise(tiles, GO, lat, 1.0, 0.0), lat)
    np.testing.assert_array_equal(oracle.fuse_and_denoise(tiles, GO, lat, 0.0, 1.0), n)
    # flow-matching Euler step from sigma 0.8 to 0.75: L + (0.75 - 0.8) * n
    np.testing.assert_allclose(oracle.fuse_and_denoise(tiles, GO, lat, 1.0, -0.05), lat - 0.05 * n, rtol=1e-15)
    np.testing.assert_allclose(oracle.fuse_and_denoise(tiles, GO, lat, 0.9, 0.3, 1, 2),
                               0.9 * lat + 0.3 * oracle.blend_shifted(tiles, GO, 1, 2), rtol=1e-15)
