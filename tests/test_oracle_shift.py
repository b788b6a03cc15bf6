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


# ------------------------------------------------------------------ the shift schedule (Algorithm 1 "ShiftThisStep")
def _golden_shift_rows():
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "shift_loop16.txt")
    return [tuple(int(v) for v in line.split()) for line in open(path) if line.strip() and not line.startswith("#")]


def test_shift_schedule_matches_the_hand_worked_loop_of_16():
    """Section 8 "Workloads": loop step 16 on the 160 x 90 latent tile, shifting every step."""
    for moves, along_160, along_90 in _golden_shift_rows():
        assert oracle.shift_schedule(moves, 90, 160, loop_step=16, frequency=1) == (along_90, along_160)


def test_shift_schedule_frequency_holds_the_partition_between_moves():
    """A frequency of x shifts every x steps: x consecutive steps share a position, and the loop takes 16 x steps."""
    rows = _golden_shift_rows()
    for freq in (1, 2, 5):
        for step in range(0, 16 * freq + 3):
            moves = (step // freq) % 16
            assert oracle.shift_schedule(step, 90, 160, 16, freq) == (rows[moves][2], rows[moves][1])
        assert oracle.shift_schedule(16 * freq, 90, 160, 16, freq) == (0, 0)
        assert oracle.shift_schedule(freq, 90, 160, 16, freq) != oracle.shift_schedule(freq - 1, 90, 160, 16, freq)


def test_shift_schedule_properties():
    for th, tw, loop in ((45, 80, 16), (48, 80, 16), (3, 4, 2), (10, 10, 7), (5, 9, 1)):
        prev = (0, 0)
        assert oracle.shift_schedule(0, th, tw, loop) == (0, 0)
        for s in range(1, loop):
            dy, dx = oracle.shift_schedule(s, th, tw, loop)
            assert 0 <= dy < th and 0 <= dx < tw
            # every move is 1/loop of the tile, to within the one token that rounding costs
            assert dy - prev[0] in (th // loop, -(-th // loop)) and dx - prev[1] in (tw // loop, -(-tw // loop))
            prev = (dy, dx)
        assert oracle.shift_schedule(loop, th, tw, loop) == (0, 0)            # the loop closes
    with pytest.raises(ValueError):
        oracle.shift_schedule(-1, 4, 4)
    with pytest.raises(ValueError):
        oracle.shift_schedule(0, 4, 4, loop_step=0)
    with pytest.raises(ValueError):
        oracle.shift_schedule(0, 4, 4, frequency=0)


def test_a_whole_tile_of_shift_is_the_same_partition():
    """Why the count of moves is taken modulo the loop step: moved by one whole tile along both directions, a
    non-overlapping wrapping partition consists of the same windows (tile (r, c) sits where (r + 1, c + 1) sat)."""
    c = _canvas(GP, 7)
    for tr in range(GP.n_tile_rows):
        for tc in range(GP.n_tile_cols):
            moved = oracle.slice_tile_shifted(c, GP, tr, tc, GP.tile_h, GP.tile_w)
            np.testing.assert_array_equal(moved, oracle.slice_tile(c, GP, (tr + 1) % GP.n_tile_rows, (tc + 1) % GP.n_tile_cols))
