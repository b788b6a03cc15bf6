"""Pins for the oracle's attention: library special case, brute force, closed forms,
invariants.  CPU only."""
import math

import numpy as np
import pytest
import torch

import oracle
from synthetic import TileGeometry


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def brute_force_attention(Q, K, V, scale):
    """Separately written triple loop with math.exp (no numpy reductions)."""
    N, d = len(K), len(K[0])
    out = []
    for q in Q:
        s = [scale * sum(q[c] * K[m][c] for c in range(d)) for m in range(N)]
        mx = max(s)
        e = [math.exp(x - mx) for x in s]
        tot = sum(e)
        out.append([sum(e[m] * V[m][c] for m in range(N)) / tot for c in range(d)])
    return np.array(out)


@pytest.mark.parametrize("N,d", [(1, 4), (2, 3), (5, 8), (8, 16)])
def test_matches_brute_force(N, d):
    Q, K, V = _rand((N, d), 1), _rand((N, d), 2), _rand((N, d), 3)
    ref = brute_force_attention(Q.tolist(), K.tolist(), V.tolist(), 0.37)
    np.testing.assert_allclose(oracle.attention(Q, K, V, 0.37), ref, rtol=1e-13, atol=1e-14)


@pytest.mark.parametrize("N,d", [(37, 64), (300, 64), (257, 128)])
def test_matches_torch_sdpa_fp64(N, d):
    """A non-square, asymmetric case so a transposed operand or a dropped scale fails."""
    Q, K, V = _rand((N // 2 + 1, d), 4), _rand((N, d), 5), _rand((N, d), 6)
    scale = 1.0 / math.sqrt(d)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(Q)[None], torch.from_numpy(K)[None], torch.from_numpy(V)[None],
        scale=scale)[0].numpy()
    np.testing.assert_allclose(oracle.attention_rows(Q, K, V, scale), ref, rtol=1e-11, atol=1e-13)


def test_softmax_rows_sum_to_one_and_are_positive():
    p = oracle.softmax_rows(_rand((17, 301), 7) * 30.0)
    np.testing.assert_allclose(p.sum(axis=1), 1.0, rtol=0, atol=1e-14)
    assert (p >= 0).all()


def test_two_key_closed_form():
    """q.k1 - q.k2 = ln 3 / scale  ->  weights 3/4 and 1/4."""
    scale = 0.5
    q = np.array([[1.0, 0.0]])
    K = np.array([[math.log(3.0) / scale, 0.0], [0.0, 5.0]])
    V = np.array([[8.0, -4.0], [0.0, 4.0]])
    np.testing.assert_allclose(oracle.attention_rows(q, K, V, scale), [[6.0, -2.0]], rtol=1e-14)


def test_single_key_returns_v():
    Q, K, V = _rand((6, 8), 8), _rand((1, 8), 9), _rand((1, 8), 10)
    np.testing.assert_allclose(oracle.attention_rows(Q, K, V, 0.3), np.repeat(V, 6, 0), rtol=1e-15)


def test_scale_zero_and_identical_keys_give_mean_v():
    Q, K, V = _rand((5, 8), 11), _rand((9, 8), 12), _rand((9, 8), 13)
    mean = np.repeat(V.mean(0, keepdims=True), 5, 0)
    np.testing.assert_allclose(oracle.attention_rows(Q, K, V, 0.0), mean, rtol=1e-13)
    Ksame = np.repeat(K[:1], 9, 0)
    np.testing.assert_allclose(oracle.attention_rows(Q, Ksame, V, 0.8), mean, rtol=1e-13)


def test_constant_v_gives_constant_output():
    Q, K = _rand((7, 16), 14), _rand((33, 16), 15)
    V = np.tile(np.arange(16.0), (33, 1))
    np.testing.assert_allclose(oracle.attention_rows(Q, K, V, 0.25), np.tile(np.arange(16.0), (7, 1)),
                               rtol=1e-13, atol=1e-13)


def test_key_shift_invariance():
    """Adding one vector to every key shifts each query's logits by a constant."""
    Q, K, V = _rand((7, 16), 16), _rand((33, 16), 17), _rand((33, 16), 18)
    a = oracle.attention_rows(Q, K, V, 0.25)
    b = oracle.attention_rows(Q, K + _rand((1, 16), 19), V, 0.25)
    np.testing.assert_allclose(a, b, rtol=1e-11, atol=1e-12)


def test_dominant_key_selects_its_value():
    Q, K, V = np.ones((1, 4)), _rand((10, 4), 20), _rand((10, 4), 21)
    K[3] = 1000.0
    np.testing.assert_allclose(oracle.attention_rows(Q, K, V, 1.0), V[3:4], rtol=1e-12)


def test_token_permutation_equivariance():
    N, d = 41, 8
    Q, K, V = _rand((N, d), 22), _rand((N, d), 23), _rand((N, d), 24)
    perm = np.random.default_rng(25).permutation(N)
    base = oracle.attention(Q, K, V, 0.4)
    np.testing.assert_allclose(oracle.attention(Q[perm], K[perm], V[perm], 0.4), base[perm],
                               rtol=1e-12, atol=1e-13)
    # permuting keys and values jointly leaves every query's output unchanged
    np.testing.assert_allclose(oracle.attention(Q, K[perm], V[perm], 0.4), base, rtol=1e-12, atol=1e-13)


def test_output_rms_at_iid_normal_inputs():
    """i.i.d. N(0,1) inputs, scale 1/sqrt(d): logits ~ N(0,1), so sum p^2 ~ e/N and
    output components have rms ~ sqrt(e/N) (order-of-magnitude scale check)."""
    N, d = 4000, 64
    Q, K, V = _rand((64, d), 26), _rand((N, d), 27), _rand((N, d), 28)
    rms = math.sqrt((oracle.attention_rows(Q, K, V, 1 / math.sqrt(d)) ** 2).mean())
    assert 0.7 * math.sqrt(math.e / N) < rms < 1.4 * math.sqrt(math.e / N)


# ---------------------------------------------------------------- tiling
G = TileGeometry("t", 2, 7, 9, 4, 5, 3, 4, 2, 2, 2, 8, "f32", 0)


def test_slice_tile_is_spatial_only_and_full_temporal():
    grid = _rand(G.grid_shape, 30)
    t = oracle.slice_tile(grid, G, 1, 1)
    assert t.shape == G.tile_shape
    np.testing.assert_array_equal(t, grid[:, :, 3:7, 4:9, :])
    assert oracle.tile_origin(G, 1, 0) == (3, 0)
    with pytest.raises(IndexError):
        oracle.tile_origin(G, 2, 0)


def test_tile_view_equals_packed_copy_and_single_tile_equals_untiled():
    q, k, v = (_rand(G.grid_shape, s) for s in (31, 32, 33))
    o = oracle.tile_attention(q, k, v, G, 0, 1, 0.3)
    one = G.single_tile()
    packed = [np.ascontiguousarray(oracle.slice_tile(x, G, 0, 1)) for x in (q, k, v)]
    o2 = oracle.tile_attention(*packed, one, 0, 0, 0.3)
    for a in range(G.heads):
        np.testing.assert_array_equal(o[a], o2[a])
        N = G.tile_tokens
        np.testing.assert_allclose(
            o[a], oracle.attention(packed[0][a].reshape(N, -1), packed[1][a].reshape(N, -1),
                                   packed[2][a].reshape(N, -1), 0.3), rtol=1e-13)
    rows = [0, 5, N - 1]
    o3 = oracle.tile_attention(q, k, v, G, 0, 1, 0.3, heads=[1], rows=rows)
    np.testing.assert_array_equal(o3[1], o[1][rows])


def test_paper_tile_counts(repo_root):
    """Non-overlapping 720p tiles: 2K -> 4 tiles, 4K -> 9 tiles."""
    for line in open(f"{repo_root}/tests/golden/tile_counts.txt"):
        if line.startswith("#") or not line.strip():
            continue
        H, W, th, tw, n = map(int, line.split())
        assert math.ceil(H / th) * math.ceil(W / tw) == n
        g = TileGeometry("p", 1, H, W, th, tw, th, tw, H // th, W // tw, 1, 4, "f32", 0)
        origins = [oracle.tile_origin(g, r, c) for r in range(g.n_tile_rows) for c in range(g.n_tile_cols)]
        assert len(set(origins)) == n
        assert max(o[0] for o in origins) + th == H and max(o[1] for o in origins) + tw == W


def test_partition_tiles_gives_the_paper_counts_and_the_benchmark_tilings(repo_root):
    """PartitionTiles against what is fixed elsewhere: the paper's 4 and 9 tiles (Section 8 "Workloads"), the five
    benchmark geometries (their tile counts and strides are inputs there, not derived), and coverage by brute force."""
    from synthetic import CONFIGS
    for line in open(f"{repo_root}/tests/golden/tile_counts.txt"):
        if line.startswith("#") or not line.strip():
            continue
        H, W, th, tw, n = map(int, line.split())
        nr, nc, sh, sw = oracle.partition_tiles(H, W, th, tw)
        assert nr * nc == n and (sh, sw) == (th, tw)
    for g in CONFIGS.values():
        got = oracle.partition_tiles(g.H, g.W, g.tile_h, g.tile_w, g.tile_h - g.stride_h if g.n_tile_rows > 1 else 0,
                                     g.tile_w - g.stride_w if g.n_tile_cols > 1 else 0)
        assert got[:2] == (g.n_tile_rows, g.n_tile_cols)
        if g.n_tile_rows > 1:
            assert got[2] == g.stride_h
        if g.n_tile_cols > 1:
            assert got[3] == g.stride_w
    # brute force: every row and column is covered, no tile sticks out, neighbours share exactly the overlap
    for H, th, oh in ((16, 10, 4), (90, 48, 27), (135, 45, 15), (12, 4, 0), (7, 7, 0), (9, 5, 3)):
        nr, _, sh, _ = oracle.partition_tiles(H, 8, th, 8, oh, 0)
        cover = np.zeros(H, dtype=int)
        for r in range(nr):
            assert r * sh + th <= H
            cover[r * sh:r * sh + th] += 1
        assert cover.min() >= 1 and (nr - 1) * sh + th == H
        if nr > 1:
            assert th - sh == oh
    for bad in ((10, 8, 4, 8, 0, 0), (16, 8, 10, 8, 3, 0), (16, 8, 20, 8, 0, 0), (16, 8, 4, 8, 4, 0), (16, 8, 0, 8, 0, 0)):
        with pytest.raises(ValueError):
            oracle.partition_tiles(*bad)
