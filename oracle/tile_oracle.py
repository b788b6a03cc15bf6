"""Plain fp64 definitions of tile attention, tile fusing (blend) and the cache gate.

TEST INFRASTRUCTURE: slow on purpose, numpy fp64 throughout, no blocking, no
fusion, no reordering beyond what each definition states.  Inputs are the stored
values (bf16 / fp32) widened exactly to fp64 by the caller.

Notation follows the paper: a latent canvas of T x H x W tokens is partitioned
along H and W only, every tile keeps all T frames (Section 4.2); I_t is a tile's
input, O_t its output, tau the cache threshold (Section 5.1).

Geometry arguments are passed as an object `g` with integer attributes
    T, H, W, tile_h, tile_w, stride_h, stride_w, n_tile_rows, n_tile_cols
Grid tensors are numpy arrays shaped [heads, T, H, W, d]; a packed tile is
[heads, T, tile_h, tile_w, d]; tokens of a tile are ordered (t, i, j), j fastest.

Pins (tests/test_oracle_*.py): agreement with torch's fp64
scaled_dot_product_attention, a separately written triple-loop brute force,
closed forms (two-key softmax, scale 0 -> mean(V), two-tile ramp weights sum to
1, |a| scaling of the relative L1), invariances (row sums, permutation, key
shift) and the tile counts the paper states for 2K and 4K canvases.
"""
import numpy as np


# --------------------------------------------------------------------------
# Tile geometry: PartitionTiles / SliceTile (Algorithm 1, stage 2; Section 4.2)
# --------------------------------------------------------------------------
def tile_origin(g, tile_row, tile_col):
    """Top-left grid token (row, col) of tile (tile_row, tile_col)."""
    if not (0 <= tile_row < g.n_tile_rows and 0 <= tile_col < g.n_tile_cols):
        raise IndexError("tile index out of range")
    return tile_row * g.stride_h, tile_col * g.stride_w


def slice_tile(grid, g, tile_row, tile_col):
    """SliceTile: the tile's sub-volume, all T frames, a tile_h x tile_w window."""
    r0, c0 = tile_origin(g, tile_row, tile_col)
    assert grid.shape[1:4] == (g.T, g.H, g.W)
    assert r0 + g.tile_h <= g.H and c0 + g.tile_w <= g.W
    return grid[:, :, r0:r0 + g.tile_h, c0:c0 + g.tile_w, :]


# --------------------------------------------------------------------------
# 3D full self-attention over one tile's tokens (Section 2.1 "full attention";
# Section 3: no Q/K/V exchange across tiles)
# --------------------------------------------------------------------------
def softmax_rows(s):
    """Row softmax of a score matrix s[n, N]; returns p with rows summing to 1."""
    s = np.asarray(s, dtype=np.float64)
    m = s.max(axis=1, keepdims=True)
    e = np.exp(s - m)
    return e / e.sum(axis=1, keepdims=True)


def attention_rows(q_rows, K, V, scale):
    """o[n] = sum_m softmax_m(scale * <q[n], K[m]>) V[m] for the given query rows.

    q_rows [n, d], K [N, d], V [N, d]  ->  [n, d], all fp64.
    """
    q_rows = np.asarray(q_rows, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    s = float(scale) * (q_rows @ K.T)
    return softmax_rows(s) @ V


def attention(Q, K, V, scale):
    """Full bidirectional attention of one head: Q, K, V [N, d] -> O [N, d]."""
    return attention_rows(Q, K, V, scale)


def tile_attention(q_grid, k_grid, v_grid, g, tile_row, tile_col, scale,
                   heads=None, rows=None):
    """Attention of tile (tile_row, tile_col) read out of grid tensors.

    Returns a dict {head: O[len(rows), d]}; rows index the tile's tokens in
    (t, i, j) order (all tokens if rows is None).
    """
    qt = slice_tile(q_grid, g, tile_row, tile_col)
    kt = slice_tile(k_grid, g, tile_row, tile_col)
    vt = slice_tile(v_grid, g, tile_row, tile_col)
    n_heads, d = qt.shape[0], qt.shape[-1]
    N = g.T * g.tile_h * g.tile_w
    out = {}
    for a in (range(n_heads) if heads is None else heads):
        Q = np.ascontiguousarray(qt[a], dtype=np.float64).reshape(N, d)
        K = np.ascontiguousarray(kt[a], dtype=np.float64).reshape(N, d)
        V = np.ascontiguousarray(vt[a], dtype=np.float64).reshape(N, d)
        out[a] = attention_rows(Q if rows is None else Q[np.asarray(rows)], K, V, scale)
    return out


# --------------------------------------------------------------------------
# Fuse: merge tile outputs into the full canvas (Algorithm 1 "Fuse";
# Section 4.2: aggregation before the scheduler update; Tile Fuser, Section 5)
# --------------------------------------------------------------------------
def ramp_weight(L, o):
    """Per-axis blend weight w(i) = min(1, (i+1)/(o+1), (L-i)/(o+1)), i in [0, L).

    L = tile length along the axis, o = overlap = L - stride.  o = 0 gives w = 1
    everywhere, i.e. the paper's non-overlapping placement.
    """
    i = np.arange(L, dtype=np.float64)
    return np.minimum(1.0, np.minimum((i + 1.0) / (o + 1.0), (L - i) / (o + 1.0)))


def blend(tile_outs, g):
    """out[token] = sum_tiles w * O_tile / sum_tiles w over the tiles covering it.

    tile_outs: list, row-major over (tile_row, tile_col), of [heads, T, tile_h,
    tile_w, d] arrays.  w = w_h(i) * w_w(j); the T axis is not tiled and carries
    weight 1.  Returns the [heads, T, H, W, d] canvas.
    """
    assert len(tile_outs) == g.n_tile_rows * g.n_tile_cols
    heads, d = tile_outs[0].shape[0], tile_outs[0].shape[-1]
    wh = ramp_weight(g.tile_h, g.tile_h - g.stride_h)
    ww = ramp_weight(g.tile_w, g.tile_w - g.stride_w)
    w = (wh[:, None] * ww[None, :])[None, None, :, :, None]
    num = np.zeros((heads, g.T, g.H, g.W, d), dtype=np.float64)
    den = np.zeros((1, 1, g.H, g.W, 1), dtype=np.float64)
    for tr in range(g.n_tile_rows):
        for tc in range(g.n_tile_cols):
            r0, c0 = tile_origin(g, tr, tc)
            o = np.asarray(tile_outs[tr * g.n_tile_cols + tc], dtype=np.float64)
            assert o.shape == (heads, g.T, g.tile_h, g.tile_w, d)
            num[:, :, r0:r0 + g.tile_h, c0:c0 + g.tile_w, :] += w * o
            den[:, :, r0:r0 + g.tile_h, c0:c0 + g.tile_w, :] += w
    if not (den > 0).all():
        raise ValueError("tiles do not cover the canvas")
    return num / den


# --------------------------------------------------------------------------
# Cache gate: relative L1 change of a tile's input against the cached input
# (Equation 3: the older tensor is the denominator; Equation 7: strictly below
# the threshold reuses, at or above recomputes)
# --------------------------------------------------------------------------
def gate_score(x_cur, x_cached):
    """||x_cur - x_cached||_1 / ||x_cached||_1 ; +inf when the denominator is 0."""
    a = np.asarray(x_cur, dtype=np.float64).ravel()
    b = np.asarray(x_cached, dtype=np.float64).ravel()
    assert a.shape == b.shape
    num = np.abs(a - b).sum()
    den = np.abs(b).sum()
    return float("inf") if den == 0.0 else float(num / den)


def cache_gate(x_cur, x_cached, has_cache, threshold):
    """Per tile: recompute = (no cache) or (score >= threshold).

    Returns (scores, recompute); the score of a tile without a cache is +inf.
    """
    scores, recompute = [], []
    for xk, xc, hc in zip(x_cur, x_cached, has_cache):
        s = gate_score(xk, xc) if hc else float("inf")
        scores.append(s)
        recompute.append(bool((not hc) or s >= float(threshold)))
    return np.array(scores, dtype=np.float64), np.array(recompute, dtype=bool)


# --------------------------------------------------------------------------
# One tiled denoising step with the tile-wise cache store
# (Algorithm 1 stage-2 loop body; Section 5.1 pipeline: gate -> recompute or
# reuse -> Tile Fuser)
# --------------------------------------------------------------------------
class StepState:
    """Tile-wise cache store: per tile the cached input, cached output, valid flag."""

    def __init__(self, n_tiles):
        self.has_cache = [False] * n_tiles
        self.cache_x = [None] * n_tiles
        self.cache_out = [None] * n_tiles


def denoise_step_tiled(tile_x, g, scale, state, threshold, attend=None):
    """tile_x[i] = (Q, K, V) packed tiles, each [heads, T, tile_h, tile_w, d].

    Gate every tile on concat(Q, K, V) against its cached input; recompute the
    flagged tiles' attention and refresh their cache entries (the cache of a
    reused tile is left untouched, so drift keeps being measured from the last
    recomputed step c); blend all cached outputs.  threshold < 0 disables the
    gate (every tile recomputes).  `attend(i, Q, K, V)` may replace the full
    attention (used to evaluate sampled rows only).
    Returns (canvas, scores, recompute).
    """
    n = len(tile_x)
    flat = [np.concatenate([np.asarray(t, dtype=np.float64).ravel() for t in x]) for x in tile_x]
    if threshold < 0:
        scores = np.full(n, np.inf)
        recompute = np.ones(n, dtype=bool)
    else:
        cached = [c if c is not None else np.zeros_like(f) for c, f in zip(state.cache_x, flat)]
        scores, recompute = cache_gate(flat, cached, state.has_cache, threshold)
    for i in range(n):
        if recompute[i]:
            Q, K, V = (np.asarray(t, dtype=np.float64) for t in tile_x[i])
            if attend is not None:
                state.cache_out[i] = attend(i, Q, K, V)
            else:
                heads, d = Q.shape[0], Q.shape[-1]
                o = np.stack([attention(Q[a].reshape(-1, d), K[a].reshape(-1, d),
                                        V[a].reshape(-1, d), scale) for a in range(heads)])
                state.cache_out[i] = o.reshape(Q.shape)
            state.cache_x[i] = flat[i]
            state.has_cache[i] = True
    canvas = blend(state.cache_out, g)
    return canvas, scores, recompute
