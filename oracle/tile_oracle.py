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
shift) and the tile counts the paper states for 2K and 4K canvases; for the
gain / path-length policy (tests/test_oracle_gain.py): geometric drift with a
closed-form recompute period, g = 1 for any scalar model, g_c L = Equation 4's
accumulated error whenever the gain is constant, exact reuse for a model that
adds a constant, and a hand-computed three-step trace.
"""
import numpy as np


# --------------------------------------------------------------------------
# Tile geometry: PartitionTiles / SliceTile (Algorithm 1, stage 2; Section 4.2)
# --------------------------------------------------------------------------
def partition_tiles(H, W, tile_h, tile_w, overlap_h=0, overlap_w=0):
    """PartitionTiles: how many tiles of tile_h x tile_w tokens, neighbours sharing overlap_h /
    overlap_w tokens, cover an H x W canvas exactly -> (n_tile_rows, n_tile_cols, stride_h,
    stride_w).  The paper's partition is the case overlap = 0 (Section 4.2: non-overlapping
    tiles).  Tiles are placed at multiples of stride = tile - overlap; the last one must end
    at the canvas edge, otherwise the canvas has no such partition (ValueError).
    """
    out = []
    for extent, tile, overlap in ((int(H), int(tile_h), int(overlap_h)), (int(W), int(tile_w), int(overlap_w))):
        if tile < 1 or extent < tile or not (0 <= overlap < tile):
            raise ValueError("need 1 <= tile <= extent and 0 <= overlap < tile")
        stride = tile - overlap
        origins = list(range(0, extent - tile + 1, stride))
        if origins[-1] + tile != extent:
            raise ValueError("tiles of %d with overlap %d do not end at %d" % (tile, overlap, extent))
        out.append((len(origins), stride))
    return out[0][0], out[1][0], out[0][1], out[1][1]


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
    """Per tile: reuse only with a cache and a score strictly below the threshold
    (Equation 7); everything else recomputes, which includes a tie and a NaN score
    (NaN or Inf in the inputs: never "below").

    Returns (scores, recompute); the score of a tile without a cache is +inf.
    """
    scores, recompute = [], []
    for xk, xc, hc in zip(x_cur, x_cached, has_cache):
        s = gate_score(xk, xc) if hc else float("inf")
        scores.append(s)
        recompute.append(not (bool(hc) and s < float(threshold)))
    return np.array(scores, dtype=np.float64), np.array(recompute, dtype=bool)


# --------------------------------------------------------------------------
# Similarity of a tensor across adjacent denoising steps (Equation 3): the
# relative L1 distance with the earlier step's tensor in the denominator, and
# the cosine similarity.  The paper profiles predicted noise and cache
# residuals with this pair (Section 3, Section 5.1).
# --------------------------------------------------------------------------
def similarity(x_new, x_old):
    """(L1_rel, CosSim) of Equation 3 for one pair of tensors.

    L1_rel = ||x_new - x_old||_1 / ||x_old||_1 (+inf when the denominator is 0);
    CosSim = <x_new, x_old> / (||x_new||_2 ||x_old||_2), taken as 0 when either
    norm is 0 (the paper leaves the direction of a zero tensor open).
    """
    a = np.asarray(x_new, dtype=np.float64).ravel()
    b = np.asarray(x_old, dtype=np.float64).ravel()
    assert a.shape == b.shape
    l1 = gate_score(a, b)
    na, nb = float(np.sqrt((a * a).sum())), float(np.sqrt((b * b).sum()))
    cos = 0.0 if na == 0.0 or nb == 0.0 else float((a * b).sum() / (na * nb))
    return l1, cos


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


# --------------------------------------------------------------------------
# Inter-step tile-wise cache policy of Section 5.1: cache residual
# delta_c = O_c - I_c, gain g_c (Equation 5), latent path length L_{c->t}
# (Equation 6) and the recompute rule g_c L_{c->t} >= tau (Equation 7).
#
# The paper writes ||.|| without naming the norm; its profiling figures and
# Equation 3 use the relative L1 distance, and its thresholds (0.05, 0.09) are
# dimensionless, so every ||X_z - X_{z-1}|| below is the relative L1 change
# ||X_z - X_{z-1}||_1 / ||X_{z-1}||_1 (older tensor in the denominator).
# --------------------------------------------------------------------------
def rel_l1(new, old):
    """||new - old||_1 / ||old||_1 ; +inf when the denominator is 0."""
    return gate_score(new, old)


def accumulated_error(outputs):
    """Equation 4: E_{c->t} = sum_{z=c+1..t} ||O_z - O_{z-1}|| for outputs [O_c, ..., O_t]."""
    return float(sum(rel_l1(outputs[z], outputs[z - 1]) for z in range(1, len(outputs))))


def gain(o_new, o_old, i_new, i_old):
    """Equation 5: g_t = ||O_t - O_{t-1}|| / ||I_t - I_{t-1}||."""
    return rel_l1(o_new, o_old) / rel_l1(i_new, i_old)


class GainState:
    """Tile-wise Cache Store of Section 5.1, per tile:
    x_prev, o_prev   I_{t-1} and O_{t-1} (has_prev says whether a previous step exists)
    delta            cache residual delta_c = O_c - I_c of the last recomputed step c
    gain, has_gain   g_c and whether it is known yet (it needs two consecutive outputs)
    path_len         L_{c->t}, the latent path length since step c
    """

    def __init__(self, n_tiles):
        self.has_prev = [False] * n_tiles
        self.has_gain = [False] * n_tiles
        self.gain = [0.0] * n_tiles
        self.path_len = [0.0] * n_tiles
        self.x_prev = [None] * n_tiles
        self.o_prev = [None] * n_tiles
        self.delta = [None] * n_tiles


def gain_gate(x_cur, state, thresholds):
    """Error Calculator + Threshold Comparator: per tile
        d_t = ||I_t - I_{t-1}||          (0 on the first step: nothing to compare with)
        L  <- L + d_t                    (Equation 6)
        score = g_c * L                  (+inf while g_c is unknown)
        reuse iff g_c known and score < tau_i, else recompute   (Equation 7)
    x_cur[i] is tile i's flattened input.  Updates state.path_len.
    Returns (step_change d, scores, recompute)."""
    n = len(x_cur)
    d = np.zeros(n)
    scores = np.full(n, np.inf)
    recompute = np.ones(n, dtype=bool)
    for i in range(n):
        if state.has_prev[i]:
            d[i] = rel_l1(x_cur[i], state.x_prev[i])
        state.path_len[i] += d[i]
        if state.has_gain[i]:
            scores[i] = state.gain[i] * state.path_len[i]
            recompute[i] = not (scores[i] < float(thresholds[i]))
    return d, scores, recompute


def gain_refresh(o_new, latent, recompute, d, state):
    """After the Denoising Engine ran on the tiles to recompute (o_new[i] holds their
    new outputs, anything for the others).  Per tile:
      recomputed: g_c <- ||O_t - O_{t-1}|| / d_t if a previous output exists and d_t is
                  finite and > 0 (otherwise g_c keeps its state); L <- 0;
                  delta_c <- O_t - I_t                              (c <- t)
      reused:     O_t <- I_t + delta_c                              (Residual Approximation)
    latent[i] is the tensor I_t the residual is taken against (same shape as O).
    Returns the list of this step's outputs O_t; the caller stores them (and the
    inputs) as the next step's o_prev / x_prev."""
    outs = []
    for i in range(len(o_new)):
        lat = np.asarray(latent[i], dtype=np.float64)
        if recompute[i]:
            o = np.asarray(o_new[i], dtype=np.float64)
            if state.has_prev[i] and np.isfinite(d[i]) and d[i] > 0.0:
                state.gain[i] = rel_l1(o, state.o_prev[i]) / d[i]
                state.has_gain[i] = True
            state.path_len[i] = 0.0
            state.delta[i] = o - lat
        else:
            o = lat + state.delta[i]
        outs.append(o)
    return outs


def denoise_step_gain(tile_x, g, scale, state, thresholds, model=None, latent_of=None, store=None):
    """One stage-2 step under the cache policy of Section 5.1.

    tile_x[i] = (Q, K, V) packed tiles.  The gate reads concat(Q, K, V) as the tile
    input I_t; the residual is taken against latent_of(tile_x[i]) (default: Q, which
    has the shape of the output).  `model(i, Q, K, V)` is the Denoising Engine
    (default: full attention per head).  `store(a)` rounds an output to the storage
    type before it enters the state (default: identity).
    Returns (canvas, step_change, scores, recompute, outs)."""
    n = len(tile_x)
    flat = [np.concatenate([np.asarray(t, dtype=np.float64).ravel() for t in x]) for x in tile_x]
    latent = [np.asarray((latent_of(x) if latent_of else x[0]), dtype=np.float64) for x in tile_x]
    d, scores, recompute = gain_gate(flat, state, thresholds)
    o_new = [None] * n
    for i in range(n):
        if recompute[i]:
            Q, K, V = (np.asarray(t, dtype=np.float64) for t in tile_x[i])
            if model is not None:
                o_new[i] = model(i, Q, K, V)
            else:
                heads, dd = Q.shape[0], Q.shape[-1]
                o = np.stack([attention(Q[a].reshape(-1, dd), K[a].reshape(-1, dd), V[a].reshape(-1, dd), scale)
                              for a in range(heads)])
                o_new[i] = o.reshape(Q.shape)
            if store is not None:
                o_new[i] = store(o_new[i])
        else:
            o_new[i] = latent[i]   # placeholder, not read
    outs = gain_refresh(o_new, latent, recompute, d, state)
    if store is not None:
        outs = [store(o) for o in outs]
    for i in range(n):
        state.x_prev[i] = flat[i]
        state.o_prev[i] = outs[i]
        state.has_prev[i] = True
    canvas = blend(outs, g)
    return canvas, d, scores, recompute, outs


# --------------------------------------------------------------------------
# Intra-step region-aware cache control (Section 5.2; Appendix Algorithm 2):
# an online tracker of the standard deviation of each tile's predicted noise,
# and every Delta steps per-tile thresholds tau_i = tau_base * (1 + delta_i)
# from the "MaxMin" or the "TopSelect" policy.
#
# Readings (the paper leaves them open): the tracker keeps, per tile, the
# running mean over the steps seen so far of the population standard deviation
# of that step's tile output; Normalized() is min-max scaling across tiles
# (both policies only use the order of the normalised values, so any increasing
# normalisation gives the same thresholds); ties go to the lowest tile index.
# --------------------------------------------------------------------------
def tile_std(x):
    """Population standard deviation of all elements of one tile's output."""
    a = np.asarray(x, dtype=np.float64).ravel()
    return float(np.sqrt(np.mean((a - a.mean()) ** 2)))


class StdTracker:
    """StdTracker of Algorithm 2: running mean, per tile, of the per-step standard deviation."""

    def __init__(self, n_tiles):
        self.mean = np.zeros(n_tiles)
        self.count = 0

    def update(self, stds):
        stds = np.asarray(stds, dtype=np.float64)
        self.count += 1
        self.mean = self.mean + (stds - self.mean) / self.count

    def normalized(self):
        lo, hi = self.mean.min(), self.mean.max()
        return np.zeros_like(self.mean) if hi == lo else (self.mean - lo) / (hi - lo)


def region_thresholds(sigma, tau_base, alpha, mode):
    """tau_i = tau_base * (1 + delta_i) with delta = 0 except
    "MaxMin":    delta[argmax sigma] = alpha, delta[argmin sigma] = -alpha / 2
    "TopSelect": delta[largest] = alpha, delta[second largest] = alpha / 2
    (argmin is applied after argmax, so with a single tile or all-equal values it wins)."""
    sigma = np.asarray(sigma, dtype=np.float64)
    delta = np.zeros(len(sigma))
    if mode == "MaxMin":
        delta[int(np.argmax(sigma))] = alpha
        delta[int(np.argmin(sigma))] = -0.5 * alpha
    elif mode == "TopSelect":
        order = sorted(range(len(sigma)), key=lambda i: (-sigma[i], i))
        delta[order[0]] = alpha
        if len(order) > 1:
            delta[order[1]] = 0.5 * alpha
    else:
        raise ValueError("mode must be 'MaxMin' or 'TopSelect'")
    return float(tau_base) * (1.0 + delta)


# --------------------------------------------------------------------------
# Tile shifting (Algorithm 1 "ShiftThisStep" / "Shift"; Section 4.2: deterministic
# shifts along both spatial directions with a fixed stride, which lets the tiles
# stay non-overlapping).  The paper does not say what happens at the canvas edge;
# the reading here keeps every tile whole and the canvas covered by wrapping
# around: with shift (dy, dx) the token (i, j) of the tile with origin (r0, c0)
# sits at canvas position ((r0 + i + dy) mod H, (c0 + j + dx) mod W).  That is the
# unshifted partition applied to the canvas rolled by (-dy, -dx).
# --------------------------------------------------------------------------
def shift_schedule(step, tile_h, tile_w, loop_step=16, frequency=1):
    """Offset (dy, dx) of the partition at denoising step `step` = 0, 1, ... (Algorithm 1
    "ShiftThisStep" / "Shift"; Section 8 "Workloads": loop step 16, i.e. a shift stride of
    1/16 of the tile size, shifting every step; appendix: loop step = 1 / shift stride, and a
    frequency x shifts every x steps).

    The partition moves after every `frequency`-th step, along both directions at once, by
    1 / loop_step of the tile size; after loop_step moves it has travelled one whole tile,
    which for equal non-overlapping tiles on a wrapping canvas is the partition it started
    from, so the count of moves is taken modulo loop_step.  Where the tile size is not a
    multiple of loop_step the s-th position is floor(s * tile / loop_step): the stride stays
    1 / loop_step of a tile on average and the loop still closes.
    """
    step, loop_step, frequency = int(step), int(loop_step), int(frequency)
    if step < 0 or loop_step < 1 or frequency < 1:
        raise ValueError("step >= 0, loop_step >= 1, frequency >= 1")
    moves = (step // frequency) % loop_step
    return (moves * int(tile_h)) // loop_step, (moves * int(tile_w)) // loop_step


def slice_tile_shifted(grid, g, tile_row, tile_col, shift_h, shift_w):
    """SliceTile under a shifted partition: the unshifted window of the rolled canvas."""
    rolled = np.roll(np.asarray(grid), shift=(-int(shift_h), -int(shift_w)), axis=(2, 3))
    return slice_tile(rolled, g, tile_row, tile_col)


def blend_shifted(tile_outs, g, shift_h, shift_w):
    """Fuse under a shifted partition: the unshifted blend, rolled back by (dy, dx)."""
    return np.roll(blend(tile_outs, g), shift=(int(shift_h), int(shift_w)), axis=(2, 3))


# --------------------------------------------------------------------------
# Scheduler update after Fuse (Algorithm 1: L <- Model.Denoise(L, n); Section 4.2:
# the tile predictions are aggregated first so the whole canvas follows one
# trajectory).  The paper does not fix the sampler; every first-order sampler step
# (flow-matching Euler, DDIM) is affine in the latent and the fused prediction:
#     L <- c_latent * L + c_noise * n .
# --------------------------------------------------------------------------
def fuse_and_denoise(tile_outs, g, latent, c_latent, c_noise, shift_h=0, shift_w=0):
    n = blend_shifted(tile_outs, g, shift_h, shift_w)
    return float(c_latent) * np.asarray(latent, dtype=np.float64) + float(c_noise) * n
