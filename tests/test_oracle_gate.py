"""Pins for the oracle's cache gate and tiled step.  CPU only."""
import numpy as np
import pytest

import oracle
from synthetic import TileGeometry


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def test_identical_input_scores_zero_and_reuses():
    x = _rand(1000, 1)
    s, r = oracle.cache_gate([x], [x.copy()], [True], 0.05)
    assert s[0] == 0.0 and not r[0]


@pytest.mark.parametrize("a,expect", [(0.0625, True), (0.03125, False), (-0.0625, True)])
def test_scaled_input_scores_abs_a_exactly(a, expect):
    xc = np.round(_rand(4096, 2) * 64) / 64          # exactly representable, so (1+a)x is exact
    s, r = oracle.cache_gate([(1 + a) * xc], [xc], [True], 0.05)
    assert s[0] == pytest.approx(abs(a), rel=1e-14)
    assert bool(r[0]) is expect


def test_denominator_is_the_cached_tensor():
    """Equation 3 divides by the older tensor: ||2-1||/||1|| = 1, not 1/2."""
    assert oracle.gate_score(np.full(8, 2.0), np.full(8, 1.0)) == 1.0
    assert oracle.gate_score(np.full(8, 1.0), np.full(8, 2.0)) == 0.5
    assert oracle.gate_score(np.array([3.0, -1.0]), np.array([1.0, 1.0])) == 2.0   # L1, not L2 (sqrt(2))


def test_tie_recomputes_and_strictly_below_reuses():
    xc = np.ones(16)
    thr = 0.0625
    s, r = oracle.cache_gate([xc * (1 + thr), xc * (1 + thr / 2)], [xc, xc], [True, True], thr)
    assert s[0] == thr and r[0] and not r[1]


def test_no_cache_or_zero_cache_recomputes():
    x = _rand(32, 3)
    s, r = oracle.cache_gate([x, x], [x, np.zeros(32)], [False, True], 0.05)
    assert r.all() and np.isinf(s).all()


@pytest.mark.parametrize("where,bad", [("cur", np.nan), ("cached", np.nan), ("cur", np.inf), ("cached", np.inf)])
def test_nan_or_inf_input_never_reuses(where, bad):
    """Equation 7 reuses only while the score is strictly below the threshold: a score that is NaN or +inf is not."""
    xc = _rand(64, 6)
    x = xc * 1.001                       # would reuse (score 0.001) without the bad element
    assert not oracle.cache_gate([x], [xc], [True], 0.05)[1][0]
    x, xc = x.copy(), xc.copy()
    (x if where == "cur" else xc)[17] = bad
    s, r = oracle.cache_gate([x], [xc], [True], 0.05)
    assert r[0] and not (s[0] < 0.05)


def test_brute_force_small():
    a, b = _rand(257, 4), _rand(257, 5)
    num = sum(abs(float(x) - float(y)) for x, y in zip(a, b))
    den = sum(abs(float(y)) for y in b)
    assert oracle.gate_score(a, b) == pytest.approx(num / den, rel=1e-13)


def test_paper_thresholds_fixture(repo_root):
    vals = dict(l.split() for l in open(f"{repo_root}/tests/golden/thresholds.txt") if not l.startswith("#"))
    assert float(vals["hunyuanvideo"]) == 0.05 and float(vals["cogvideox"]) == 0.09


# ------------------------------------------------------------------ step
G = TileGeometry("s", 1, 5, 7, 3, 4, 2, 3, 2, 2, 2, 4, "f32", 0)


def _tiles(seed):
    return [tuple(_rand(G.tile_shape, seed + 10 * i + j) for j in range(3)) for i in range(G.n_tiles)]


def test_step_state_machine():
    st = oracle.StepState(G.n_tiles)
    x0 = _tiles(1000)
    c0, s0, r0 = oracle.denoise_step_tiled(x0, G, 0.5, st, 0.05)
    assert r0.all() and all(st.has_cache)                      # empty cache: every tile recomputes
    # step 1: tiles 0, 2 barely move (reuse), tiles 1, 3 move a lot (recompute)
    x1 = [tuple(t + (0.001 if i % 2 == 0 else 0.5) * _rand(t.shape, 77 + i) for t in x) for i, x in enumerate(x0)]
    cached_before = [st.cache_out[i].copy() for i in range(4)]
    cachex_before = [st.cache_x[i].copy() for i in range(4)]
    c1, s1, r1 = oracle.denoise_step_tiled(x1, G, 0.5, st, 0.05)
    assert list(r1) == [False, True, False, True]
    for i in (0, 2):                                           # reuse leaves the cache untouched
        np.testing.assert_array_equal(st.cache_out[i], cached_before[i])
        np.testing.assert_array_equal(st.cache_x[i], cachex_before[i])
    for i in (1, 3):
        assert not np.array_equal(st.cache_out[i], cached_before[i])
        np.testing.assert_array_equal(st.cache_x[i], np.concatenate([t.ravel() for t in x1[i]]))
    # the canvas is the blend of cached outputs: reused tiles contribute last step's output
    np.testing.assert_array_equal(c1, oracle.blend(st.cache_out, G))
    # step 2 with the same inputs as step 1: drift of reused tiles is still measured from step 0
    _, s2, r2 = oracle.denoise_step_tiled(x1, G, 0.5, st, 0.05)
    assert s2[0] == s1[0] and s2[1] == 0.0 and not r2.any()


def test_gate_disabled_equals_ungated_step():
    st = oracle.StepState(G.n_tiles)
    x0, x1 = _tiles(2000), _tiles(3000)
    oracle.denoise_step_tiled(x0, G, 0.5, st, -1.0)
    c_gate_off, _, r = oracle.denoise_step_tiled(x1, G, 0.5, st, -1.0)
    assert r.all()
    fresh = oracle.StepState(G.n_tiles)
    c_fresh, _, _ = oracle.denoise_step_tiled(x1, G, 0.5, fresh, 0.05)
    np.testing.assert_array_equal(c_gate_off, c_fresh)
    # and equals attention per tile followed by blend, written out
    outs = []
    for q, k, v in x1:
        o = np.stack([oracle.attention(q[a].reshape(-1, 4), k[a].reshape(-1, 4), v[a].reshape(-1, 4), 0.5)
                      for a in range(G.heads)]).reshape(G.tile_shape)
        outs.append(o)
    np.testing.assert_array_equal(c_fresh, oracle.blend(outs, G))
