"""Pins of the oracle's inter-step cache policy (paper Section 5.1: cache residual, gain of
Equation 5, path length of Equation 6, recompute rule of Equation 7) against closed forms, a
scalar re-derivation written separately, and Equation 4's accumulated error."""
import numpy as np
import pytest

import oracle
from synthetic import TileGeometry

G = TileGeometry("g", 1, 5, 7, 3, 4, 2, 3, 2, 2, 2, 4, "f32", 0)      # 2 x 2 tiles of 1 x 3 x 4 tokens
N_TILES = G.n_tiles


def _base(seed):
    """Positive, exactly representable tile inputs (small integers / 8)."""
    rng = np.random.default_rng(seed)
    return [tuple(rng.integers(1, 9, size=G.tile_shape).astype(np.float64) / 8 for _ in range(3))
            for _ in range(N_TILES)]


def _scaled(x, f):
    return [tuple(t * f for t in tile) for tile in x]


def _double_q(i, Q, K, V):          # a model that is a scalar multiple of the latent
    return 2.0 * Q


def test_gain_is_one_for_any_scalar_model_and_matches_equation_5():
    rng = np.random.default_rng(1)
    i0, i1 = rng.normal(size=500), rng.normal(size=500)
    for a in (0.3, -2.0, 7.5):
        assert oracle.gain(a * i1, a * i0, i1, i0) == pytest.approx(1.0, rel=1e-13)
    # Equation 5 written out on a hand-sized case: O: [1, 2] -> [2, 1], I: [4, 4] -> [5, 4]
    #   ||dO|| = (1 + 1) / 3, ||dI|| = 1 / 8  ->  g = 16 / 3
    assert oracle.gain([2.0, 1.0], [1.0, 2.0], [5.0, 4.0], [4.0, 4.0]) == pytest.approx(16.0 / 3.0, rel=1e-15)


def test_path_length_accumulates_and_equals_equation_4_when_the_gain_is_constant():
    """With a scalar model the output moves exactly as the input (g = 1), so g_c L_{c->t} must equal
    Equation 4's accumulated error of the true outputs, step for step."""
    b = 1.0 / 64
    x0 = _base(3)
    st = oracle.GainState(N_TILES)
    thr = [1e9] * N_TILES                                   # never recompute once the gain is known
    true_outs = []
    for t in range(8):
        xt = _scaled(x0, (1 + b) ** t)
        _, d, scores, rec, _ = oracle.denoise_step_gain(xt, G, 0.5, st, thr, model=_double_q)
        true_outs.append([2.0 * tile[0] for tile in xt])
        if t == 0:
            assert rec.all() and (d == 0).all()             # nothing to compare with yet
        elif t == 1:
            assert rec.all()                                # gain still unknown: it needs two outputs
            assert all(st.has_gain) and st.gain == pytest.approx([1.0] * N_TILES, rel=1e-12)
            assert st.path_len == [0.0] * N_TILES
        else:
            assert not rec.any()
            assert d == pytest.approx([b] * N_TILES, rel=1e-12)
            for i in range(N_TILES):
                e = oracle.accumulated_error([true_outs[z][i] for z in range(1, t + 1)])   # c = 1
                assert scores[i] == pytest.approx(e, rel=1e-12)
                assert st.path_len[i] == pytest.approx((t - 1) * b, rel=1e-12)


def _scalar_trace(r, tau, steps, model_gain=2.0):
    """The same policy on one positive scalar x_t = r^t (every tensor of the tile run is a positive
    multiple of one array, so relative L1 distances reduce to |a - b| / |b| of the multipliers)."""
    has_gain = False
    g = L = delta = 0.0
    x_prev = o_prev = None
    rec_log, out_log = [], []
    for t in range(steps):
        x = r ** t
        d = abs(x - x_prev) / abs(x_prev) if x_prev is not None else 0.0
        L += d
        rec = not (has_gain and g * L < tau)
        if rec:
            o = model_gain * x
            if o_prev is not None and d > 0:
                g = (abs(o - o_prev) / abs(o_prev)) / d
                has_gain = True
            L = 0.0
            delta = o - x
        else:
            o = x + delta
        x_prev, o_prev = x, o
        rec_log.append(rec)
        out_log.append(o)
    return rec_log, out_log


def test_geometric_drift_recompute_pattern_closed_form():
    """I_t = (1 + 1/64)^t I_0, model O = 2 Q, tau = 0.05.  By hand: steps 0 and 1 recompute (g = 1
    after step 1); L = 1/64, 2/64, 3/64 < 0.05 reuse; 4/64 >= 0.05 recomputes at step 5, where the
    previous output is the approximated one, O_4 = Q_4 + Q_1, so
    g = (2 r^5 - r^4 - r) / (r^4 + r) / (1/64) = 2.511..., and then 1 * g / 64 < 0.05 <= 2 g / 64."""
    b, r = 1.0 / 64, 1.0 + 1.0 / 64
    x0 = _base(5)
    st = oracle.GainState(N_TILES)
    recs, outs = [], []
    for t in range(10):
        xt = _scaled(x0, r ** t)
        _, d, s, rec, o = oracle.denoise_step_gain(xt, G, 0.5, st, [0.05] * N_TILES, model=_double_q)
        recs.append(rec.copy())
        outs.append(o)
        if t == 5:
            g5 = (2 * r ** 5 - r ** 4 - r) / (r ** 4 + r) / b
            assert 2.5 < g5 < 2.52
            assert st.gain == pytest.approx([g5] * N_TILES, rel=1e-12)
    hand = [True, True, False, False, False, True, False, True]
    for t, h in enumerate(hand):
        assert list(recs[t]) == [h] * N_TILES, t
    exp_rec, exp_out = _scalar_trace(r, 0.05, 10)
    for t in range(10):
        assert list(recs[t]) == [exp_rec[t]] * N_TILES
        for i in range(N_TILES):                               # outputs are exp_out[t] * Q_0
            np.testing.assert_allclose(outs[t][i], exp_out[t] * x0[i][0], rtol=1e-13)


def test_reuse_is_exact_for_a_model_that_adds_a_constant():
    """O = I + const has a constant residual, so O_t = I_t + delta_c reproduces the true output."""
    x0 = _base(7)
    st = oracle.GainState(N_TILES)
    add = lambda i, Q, K, V: Q + 0.25
    rng = np.random.default_rng(8)
    reused = 0
    for t in range(6):
        xt = [tuple(a + 1e-3 * t * rng.random(a.shape) for a in tile) for tile in x0]
        _, _, _, rec, outs = oracle.denoise_step_gain(xt, G, 0.5, st, [0.5] * N_TILES, model=add)
        for i in range(N_TILES):
            np.testing.assert_allclose(outs[i], xt[i][0] + 0.25, rtol=0, atol=1e-15)
            np.testing.assert_allclose(st.delta[i], 0.25, rtol=0, atol=1e-15)
        reused += int((~rec).sum())
    assert reused > 0


def test_tie_recomputes_and_per_tile_thresholds():
    """g = 1, one step of relative size 1/16: score = 1/16 exactly.  tau = 1/16 recomputes (>=),
    a larger tau reuses; thresholds are per tile."""
    x0 = _base(9)
    st = oracle.GainState(N_TILES)
    for t in range(2):
        oracle.denoise_step_gain(_scaled(x0, 1.0625 ** t), G, 0.5, st, [1.0] * N_TILES, model=_double_q)
    assert st.gain == pytest.approx([1.0] * N_TILES, rel=1e-13)
    st.gain = [1.0] * N_TILES                                   # exact, so the tie is exact
    x2 = _scaled(_scaled(x0, 1.0625), 1.0625)
    flat = [np.concatenate([a.ravel() for a in tile]) for tile in x2]
    d, s, rec = oracle.gain_gate(flat, st, [0.0625, 0.0626, 0.0625, 1.0])
    assert list(s) == [0.0625] * N_TILES
    assert list(rec) == [True, False, True, False]


def test_unchanged_input_adds_no_path_and_keeps_the_gain():
    x0 = _base(11)
    st = oracle.GainState(N_TILES)
    for t in range(2):
        oracle.denoise_step_gain(_scaled(x0, 1.25 ** t), G, 0.5, st, [0.05] * N_TILES, model=_double_q)
    g_before = list(st.gain)
    x1 = _scaled(x0, 1.25)
    _, d, s, rec, _ = oracle.denoise_step_gain(x1, G, 0.5, st, [0.05] * N_TILES, model=_double_q)
    assert (d == 0).all() and (s == 0).all() and not rec.any() and st.path_len == [0.0] * N_TILES
    # a forced recompute on an unchanged input cannot form Equation 5 (0 / 0): the gain stays
    _, d, s, rec, _ = oracle.denoise_step_gain(x1, G, 0.5, st, [0.0] * N_TILES, model=_double_q)
    assert rec.all() and st.gain == g_before


def test_default_model_is_tile_attention_and_store_rounds_the_state():
    rng = np.random.default_rng(13)
    x = [tuple(rng.normal(size=G.tile_shape) for _ in range(3)) for _ in range(N_TILES)]
    st = oracle.GainState(N_TILES)
    canvas, _, _, rec, outs = oracle.denoise_step_gain(x, G, 0.5, st, [0.05] * N_TILES)
    assert rec.all()
    ref = []
    for q, k, v in x:
        o = np.stack([oracle.attention(q[a].reshape(-1, 4), k[a].reshape(-1, 4), v[a].reshape(-1, 4), 0.5)
                      for a in range(G.heads)]).reshape(G.tile_shape)
        ref.append(o)
        np.testing.assert_array_equal(outs[len(ref) - 1], o)
    np.testing.assert_array_equal(canvas, oracle.blend(ref, G))
    for i in range(N_TILES):
        np.testing.assert_array_equal(st.delta[i], ref[i] - x[i][0])
    st2 = oracle.GainState(N_TILES)
    r3 = lambda a: np.round(a, 3)
    _, _, _, _, outs2 = oracle.denoise_step_gain(x, G, 0.5, st2, [0.05] * N_TILES, store=r3)
    for i in range(N_TILES):
        np.testing.assert_array_equal(outs2[i], np.round(ref[i], 3))
        np.testing.assert_array_equal(st2.o_prev[i], np.round(ref[i], 3))
