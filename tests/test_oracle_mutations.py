"""Do the pins pin?  One plausible mistake at a time is planted in a COPY of the oracle (a dropped term,
a wrong sign or index, a swapped operand), the pin tests of the function's file run against the copy on
the CPU, and they must fail.  The unmutated copy must pass, so a failure is the pins' doing."""
import os
import shutil
import subprocess
import sys

import pytest

A, B, G, N, R, S, M = ("test_oracle_attention.py", "test_oracle_blend.py", "test_oracle_gate.py",
                       "test_oracle_gain.py", "test_oracle_region.py", "test_oracle_shift.py", "test_oracle_similarity.py")

MUTATIONS = [
    # name, pin file, text in oracle/tile_oracle.py, replacement
    ("softmax_shift_sign", A, "e = np.exp(s - m)", "e = np.exp(m - s)"),
    ("scores_against_values", A, "s = float(scale) * (q_rows @ K.T)", "s = float(scale) * (q_rows @ V.T)"),
    ("scale_dropped", A, "s = float(scale) * (q_rows @ K.T)", "s = (q_rows @ K.T)"),
    ("softmax_over_queries", A, "return e / e.sum(axis=1, keepdims=True)", "return e / e.sum(axis=0, keepdims=True)"),
    ("partition_stride_ignores_overlap", A, "        stride = tile - overlap\n", "        stride = tile\n"),
    ("partition_accepts_a_gap_at_the_edge", A, "        if origins[-1] + tile != extent:", "        if origins[-1] + tile > extent:"),
    ("partition_drops_the_last_tile", A, "origins = list(range(0, extent - tile + 1, stride))", "origins = list(range(0, extent - tile, stride)) or [0]"),
    ("ramp_i_not_i_plus_1", B, "np.minimum((i + 1.0) / (o + 1.0), (L - i) / (o + 1.0))",
     "np.minimum(i / (o + 1.0), (L - i) / (o + 1.0))"),
    ("ramp_falling_edge_off_by_one", B, "(L - i) / (o + 1.0)))", "(L - i - 1.0) / (o + 1.0)))"),
    ("ramp_divides_by_o", B, "np.minimum((i + 1.0) / (o + 1.0), (L - i) / (o + 1.0))",
     "np.minimum((i + 1.0) / max(o, 1e-300), (L - i) / (o + 1.0))"),
    ("blend_not_normalised", B, "return num / den\n", "return num\n"),
    ("tile_origin_strides_swapped", B, "return tile_row * g.stride_h, tile_col * g.stride_w",
     "return tile_row * g.stride_w, tile_col * g.stride_h"),
    ("gate_denominator_is_current", G, 'den = np.abs(b).sum()\n    return float("inf")', 'den = np.abs(a).sum()\n    return float("inf")'),
    ("gate_l2_norm", G, "num = np.abs(a - b).sum()\n    den = np.abs(b).sum()",
     "num = np.sqrt(((a - b) ** 2).sum())\n    den = np.sqrt((b ** 2).sum())"),
    ("gate_tie_reuses", G, "recompute.append(not (bool(hc) and s < float(threshold)))",
     "recompute.append(not (bool(hc) and s <= float(threshold)))"),
    ("gate_nan_score_reuses", G, "recompute.append(not (bool(hc) and s < float(threshold)))",
     "recompute.append(bool((not hc) or s >= float(threshold)))"),
    ("cosine_normalised_by_l1_norms", M, "na, nb = float(np.sqrt((a * a).sum())), float(np.sqrt((b * b).sum()))",
     "na, nb = float(np.abs(a).sum()), float(np.abs(b).sum())"),
    ("cosine_of_magnitudes", M, "float((a * b).sum() / (na * nb))", "float(np.abs(a * b).sum() / (na * nb))"),
    ("cosine_divides_by_one_norm_squared", M, "float((a * b).sum() / (na * nb))", "float((a * b).sum() / (nb * nb))"),
    ("similarity_l1_denominator_is_new", M, "    l1 = gate_score(a, b)\n", "    l1 = gate_score(b, a)\n"),
    ("gain_tie_reuses", N, "recompute[i] = not (scores[i] < float(thresholds[i]))",
     "recompute[i] = not (scores[i] <= float(thresholds[i]))"),
    ("path_length_not_accumulated", N, "state.path_len[i] += d[i]", "state.path_len[i] = d[i]"),
    ("gain_inverted", N, "return rel_l1(o_new, o_old) / rel_l1(i_new, i_old)", "return rel_l1(i_new, i_old) / rel_l1(o_new, o_old)"),
    ("gain_denominator_is_new_output", N, "state.gain[i] = rel_l1(o, state.o_prev[i]) / d[i]",
     "state.gain[i] = rel_l1(state.o_prev[i], o) / d[i]"),
    ("path_not_reset_on_recompute", N, "            state.path_len[i] = 0.0\n", "            pass\n"),
    ("residual_sign", N, "state.delta[i] = o - lat", "state.delta[i] = lat - o"),
    ("reuse_without_residual", N, "o = lat + state.delta[i]", "o = lat"),
    ("accumulated_error_skips_a_step", N, "for z in range(1, len(outputs))", "for z in range(2, len(outputs))"),
    ("sample_std", R, "return float(np.sqrt(np.mean((a - a.mean()) ** 2)))",
     "return float(np.sqrt(((a - a.mean()) ** 2).sum() / (len(a) - 1)))"),
    ("tracker_keeps_last_value", R, "self.mean = self.mean + (stds - self.mean) / self.count", "self.mean = stds"),
    ("maxmin_minimum_gets_full_alpha", R, "delta[int(np.argmin(sigma))] = -0.5 * alpha", "delta[int(np.argmin(sigma))] = -alpha"),
    ("topselect_second_gets_full_alpha", R, "delta[order[1]] = 0.5 * alpha", "delta[order[1]] = alpha"),
    ("threshold_additive", R, "return float(tau_base) * (1.0 + delta)", "return float(tau_base) + delta"),
    ("slice_shift_sign", S, "shift=(-int(shift_h), -int(shift_w)), axis=(2, 3))", "shift=(int(shift_h), int(shift_w)), axis=(2, 3))"),
    ("blend_shift_axes_swapped", S, "shift=(int(shift_h), int(shift_w)), axis=(2, 3))", "shift=(int(shift_w), int(shift_h)), axis=(2, 3))"),
    ("shift_ignores_frequency", S, "moves = (step // frequency) % loop_step", "moves = step % loop_step"),
    ("shift_loop_never_closes", S, "moves = (step // frequency) % loop_step", "moves = step // frequency"),
    ("shift_axes_swapped", S, "return (moves * int(tile_h)) // loop_step, (moves * int(tile_w)) // loop_step",
     "return (moves * int(tile_w)) // loop_step, (moves * int(tile_h)) // loop_step"),
    ("shift_stride_rounded_per_move", S, "return (moves * int(tile_h)) // loop_step, (moves * int(tile_w)) // loop_step",
     "return moves * (int(tile_h) // loop_step), moves * (int(tile_w) // loop_step)"),
    ("update_coefficients_swapped", S,
     "return float(c_latent) * np.asarray(latent, dtype=np.float64) + float(c_noise) * n",
     "return float(c_noise) * np.asarray(latent, dtype=np.float64) + float(c_latent) * n"),
]


@pytest.fixture(scope="module")
def sandbox(repo_root, tmp_path_factory):
    """A copy of the oracle, its pin tests and what they import; nothing of the HIP path."""
    box = tmp_path_factory.mktemp("oracle_copy")
    ignore = shutil.ignore_patterns("__pycache__")
    shutil.copytree(os.path.join(repo_root, "oracle"), box / "oracle", ignore=ignore)
    shutil.copytree(os.path.join(repo_root, "synthetic"), box / "synthetic", ignore=ignore)
    os.makedirs(box / "tests")
    shutil.copytree(os.path.join(repo_root, "tests", "golden"), box / "tests" / "golden")
    for f in (A, B, G, N, R, S, M, "conftest.py"):
        shutil.copy(os.path.join(repo_root, "tests", f), box / "tests" / f)
    return box


def _run_pins(box, test_file):
    return subprocess.run([sys.executable, "-m", "pytest", os.path.join("tests", test_file), "-x", "-q", "-m", "not gpu",
                           "-p", "no:cacheprovider"], cwd=box, capture_output=True, text=True, timeout=300)


def test_the_unmutated_copy_passes(sandbox):
    for f in (B, G, N, R, S, M):    # the attention pins run in the main suite; here they would only pay torch's import again
        r = _run_pins(sandbox, f)
        assert r.returncode == 0, r.stdout[-2000:]


@pytest.mark.parametrize("name,test_file,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_a_planted_mistake_fails_a_pin(sandbox, name, test_file, old, new):
    path = sandbox / "oracle" / "tile_oracle.py"
    original = path.read_text()
    assert original.count(old) >= 1, "the mutation no longer applies: update it with the oracle"
    try:
        path.write_text(original.replace(old, new, 1))
        r = _run_pins(sandbox, test_file)
    finally:
        path.write_text(original)
    assert r.returncode == 1 and "failed" in r.stdout, f"{name}: the pins did not notice\n{r.stdout[-1500:]}"
