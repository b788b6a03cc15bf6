"""Pins for the oracle's similarity pair of Equation 3 (relative L1 distance and cosine similarity).  CPU only."""
import math

import numpy as np
import pytest

import oracle


def _rand(n, seed):
    return np.random.default_rng(seed).standard_normal(n)


def test_identical_opposite_and_orthogonal():
    x = _rand(1000, 1)
    l1, cos = oracle.similarity(x, x.copy())
    assert l1 == 0.0 and cos == pytest.approx(1.0, abs=1e-15)
    l1, cos = oracle.similarity(-x, x)
    assert l1 == pytest.approx(2.0, rel=1e-14) and cos == pytest.approx(-1.0, abs=1e-15)
    e0, e1 = np.array([3.0, 0.0, 0.0]), np.array([0.0, -2.0, 0.0])
    assert oracle.similarity(e0, e1) == (2.5, 0.0)            # (3 + 2) / 2 ; perpendicular


def test_hand_values():
    # 45 degrees: (1, 1) against (1, 0)
    l1, cos = oracle.similarity(np.array([1.0, 1.0]), np.array([1.0, 0.0]))
    assert l1 == 1.0 and cos == pytest.approx(1.0 / math.sqrt(2.0), rel=1e-15)
    # 3-4-5: <(3, 4), (4, 3)> = 24, norms 5 and 5; L1 = (1 + 1) / 7
    l1, cos = oracle.similarity(np.array([3.0, 4.0]), np.array([4.0, 3.0]))
    assert l1 == pytest.approx(2.0 / 7.0, rel=1e-15) and cos == pytest.approx(24.0 / 25.0, rel=1e-15)


def test_cosine_ignores_scale_and_l1_does_not():
    a, b = _rand(513, 2), _rand(513, 3)
    l1, cos = oracle.similarity(a, b)
    l1s, coss = oracle.similarity(4.0 * a, 0.25 * b)
    assert coss == pytest.approx(cos, rel=1e-13) and l1s != pytest.approx(l1, rel=1e-3)
    assert oracle.similarity(2.0 * a, 2.0 * b)[0] == pytest.approx(l1, rel=1e-13)     # a common factor cancels in L1_rel
    assert oracle.similarity(b, a)[1] == pytest.approx(cos, rel=1e-13)                 # the cosine is symmetric


def test_l1_part_is_the_gate_score_with_the_older_tensor_below():
    a, b = _rand(300, 4), _rand(300, 5)
    assert oracle.similarity(a, b)[0] == oracle.gate_score(a, b)
    assert oracle.similarity(np.full(8, 2.0), np.full(8, 1.0))[0] == 1.0                # ||2 - 1|| / ||1||, not / ||2||


def test_brute_force():
    a, b = _rand(257, 6), _rand(257, 7)
    dot = sum(float(x) * float(y) for x, y in zip(a, b))
    na = math.sqrt(sum(float(x) ** 2 for x in a))
    nb = math.sqrt(sum(float(y) ** 2 for y in b))
    num = sum(abs(float(x) - float(y)) for x, y in zip(a, b))
    den = sum(abs(float(y)) for y in b)
    l1, cos = oracle.similarity(a, b)
    assert l1 == pytest.approx(num / den, rel=1e-13) and cos == pytest.approx(dot / (na * nb), rel=1e-13)
    assert abs(cos) <= 1.0


def test_library_cross_check():
    """The same cosine from torch's own routine (fp64)."""
    import torch
    a, b = _rand(4097, 8), _rand(4097, 9) + 0.5
    want = float(torch.nn.functional.cosine_similarity(torch.from_numpy(a), torch.from_numpy(b), dim=0))
    assert oracle.similarity(a, b)[1] == pytest.approx(want, rel=1e-12)


def test_zero_tensors():
    z, x = np.zeros(16), _rand(16, 10)
    assert oracle.similarity(x, z) == (float("inf"), 0.0)
    assert oracle.similarity(z, x) == (1.0, 0.0)
    assert oracle.similarity(z, z) == (float("inf"), 0.0)
