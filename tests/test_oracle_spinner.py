"""CPU pins for the oracle's three-round product y = H D3 H D2 H D1 x
(Section 1 and Section 3; Condition 1: M1 = H D1 and M2 M1 = H D2 H D1 are
isometries).  Checks use the hand-expanded n = 2 closed form, brute force with
scipy's Hadamard matrix and numpy's dense algebra, and algebraic invariants.
"""
import itertools
import math
import os

import numpy as np
import pytest
import scipy.linalg

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _dense_reference(x, d1, d2, d3):
    """Brute force with explicitly formed n x n matrices from a different construction."""
    n = x.shape[-1]
    H = scipy.linalg.hadamard(n).astype(np.float64) / math.sqrt(n)
    G = H @ np.diag(d3.astype(np.float64)) @ H @ np.diag(d2.astype(np.float64)) @ H @ np.diag(d1.astype(np.float64))
    return (G @ x.astype(np.float64).T).T


def test_n2_hand_expanded_closed_form(oracle):
    rows = [l.split() for l in open(os.path.join(GOLDEN, "n2_closed_form.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 12
    x = np.array([3.0, 5.0], dtype=np.float32)
    for r in rows:
        v = [float(t) for t in r]
        d1, d2, d3 = (np.array(v[k:k + 2], dtype=np.float32) for k in (0, 2, 4))
        y = oracle.spinner(x, d1, d2, d3)
        assert np.allclose(y * 2.0 * math.sqrt(2.0), v[6:8], rtol=0, atol=1e-13), r


def test_n2_all_sign_patterns_formula(oracle):
    x = np.array([0.75, -1.5], dtype=np.float32)
    for s in itertools.product([1.0, -1.0], repeat=6):
        d1, d2, d3 = (np.array(s[k:k + 2], dtype=np.float32) for k in (0, 2, 4))
        a, b = s[0] * float(x[0]), s[1] * float(x[1])
        p = s[2] * (a + b) + s[3] * (a - b)
        q = s[2] * (a + b) - s[3] * (a - b)
        want = np.array([s[4] * p + s[5] * q, s[4] * p - s[5] * q]) / (2.0 * math.sqrt(2.0))
        assert np.allclose(oracle.spinner(x, d1, d2, d3), want, rtol=0, atol=1e-14)


@pytest.mark.parametrize("n", [2, 4, 8, 16, 32, 64])
def test_brute_force_dense_product_small_n(oracle, n):
    rng = np.random.default_rng(100 + n)
    x = rng.standard_normal((5, n)).astype(np.float32)
    # distinct, non-symmetric, non-+-1 diagonals so that a swapped or dropped D shows up
    d1 = rng.standard_normal(n).astype(np.float32)
    d2 = rng.uniform(0.5, 2.0, n).astype(np.float32)
    d3 = (1.0 - 2.0 * rng.integers(0, 2, n)).astype(np.float32) * np.float32(3.0)
    got = oracle.spinner(x, d1, d2, d3)
    want = _dense_reference(x, d1, d2, d3)
    assert np.allclose(got, want, rtol=0, atol=1e-12 * np.max(np.abs(want)))


@pytest.mark.parametrize("n", [128, 1024])
def test_rademacher_spinner_is_isometry_and_linear(oracle, n):
    rng = np.random.default_rng(n)
    d = (1.0 - 2.0 * rng.integers(0, 2, (3, n))).astype(np.float32)
    x = rng.standard_normal((4, n)).astype(np.float32)
    y = oracle.spinner(x, d[0], d[1], d[2])
    assert np.allclose(np.linalg.norm(y, axis=1), np.linalg.norm(x.astype(np.float64), axis=1), rtol=1e-12)
    # linearity on fp32-exact combinations
    z = (2.0 * x[0] - 0.5 * x[1]).astype(np.float32)
    exact = 2.0 * x[0].astype(np.float64) - 0.5 * x[1].astype(np.float64)
    if np.array_equal(z.astype(np.float64), exact):   # only when the combination is exact in fp32
        assert np.allclose(oracle.spinner(z, d[0], d[1], d[2]), 2.0 * y[0] - 0.5 * y[1], atol=1e-12)
    y2 = oracle.spinner((4.0 * x[2]).astype(np.float32), d[0], d[1], d[2])
    assert np.allclose(y2, 4.0 * y[2], rtol=0, atol=1e-12)


@pytest.mark.parametrize("n", [64, 512])
def test_identity_diagonals_reduce_to_one_transform(oracle, n):
    # D1 = D2 = D3 = I  =>  y = H^3 x = H x (H is an involution).
    rng = np.random.default_rng(5)
    x = rng.standard_normal((3, n)).astype(np.float32)
    one = np.ones(n, dtype=np.float32)
    want = (scipy.linalg.hadamard(n).astype(np.float64) @ x.astype(np.float64).T).T / math.sqrt(n)
    assert np.allclose(oracle.spinner(x, one, one, one), want, rtol=0, atol=1e-12)
    y = oracle.spinner(np.ones(n, dtype=np.float32), one, one, one)
    want1 = np.zeros(n)
    want1[0] = math.sqrt(n)
    assert np.allclose(y, want1, atol=1e-12)


@pytest.mark.parametrize("n", [32, 256])
def test_inverse_recovers_input(oracle, n):
    # (H D3 H D2 H D1)^-1 = D1 H D2 H D3 H for +-1 diagonals.
    rng = np.random.default_rng(9)
    d = (1.0 - 2.0 * rng.integers(0, 2, (3, n))).astype(np.float32)
    x = rng.standard_normal((2, n)).astype(np.float32)
    y = oracle.spinner(x, d[0], d[1], d[2])
    t = oracle.hadamard_apply(y)
    t = oracle.hadamard_apply(d[2] * t)
    t = d[0] * oracle.hadamard_apply(d[1] * t)
    assert np.allclose(t, x.astype(np.float64), rtol=0, atol=1e-12)


def test_single_round_pieces_compose(oracle):
    # The three rounds really are applied in the order D1, H, D2, H, D3, H.
    n = 64
    rng = np.random.default_rng(21)
    d = rng.standard_normal((3, n)).astype(np.float32)
    x = rng.standard_normal(n).astype(np.float32)
    t = x.astype(np.float64)
    for k in range(3):
        t = oracle.hadamard_apply(d[k].astype(np.float64) * t)
    assert np.allclose(oracle.spinner(x, d[0], d[1], d[2]), t, rtol=0, atol=1e-13)
    # and the order matters for these diagonals (guards against a symmetric test)
    assert not np.allclose(oracle.spinner(x, d[2], d[1], d[0]), t, atol=1e-6)


@pytest.mark.parametrize("n,a", [(256, 16), (1024, 32), (4096, 64), (4096, 128), (2048, 64)])
def test_kronecker_route_equals_dense_route(oracle, n, a):
    rng = np.random.default_rng(n + a)
    d = (1.0 - 2.0 * rng.integers(0, 2, (3, n))).astype(np.float32)
    d[2] = rng.standard_normal(n).astype(np.float32)      # Gaussian third diagonal (Lemma 1)
    x = rng.standard_normal((3, n)).astype(np.float32)
    dense = oracle.spinner(x, d[0], d[1], d[2], kron_a=0)
    kron = oracle.spinner(x, d[0], d[1], d[2], kron_a=a)
    assert np.allclose(kron, dense, rtol=0, atol=1e-11 * np.max(np.abs(dense)))


def test_default_route_selection(oracle):
    assert oracle.default_kron_a(1 << 14) == 0
    assert oracle.default_kron_a(1 << 15) == 256
    assert oracle.default_kron_a(1 << 20) == 1024


def test_thread_count_does_not_change_results(oracle):
    n = 256
    rng = np.random.default_rng(2)
    d = (1.0 - 2.0 * rng.integers(0, 2, (3, n))).astype(np.float32)
    x = rng.standard_normal((16, n)).astype(np.float32)
    y1 = oracle.spinner(x, d[0], d[1], d[2], nthreads=1)
    y4 = oracle.spinner(x, d[0], d[1], d[2], nthreads=4)
    assert np.array_equal(y1, y4)
