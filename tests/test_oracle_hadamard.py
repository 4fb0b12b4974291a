"""CPU pins for the oracle's Hadamard matrix (Section 3: H is the L2-normalised
Hadamard matrix; supplement, proof of the balancedness remark: entries of
magnitude 1/sqrt(n), orthogonal rows, H D is an isometry).

Every check here compares the oracle with something that is not the oracle:
a hand-typed fixture, scipy's own Sylvester construction, the Kronecker
recursion built with numpy, or an algebraic invariant.
"""
import math
import os

import numpy as np
import pytest
import scipy.linalg

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _read_pm_matrix(path):
    rows = [l.strip() for l in open(path) if l.strip() and not l.startswith("#")]
    return np.array([[1 if c == "+" else -1 for c in r] for r in rows], dtype=np.int64)


def test_h8_matches_hand_typed_fixture(oracle):
    want = _read_pm_matrix(os.path.join(GOLDEN, "hadamard8_sylvester.txt"))
    assert want.shape == (8, 8)
    assert np.array_equal(oracle.hadamard_dense(8).astype(np.int64), want)


@pytest.mark.parametrize("n", [1, 2, 4, 16, 128, 1024])
def test_popcount_formula_equals_library_sylvester(oracle, n):
    assert np.array_equal(oracle.hadamard_dense(n).astype(np.int64), scipy.linalg.hadamard(n))


@pytest.mark.parametrize("n", [2, 8, 64, 512])
def test_sylvester_recursion(oracle, n):
    H = oracle.hadamard_dense(n).astype(np.int64)
    Hh = oracle.hadamard_dense(n // 2).astype(np.int64)
    assert np.array_equal(H, np.block([[Hh, Hh], [Hh, -Hh]]))


@pytest.mark.parametrize("a,b", [(2, 2), (4, 16), (16, 4), (64, 64), (32, 128), (1, 8)])
def test_kronecker_identity_entrywise(oracle, a, b):
    # H_{ab} = H_a (x) H_b: the identity the large-n route of the oracle relies on.
    Hab = oracle.hadamard_dense(a * b).astype(np.int64)
    kron = np.kron(oracle.hadamard_dense(a).astype(np.int64), oracle.hadamard_dense(b).astype(np.int64))
    assert np.array_equal(Hab, kron)


@pytest.mark.parametrize("n", [2, 32, 256, 2048])
def test_rows_orthogonal_exact_integers(oracle, n):
    H = oracle.hadamard_dense(n).astype(np.float64)      # exact in fp64 (|entries| <= n)
    assert np.array_equal(H @ H.T, n * np.eye(n))
    assert np.array_equal(H, H.T)


def test_rows_orthogonal_n4096_sampled(oracle):
    n = 4096
    H = oracle.hadamard_dense(n).astype(np.float64)
    rows = np.random.default_rng(7).choice(n, size=64, replace=False)
    G = H[rows] @ H.T
    want = np.zeros((64, n))
    want[np.arange(64), rows] = n
    assert np.array_equal(G, want)


def test_sign_function_matches_dense_at_large_indices(oracle):
    # spot checks far beyond what can be materialised
    assert oracle.hadamard_sign(0, (1 << 40) - 1) == 1
    assert oracle.hadamard_sign((1 << 20) - 1, (1 << 20) - 1) == 1      # 20 common bits
    assert oracle.hadamard_sign((1 << 19) - 1, (1 << 20) - 1) == -1     # 19 common bits
    assert oracle.hadamard_sign(0b1011, 0b0110) == -1                   # one common bit


@pytest.mark.parametrize("n,kron_a", [(64, 0), (64, 8), (1024, 0), (1024, 32), (2048, 64), (4096, 0)])
def test_normalised_apply_is_involution_and_isometry(oracle, n, kron_a):
    rng = np.random.default_rng(n + kron_a)
    t = rng.standard_normal((3, n))
    u = oracle.hadamard_apply(t, kron_a=kron_a)
    assert np.allclose(np.linalg.norm(u, axis=1), np.linalg.norm(t, axis=1), rtol=1e-12)
    assert np.allclose(oracle.hadamard_apply(u, kron_a=kron_a), t, rtol=0, atol=1e-11)


@pytest.mark.parametrize("n,kron_a", [(256, 0), (256, 16), (4096, 64)])
def test_apply_matches_library_matrix(oracle, n, kron_a):
    rng = np.random.default_rng(3)
    t = rng.standard_normal((2, n))
    want = (scipy.linalg.hadamard(n).astype(np.float64) @ t.T).T / math.sqrt(n)
    assert np.allclose(oracle.hadamard_apply(t, kron_a=kron_a), want, rtol=0, atol=1e-11)


@pytest.mark.parametrize("n", [16, 1024])
def test_canonical_vector_spreads_to_equal_magnitudes(oracle, n):
    # H e_j has every entry of magnitude exactly 1/sqrt(n) (perfectly balanced).
    for j in (0, 1, n - 1):
        e = np.zeros(n)
        e[j] = 1.0
        u = oracle.hadamard_apply(e)
        assert np.allclose(np.abs(u), 1.0 / math.sqrt(n), rtol=1e-15)
    ones = oracle.hadamard_apply(np.ones(n))
    want = np.zeros(n)
    want[0] = math.sqrt(n)
    assert np.allclose(ones, want, atol=1e-12)


@pytest.mark.slow
def test_balancedness_of_HD_at_n_2p20(oracle):
    # Remark 1 / its proof: for unit x, P[ ||H D x||_inf > log(n)/sqrt(n) ] <= 2 n exp(-log^2(n)/8),
    # about 8e-5 at n = 2^20, so a single draw must satisfy the bound.  Uses the
    # Kronecker route (H_1024 (x) H_1024), the only one possible at this size.
    n = 1 << 20
    rng = np.random.default_rng(11)
    x = np.zeros(n)
    x[rng.choice(n, size=64, replace=False)] = rng.standard_normal(64)   # a spiky unit vector
    x /= np.linalg.norm(x)
    d = 1.0 - 2.0 * rng.integers(0, 2, size=n)
    u = oracle.hadamard_apply(d * x, kron_a=1024)
    assert abs(np.linalg.norm(u) - 1.0) < 1e-12
    assert np.max(np.abs(u)) <= math.log(n) / math.sqrt(n)
    assert 2 * n * math.exp(-math.log(n) ** 2 / 8) < 1e-4
