"""CPU pins for the oracle's G_struct D2 H D1 members (Lemma 1 and the remark after it: Gaussian circulant,
Toeplitz, Hankel third blocks; Section 5 also uses the skew-circulant one)."""
import math

import numpy as np
import pytest
import scipy.linalg


def test_structured_matrices_match_library_constructions(oracle):
    n = 8
    rng = np.random.default_rng(1)
    g = rng.standard_normal(n)
    t = rng.standard_normal(2 * n - 1)
    # scipy's circulant has g as its first COLUMN; ours has it as the first row, shifted right row by row: the transpose
    assert np.array_equal(oracle.struct_matrix("circulant", g, n), scipy.linalg.circulant(g).T)
    # scipy.linalg.toeplitz(first column, first row): column = t[n-1], t[n-2], ..., t[0]; row = t[n-1], ..., t[2n-2]
    assert np.array_equal(oracle.struct_matrix("toeplitz", t, n), scipy.linalg.toeplitz(t[n - 1::-1], t[n - 1:]))
    assert np.array_equal(oracle.struct_matrix("hankel", t, n), scipy.linalg.hankel(t[:n], t[n - 1:]))
    S = oracle.struct_matrix("skew_circulant", g, n)
    C = oracle.struct_matrix("circulant", g, n)
    assert np.array_equal(np.triu(S), np.triu(C)) and np.array_equal(np.tril(S, -1), -np.tril(C, -1))
    # hand-typed 3 x 3 cases
    assert oracle.struct_matrix("circulant", [1, 2, 3], 3).tolist() == [[1, 2, 3], [3, 1, 2], [2, 3, 1]]
    assert oracle.struct_matrix("skew_circulant", [1, 2, 3], 3).tolist() == [[1, 2, 3], [-3, 1, 2], [-2, -3, 1]]
    assert oracle.struct_matrix("toeplitz", [1, 2, 3, 4, 5], 3).tolist() == [[3, 4, 5], [2, 3, 4], [1, 2, 3]]
    assert oracle.struct_matrix("hankel", [1, 2, 3, 4, 5], 3).tolist() == [[1, 2, 3], [2, 3, 4], [3, 4, 5]]


def test_circulant_product_is_a_cyclic_correlation(oracle):
    # (G v)_i = sum_j g[(j - i) mod n] v_j: a cyclic cross-correlation, i.e. ifft(conj(fft(g)) * fft(v)) for real g
    n = 64
    rng = np.random.default_rng(2)
    g, v = rng.standard_normal(n), rng.standard_normal(n)
    want = np.fft.ifft(np.conj(np.fft.fft(g)) * np.fft.fft(v)).real
    assert np.allclose(oracle.struct_matrix("circulant", g, n) @ v, want, atol=1e-12)


@pytest.mark.parametrize("kind", ["circulant", "skew_circulant", "toeplitz", "hankel"])
def test_struct_apply_is_the_dense_product(oracle, kind):
    n, m, batch = 32, 12, 5
    rng = np.random.default_rng(3)
    x = rng.standard_normal((batch, n)).astype(np.float32)
    d = (1.0 - 2.0 * rng.integers(0, 2, (2, n))).astype(np.float32)
    params = rng.standard_normal(n if "circ" in kind else 2 * n - 1).astype(np.float32)
    H = scipy.linalg.hadamard(n) / math.sqrt(n)
    M = oracle.struct_matrix(kind, params, n) @ np.diag(d[1]) @ H @ np.diag(d[0])
    got = oracle.struct_apply(x, kind, params, d[0], d[1], m, 1.5)
    assert got.shape == (batch, m)
    assert np.allclose(got, 1.5 * x.astype(np.float64) @ M[:m].T, atol=1e-11)
    # generator e_0 (circulant) gives the identity as third block
    if kind == "circulant":
        e0 = np.zeros(n); e0[0] = 1.0
        assert np.allclose(oracle.struct_apply(x, kind, e0, d[0], d[1], n, 1.0), (x * d[0]) @ H * d[1], atol=1e-12)


def test_gaussian_circulant_member_behaves_like_a_gaussian_projection(oracle):
    # Lemma 1 / Theorem 3: G_circ D2 H D1 x has coordinates that are N(0, |x|^2) each; check the second moment
    n = 256
    rng = np.random.default_rng(4)
    x = rng.standard_normal((1, n)).astype(np.float32)
    acc = []
    for k in range(40):
        g = rng.standard_normal(n)
        d = (1.0 - 2.0 * rng.integers(0, 2, (2, n))).astype(np.float32)
        acc.append(oracle.struct_apply(x, "circulant", g, d[0], d[1], n, 1.0)[0])
    y = np.concatenate(acc)
    assert abs(y.var() / float((x.astype(np.float64) ** 2).sum()) - 1.0) < 0.05
    assert abs(y.mean()) < 0.05 * y.std()


@pytest.mark.parametrize("kind", ["circulant", "skew_circulant", "toeplitz", "hankel"])
def test_selected_rows_are_rows_of_the_dense_matrix(oracle, kind):
    # the route for n too large for the dense matrix: rows written out one by one, checked against the dense matrix
    # (itself pinned against library constructions above) and against the FFT identity at a size the dense one
    # cannot reach
    n = 64
    rng = np.random.default_rng(5)
    params = rng.standard_normal(n if "circ" in kind else 2 * n - 1)
    rows = [0, 1, 17, 63]
    assert np.array_equal(oracle.struct_rows(kind, params, n, rows), oracle.struct_matrix(kind, params, n)[rows])
    x = rng.standard_normal((3, n)).astype(np.float32)
    d = rng.standard_normal((2, n)).astype(np.float32)
    want = oracle.struct_apply(x, kind, params, d[0], d[1], n, 0.7)[:, rows]
    assert np.allclose(oracle.struct_apply_rows(x, kind, params, d[0], d[1], rows, 0.7), want, atol=1e-12)


def test_selected_rows_at_a_large_size_against_the_fft_identity(oracle):
    n = 1 << 16
    rng = np.random.default_rng(6)
    g = rng.standard_normal(n)
    v = rng.standard_normal(n)
    rows = [0, 5, 40000, n - 1]
    want = np.fft.ifft(np.conj(np.fft.fft(g)) * np.fft.fft(v)).real[rows]
    assert np.allclose(oracle.struct_rows("circulant", g, n, rows) @ v, want, atol=1e-8)
    # Toeplitz rows are windows of the generating vector: row i is t[n - 1 - i : 2 n - 1 - i]
    t = rng.standard_normal(2 * n - 1)
    R = oracle.struct_rows("toeplitz", t, n, rows)
    for k, i in enumerate(rows):
        assert np.array_equal(R[k], t[n - 1 - i: 2 * n - 1 - i])
    # Hankel rows likewise: row i is h[i : i + n]
    R = oracle.struct_rows("hankel", t, n, rows)
    for k, i in enumerate(rows):
        assert np.array_equal(R[k], t[i: i + n])
