"""Pins of the oracle route for the largest sizes (two dense matrix products per round).

The route is checked against the plain-loop oracle (dense H_n and explicit Kronecker factors), against columns of H
given by the popcount formula, and against the invariants of an orthogonal product.
"""
import numpy as np
import pytest

from oracle import spinner_oracle as oracle


def _case(n, batch, seed, gaussian=True):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((batch, n)).astype(np.float32)
    if gaussian:
        d = rng.standard_normal((3, n)).astype(np.float32) + np.float32(0.25)
    else:
        d = (1.0 - 2.0 * rng.integers(0, 2, (3, n))).astype(np.float32)
    return x, d


@pytest.mark.parametrize("log2n", [2, 3, 6, 9, 12])
def test_matches_the_dense_definition(log2n):
    n = 1 << log2n
    x, d = _case(n, 3, 40 + log2n)
    want = oracle.spinner(x, d[0], d[1], d[2], kron_a=0)
    got = oracle.spinner_by_products(x, d[0], d[1], d[2])
    assert np.abs(got - want).max() <= 1e-12 * np.abs(want).max()


@pytest.mark.parametrize("log2n", [15, 17])
def test_matches_the_plain_loops_with_their_own_split(log2n):
    # the plain-loop oracle splits 2^15 as 2^8 x 2^7 (its default) or, forced here, 2^10 x 2^5: a different
    # factorisation than the 2^8 x 2^7 / 2^9 x 2^8 views of the product route
    n = 1 << log2n
    x, d = _case(n, 1, 50 + log2n)
    want = oracle.spinner(x, d[0], d[1], d[2], kron_a=1 << 10)
    got = oracle.spinner_by_products(x, d[0], d[1], d[2])
    assert np.abs(got - want).max() <= 1e-12 * np.abs(want).max()


def test_unit_vectors_give_columns_of_h():
    # identity diagonals: e_j -> H H H e_j = H e_j, entries (-1)^popcount(i & j) / sqrt(n)
    n = 1 << 18
    js = [0, 1, 77777, n - 1]
    x = np.zeros((len(js), n), dtype=np.float32)
    for k, j in enumerate(js):
        x[k, j] = 1.0
    one = np.ones(n, dtype=np.float32)
    y = oracle.spinner_by_products(x, one, one, one)
    i = np.arange(n, dtype=np.int64)
    for k, j in enumerate(js):
        par = np.zeros(n, dtype=np.int64)
        v = i & j
        for s in range(18):
            par ^= (v >> s) & 1
        want = (1.0 - 2.0 * par) / np.sqrt(float(n))
        assert np.abs(y[k] - want).max() <= 1e-15


def test_orthogonal_for_sign_diagonals_and_order_of_the_diagonals():
    n = 1 << 16
    x, d = _case(n, 2, 7, gaussian=False)
    y = oracle.spinner_by_products(x, d[0], d[1], d[2])
    assert np.abs(np.linalg.norm(y, axis=1) / np.linalg.norm(x.astype(np.float64), axis=1) - 1).max() <= 1e-12
    # the inverse of H D3 H D2 H D1 is D1 H D2 H D3 H: applying (1, d3, d2) to y and multiplying by d1 returns x
    one = np.ones(n, dtype=np.float32)
    # y is fp64: feed it as two fp32 parts so that nothing is lost in the cast
    hi = y.astype(np.float32)
    lo = (y - hi.astype(np.float64)).astype(np.float32)
    z = oracle.spinner_by_products(hi, one, d[2], d[1]) + oracle.spinner_by_products(lo, one, d[2], d[1])
    assert np.abs(z * d[0].astype(np.float64) - x.astype(np.float64)).max() <= 1e-9
    # swapping two diagonals changes the result
    y2 = oracle.spinner_by_products(x, d[1], d[0], d[2])
    assert np.abs(y2 - y).max() > 1e-3
