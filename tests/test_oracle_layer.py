"""CPU pins for the oracle's adaptive-layer functions (Section 1 / Section 3.2: diagonals that are learned;
Section 5: the HD3HD2HD1 block as a neural-network layer): forward activations and the backward pass."""
import math

import numpy as np
import pytest
import scipy.linalg


def _case(n, batch, seed):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((batch, n))
    d = rng.standard_normal((3, n)) + 0.3            # learned diagonals: arbitrary reals
    dy = rng.standard_normal((batch, n))
    return x, d, dy


def test_forward_matches_the_plain_spinner_and_its_activations(oracle):
    x, d, _ = _case(64, 5, 1)
    y, b1, b2 = oracle.layer_forward(x, d[0], d[1], d[2], 1.5)
    assert np.allclose(y, 1.5 * oracle.spinner(x.astype(np.float32), d[0].astype(np.float32), d[1].astype(np.float32),
                                               d[2].astype(np.float32)), rtol=1e-5, atol=1e-5)
    H = scipy.linalg.hadamard(64) / 8.0
    assert np.allclose(b1, (x * d[0]) @ H, atol=1e-12)
    assert np.allclose(b2, (b1 * d[1]) @ H, atol=1e-12)
    assert np.allclose(y, 1.5 * (b2 * d[2]) @ H, atol=1e-12)


@pytest.mark.parametrize("n", [2, 4, 16, 64])
def test_backward_is_the_transposed_dense_jacobian(oracle, n):
    x, d, dy = _case(n, 4, 10 + n)
    s = 0.75
    H = scipy.linalg.hadamard(n) / math.sqrt(n)
    J = s * H @ np.diag(d[2]) @ H @ np.diag(d[1]) @ H @ np.diag(d[0])          # y = J x
    dx, dd = oracle.layer_backward(x, d[0], d[1], d[2], dy, s)
    assert np.allclose(dx, dy @ J, atol=1e-12)                                   # rows: J^T dy
    # derivative of y with respect to each diagonal entry, column by column
    a1 = x * d[0]
    b1 = a1 @ H
    b2 = (b1 * d[1]) @ H
    for k, (left, act) in enumerate([(s * H @ np.diag(d[2]) @ H @ np.diag(d[1]) @ H, x),
                                     (s * H @ np.diag(d[2]) @ H, b1),
                                     (s * H, b2)]):
        want = np.zeros(n)
        for i in range(n):
            # dy/dd_k[i] = left[:, i] * act[:, i] per sample
            want[i] = sum(dy[b] @ left[:, i] * act[b, i] for b in range(x.shape[0]))
        assert np.allclose(dd[k], want, atol=1e-11), k


def test_backward_against_central_differences(oracle):
    n, batch, s, h = 16, 3, 1.25, 1e-6
    x, d, w = _case(n, batch, 5)

    def loss(xx, dd):
        y, _, _ = oracle.layer_forward(xx, dd[0], dd[1], dd[2], s)
        return float((w * y).sum())

    dx, dd = oracle.layer_backward(x, d[0], d[1], d[2], w, s)
    for (b, i) in [(0, 0), (1, 7), (2, 15)]:
        e = np.zeros_like(x); e[b, i] = h
        assert abs((loss(x + e, d) - loss(x - e, d)) / (2 * h) - dx[b, i]) < 1e-6
    for k in range(3):
        for i in (0, 3, 15):
            e = np.zeros_like(d); e[k, i] = h
            assert abs((loss(x, d + e) - loss(x, d - e)) / (2 * h) - dd[k, i]) < 1e-6


def test_backward_adjoint_identity_and_special_cases(oracle):
    x, d, dy = _case(128, 6, 9)
    y, _, _ = oracle.layer_forward(x, d[0], d[1], d[2], 2.0)
    dx, dd = oracle.layer_backward(x, d[0], d[1], d[2], dy, 2.0)
    assert abs((dy * y).sum() - (dx * x).sum()) < 1e-9 * abs((dy * y).sum()) + 1e-9      # <dy, Jx> = <J^T dy, x>
    # the layer is linear in each diagonal: sum_i d_k[i] * dd_k[i] = <dy, y> for every k
    for k in range(3):
        assert abs((d[k] * dd[k]).sum() - (dy * y).sum()) < 1e-9 * abs((dy * y).sum()) + 1e-9
    # identity diagonals: dx = scale * H dy
    ones = np.ones(128)
    dx1, _ = oracle.layer_backward(x, ones, ones, ones, dy, 0.5)
    assert np.allclose(dx1, 0.5 * dy @ (scipy.linalg.hadamard(128) / math.sqrt(128)), atol=1e-12)


def test_backward_closed_form_n2(oracle):
    # n = 2: H = [[1, 1], [1, -1]] / sqrt 2.  With D2 = D3 = I the layer is y = s H H H D1 x = s H D1 x, so
    # dx = s D1 H dy and dd1 = s x * (H dy), written out by hand for one sample.
    s, r = 3.0, 1.0 / math.sqrt(2.0)
    x = np.array([[2.0, -1.0]]); dy = np.array([[0.5, 4.0]]); d1 = np.array([1.5, -2.0]); one = np.ones(2)
    hdy = np.array([r * (0.5 + 4.0), r * (0.5 - 4.0)])
    dx, dd = oracle.layer_backward(x, d1, one, one, dy, s)
    assert np.allclose(dx[0], [s * 1.5 * hdy[0], s * -2.0 * hdy[1]], atol=1e-14)
    assert np.allclose(dd[0], [s * 2.0 * hdy[0], s * -1.0 * hdy[1]], atol=1e-14)
