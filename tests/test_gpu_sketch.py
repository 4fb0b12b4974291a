"""GPU parity of the Newton-sketch step (Supplement, "Additional experiments"): B = S diag(w) A with S the first
m rows of a spinner acting on the columns of A, and the sketched Gram matrix B^T B, through the C ABI, against the
fp64 oracle.  Tolerance: relative L2 error <= 1e-5 per column of B; relative Frobenius error <= 1e-5 for B^T B."""
import math
import sys

import numpy as np
import pytest

from helpers import REL_L2_TOL, rel_l2_per_vector
from paper_1610_06209_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch

    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1610_06209_amd import binding

    class G:
        pass

    g = G()
    g.torch = torch
    g.b = binding
    g.dev = torch.device("cuda:0")
    return g


@pytest.fixture(autouse=True)
def _announce(request):
    print("\n[gpu-case] %s" % request.node.nodeid, file=sys.stderr, flush=True)
    yield


def _to(g, a):
    return g.torch.from_numpy(np.ascontiguousarray(a)).to(g.dev)


@pytest.mark.parametrize("n,d,m,weights", [(256, 37, 64, True), (256, 1, 1, False), (4096, 100, 513, True),
                                           (1024, 129, 1024, True), (16384, 24, 2048, False), (1 << 17, 6, 1000, True),
                                           (1 << 17, 3, 1 << 17, False)])
def test_sketch_matches_oracle(gpu, oracle, n, d, m, weights):
    A, w = W.newton_sketch_problem(n, d, 8000 + d)
    if not weights:
        w = None
    dg = W.rademacher_diagonals(n, 3, 8100 + d)
    scale = math.sqrt(n / m)
    B = gpu.b.spinner_sketch(_to(gpu, A), _to(gpu, w) if weights else None, _to(gpu, dg[0]), _to(gpu, dg[1]),
                             _to(gpu, dg[2]), m, scale)
    gpu.torch.cuda.synchronize()
    B = B.cpu().numpy()
    want = oracle.sketch(A, w, dg[0], dg[1], dg[2], m, scale)
    assert B.shape == (m, d)
    err = rel_l2_per_vector(B.T, want.T)                     # one vector per column of A
    assert err.max() <= REL_L2_TOL, err.max()


@pytest.mark.parametrize("log2n", list(range(4, 13)))
def test_sketch_on_the_columns_as_they_lie(gpu, oracle, log2n):
    # Shapes that take the kernel which loads the columns of the row-major matrix directly (n <= 2^12, d a multiple
    # of 4 and wide enough for its size): a last column group of 4 columns, several workgroups, the 32-column tiles
    # (d >= 8192, n <= 2^11); general (non +-1) diagonals, so that a swapped or dropped diagonal would show; m ragged,
    # m = n and m = 1.  Columns are independent, so wide matrices are compared on sampled columns.
    n = 1 << log2n
    rng = np.random.default_rng(8300 + log2n)
    dmin = 4096 if log2n == 12 else (1024 if log2n == 11 else 64)
    shapes = [(dmin + 4, max(1, n // 2 - 3), True), (dmin + 256, n, False), (dmin, 1, True)]
    if log2n in (4, 8, 11):
        shapes.append((8192 + 4, max(1, n // 4 + 1), True))
    for d, m, weights in shapes:
        assert gpu.b.spinner_sketch_workspace_bytes(n, d, m) > 0
        A, w = W.newton_sketch_problem(n, d, 8400 + log2n + d)
        dg = (rng.standard_normal((3, n)) * 0.5 + 1.0).astype(np.float32)
        scale = math.sqrt(n / m)
        B = gpu.b.spinner_sketch(_to(gpu, A), _to(gpu, w) if weights else None, _to(gpu, dg[0]), _to(gpu, dg[1]),
                                 _to(gpu, dg[2]), m, scale)
        gpu.torch.cuda.synchronize()
        assert B.shape == (m, d)
        B = B.cpu().numpy().astype(np.float64)
        cols = np.arange(d) if d <= 400 else np.unique(np.concatenate([np.arange(0, 40), np.arange(d - 40, d), rng.integers(0, d, 60)]))
        want = oracle.sketch(A[:, cols], w if weights else None, dg[0], dg[1], dg[2], m, scale)
        got = B[:, cols]
        if m > 8:
            err = rel_l2_per_vector(got.T, want.T)
        else:      # a single kept coordinate can cancel to nothing: measure against the column's expected size
            WA = A[:, cols].astype(np.float64) * (w.astype(np.float64)[:, None] if weights else 1.0)
            ref = scale * math.sqrt(m / n) * np.linalg.norm(WA, axis=0)
            err = np.linalg.norm(got - want, axis=0) / np.maximum(ref, np.linalg.norm(want, axis=0))
        assert err.max() <= REL_L2_TOL, (d, m, err.max())


@pytest.mark.parametrize("m,d", [(1, 1), (7, 5), (64, 128), (1000, 129), (4096, 300), (513, 1024)])
def test_gram_matches_oracle(gpu, oracle, m, d):
    rng = np.random.default_rng(m * 7 + d)
    B = rng.standard_normal((m, d)).astype(np.float32)
    B[:, : d // 2] += 2.0                                    # correlated columns: large off-diagonal entries
    G = gpu.b.spinner_sketch_gram(_to(gpu, B))
    gpu.torch.cuda.synchronize()
    G = G.cpu().numpy().astype(np.float64)
    want = oracle.sketched_gram(B)
    assert G.shape == (d, d)
    assert np.linalg.norm(G - want) <= 1e-5 * np.linalg.norm(want)
    assert np.abs(G - G.T).max() <= 1e-5 * np.abs(want).max()


def test_full_sketch_gives_the_exact_hessian(gpu):
    # m = n, scale 1: S is orthogonal, so the sketched Hessian equals A^T W A
    n, d = 2048, 96
    A, w = W.newton_sketch_problem(n, d, 8200)
    dg = W.rademacher_diagonals(n, 3, 8201)
    B = gpu.b.spinner_sketch(_to(gpu, A), _to(gpu, w), _to(gpu, dg[0]), _to(gpu, dg[1]), _to(gpu, dg[2]), n, 1.0)
    G = gpu.b.spinner_sketch_gram(B)
    gpu.torch.cuda.synchronize()
    WA = A.astype(np.float64) * w.astype(np.float64)[:, None]
    want = WA.T @ WA
    assert np.linalg.norm(G.cpu().numpy() - want) <= 1e-5 * np.linalg.norm(want)


def test_sketch_argument_errors(gpu):
    b = gpu.b
    assert b.spinner_sketch_workspace_bytes(1024, 10, 64) >= (10 * 1024 + 10 * 64) * 4
    assert b.spinner_sketch_workspace_bytes(1000, 10, 64) == 0
    f = b.lib.spinner_sketch
    import ctypes
    one = ctypes.c_float(1.0)
    assert f(64, 1000, 4, None, 64, 64, 64, 16, one, 64, 64, None) == b.SPINNER_ERR_BAD_N
    assert f(64, 1024, 4, None, 64, 64, 64, 2000, one, 64, 64, None) == b.SPINNER_ERR_BAD_M
    assert f(64, 1024, 4, None, 64, 64, 64, 16, one, 64, None, None) == b.SPINNER_ERR_WORKSPACE
    assert f(None, 1024, 4, None, 64, 64, 64, 16, one, 64, 64, None) == b.SPINNER_ERR_NULL_PTR
    assert f(None, 1024, 0, None, None, None, None, 16, one, None, None, None) == b.SPINNER_OK
    assert b.lib.spinner_sketch_gram(None, 4, 4, 64, None, None) == b.SPINNER_ERR_NULL_PTR
    assert b.lib.spinner_sketch_gram(None, 0, 4, None, None, None) == b.SPINNER_OK
    assert b.spinner_sketch_gram_workspace_bytes(32, 16) == 0 and b.spinner_sketch_gram_workspace_bytes(4096, 128) > 0
    assert b.lib.spinner_sketch_gram(64, 4096, 128, 64, None, None) == b.SPINNER_ERR_WORKSPACE
