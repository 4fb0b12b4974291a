"""GPU parity of the G_struct D2 H D1 members (Gaussian circulant, skew-circulant, Toeplitz, Hankel third block),
through the C ABI, against the dense fp64 oracle.  Tolerance: relative L2 error <= 1e-5 per output vector."""
import sys

import numpy as np
import pytest

from helpers import REL_L2_TOL, rel_l2_per_vector

pytestmark = pytest.mark.gpu
KINDS = ["circulant", "skew_circulant", "toeplitz", "hankel"]


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


def _case(kind, n, batch, seed):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((batch, n)).astype(np.float32)
    d = (1.0 - 2.0 * rng.integers(0, 2, (2, n))).astype(np.float32)
    params = rng.standard_normal(n if "circ" in kind else 2 * n - 1).astype(np.float32)
    return x, d, params


def _run(g, kind, x, d, params, m, scale):
    n = x.shape[1]
    spec = g.b.spinner_struct_prepare(kind, _to(g, params), n)
    out = g.b.spinner_struct_apply(_to(g, x), kind, spec, _to(g, d[0]), _to(g, d[1]), m, scale)
    g.torch.cuda.synchronize()
    return out.cpu().numpy()


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("log2n", [5, 6, 7, 8, 9, 10, 11, 12, 13])
def test_struct_members_match_oracle(gpu, oracle, kind, log2n):
    n = 1 << log2n
    batch = 7 if log2n >= 12 else 33                     # odd: the last pair of vectors is half empty
    m = n if log2n % 2 else n // 4 + 3
    x, d, params = _case(kind, n, batch, 10000 + log2n)
    got = _run(gpu, kind, x, d, params, m, 1.25)
    want = oracle.struct_apply(x, kind, params, d[0], d[1], m, 1.25)
    assert got.shape == (batch, m)
    assert rel_l2_per_vector(got, want).max() <= REL_L2_TOL


@pytest.mark.parametrize("kind,log2n,batch", [("circulant", 15, 3), ("toeplitz", 14, 5), ("skew_circulant", 15, 2), ("hankel", 15, 3),
                                               ("circulant", 17, 4), ("toeplitz", 17, 1), ("hankel", 18, 2), ("circulant", 20, 2),
                                               ("toeplitz", 21, 1), ("circulant", 22, 1)])
def test_struct_members_with_transforms_through_global_memory(gpu, oracle, kind, log2n, batch):
    # transforms of 2^15 .. 2^22 points (spinner_struct_apply_ws): the dense matrix does not fit, so the oracle writes out
    # sampled rows of G_struct from the generating vector; first / last rows, rows around the block boundaries of the
    # transform and random ones; full width and a ragged row limit
    n = 1 << log2n
    x, d, params = _case(kind, n, batch, 10300 + log2n)
    rng = np.random.default_rng(log2n)
    rows = np.unique(np.concatenate([np.arange(0, 6), np.arange(n - 6, n), np.arange(4090, 4102), rng.integers(0, n, 60)]))
    spec = gpu.b.spinner_struct_prepare(kind, _to(gpu, params), n)
    assert gpu.b.spinner_struct_workspace_bytes(kind, n, batch) > 0
    got = gpu.b.spinner_struct_apply_ws(_to(gpu, x), kind, spec, _to(gpu, d[0]), _to(gpu, d[1]), n, 1.25).cpu().numpy()
    want = oracle.struct_apply_rows(x, kind, params, d[0], d[1], rows, 1.25)
    assert got.shape == (batch, n)
    assert rel_l2_per_vector(got[:, rows], want).max() <= REL_L2_TOL
    m = n // 2 + 5
    got_m = gpu.b.spinner_struct_apply_ws(_to(gpu, x), kind, spec, _to(gpu, d[0]), _to(gpu, d[1]), m, 1.25).cpu().numpy()
    assert got_m.shape == (batch, m) and np.array_equal(got_m, got[:, :m])
    with pytest.raises(gpu.b.SpinnerError):
        gpu.b.spinner_struct_apply(_to(gpu, x), kind, spec, _to(gpu, d[0]), _to(gpu, d[1]), n, 1.0)      # no workspace: stops at 2^14 points


def test_struct_apply_with_workspace_is_the_plain_call_while_the_transform_fits_the_lds(gpu):
    for kind, n in (("circulant", 1 << 14), ("toeplitz", 2048), ("hankel", 64)):
        x, d, params = _case(kind, n, 5, 10400 + n)
        spec = gpu.b.spinner_struct_prepare(kind, _to(gpu, params), n)
        assert gpu.b.spinner_struct_workspace_bytes(kind, n, 5) == 0
        a = gpu.b.spinner_struct_apply(_to(gpu, x), kind, spec, _to(gpu, d[0]), _to(gpu, d[1]), n // 2, 0.5)
        b = gpu.b.spinner_struct_apply_ws(_to(gpu, x), kind, spec, _to(gpu, d[0]), _to(gpu, d[1]), n // 2, 0.5)
        assert gpu.torch.equal(a, b)


def test_circulant_at_the_largest_size_and_special_generators(gpu, oracle):
    n, batch = 1 << 14, 3
    x, d, params = _case("circulant", n, batch, 10100)
    got = _run(gpu, "circulant", x, d, params, n, 1.0)
    want = oracle.struct_apply(x, "circulant", params, d[0], d[1], n, 1.0)
    assert rel_l2_per_vector(got, want).max() <= REL_L2_TOL
    # generator e_0: the third block is the identity, so the result is D2 H D1 x
    n = 1024
    x, d, _ = _case("circulant", n, 5, 10101)
    e0 = np.zeros(n, dtype=np.float32); e0[0] = 1.0
    got = _run(gpu, "circulant", x, d, e0, n, 1.0)
    ones = np.ones(n, dtype=np.float32)
    want = oracle.struct_apply(x, "circulant", e0, d[0], d[1], n, 1.0)
    assert rel_l2_per_vector(got, want).max() <= REL_L2_TOL
    # a Toeplitz matrix built from a circulant generator is that circulant
    g = np.random.default_rng(5).standard_normal(n).astype(np.float32)
    t = np.concatenate([g[1:], g])                       # t[j - i + n - 1] = g[(j - i) mod n]
    a = _run(gpu, "toeplitz", x, d, t, n, 1.0)
    b = _run(gpu, "circulant", x, d, g, n, 1.0)
    assert rel_l2_per_vector(a, b.astype(np.float64)).max() <= 2e-6


def test_struct_argument_errors(gpu):
    import ctypes
    b = gpu.b
    assert b.lib.spinner_struct_params(0, 1024) == 1024 and b.lib.spinner_struct_params(2, 1024) == 2047
    assert b.lib.spinner_struct_spectrum_bytes(0, 1024) == 1024 * 8 + 512 * 8
    assert b.lib.spinner_struct_spectrum_bytes(2, 1024) == 2048 * 8 + 1024 * 8
    # transforms beyond the LDS (2^15 .. 2^22 points) also carry the twiddle table of their blocks of 2^12 points
    assert b.lib.spinner_struct_spectrum_bytes(2, 1 << 14) == (1 << 15) * 8 + (1 << 14) * 8 + 2048 * 8
    assert b.lib.spinner_struct_spectrum_bytes(0, 1 << 23) == 0 and b.lib.spinner_struct_spectrum_bytes(2, 1 << 22) == 0
    assert b.lib.spinner_struct_spectrum_bytes(0, 16) == 0
    assert b.spinner_struct_workspace_bytes(0, 1 << 14, 5) == 0 and b.spinner_struct_workspace_bytes(2, 1 << 13, 5) == 0
    assert b.spinner_struct_workspace_bytes(2, 1 << 14, 5) == 5 * (1 << 14) * 4 + 3 * (1 << 15) * 8
    g = b.lib.spinner_struct_apply_ws
    assert g(64, 1 << 14, 4, 2, 64, 64, 64, 16, ctypes.c_float(1.0), 64, None, None) == b.SPINNER_ERR_WORKSPACE
    assert g(64, 1 << 23, 4, 0, 64, 64, 64, 16, ctypes.c_float(1.0), 64, 64, None) == b.SPINNER_ERR_UNSUPPORTED
    assert b.lib.spinner_struct_spectrum_bytes(7, 1024) == 0
    one = ctypes.c_float(1.0)
    f = b.lib.spinner_struct_apply
    assert f(64, 1024, 4, 9, 64, 64, 64, 1024, one, 64, None) == b.SPINNER_ERR_BAD_EPILOGUE
    assert f(64, 1000, 4, 0, 64, 64, 64, 1000, one, 64, None) == b.SPINNER_ERR_BAD_N
    assert f(64, 1 << 14, 4, 2, 64, 64, 64, 16, one, 64, None) == b.SPINNER_ERR_UNSUPPORTED
    assert f(64, 1024, 4, 0, 64, 64, 64, 2000, one, 64, None) == b.SPINNER_ERR_BAD_M
    assert f(64, 1024, 4, 0, 64, 64, 64, 1024, one, 72, None) == b.SPINNER_ERR_ALIGNMENT
    assert f(64, 1024, 4, 0, None, 64, 64, 1024, one, 64, None) == b.SPINNER_ERR_NULL_PTR
    assert f(None, 1024, 0, 0, None, None, None, 1024, one, None, None) == b.SPINNER_OK
