"""The entry point that allocates nothing (spinner_sketch_gram_static) against the entry point it is a variant
of (spinner_sketch_gram), through the C ABI: two calls in a row that share the library's built-in scratch, the
second with a smaller input, then the size limit.  Same kernels, same order of additions: results are bit-identical,
and both stay within the 1e-5 relative Frobenius bound of the fp64 oracle."""
import ctypes
import sys

import numpy as np
import pytest

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


def _case(g, m, d, seed):
    rng = np.random.default_rng(seed)
    B = rng.standard_normal((m, d)).astype(np.float32)
    B[:, : d // 2] += 2.0
    return B, g.torch.from_numpy(B).to(g.dev)


def test_static_scratch_gram_matches_the_workspace_entry_point(gpu, oracle):
    t, b = gpu.torch, gpu.b
    print("\n[gpu-case] spinner_sketch_gram_static: m=2048 d=512, then m=300 d=129", file=sys.stderr, flush=True)
    B1, B1d = _case(gpu, 2048, 512, 1)        # 16 slabs of 1 MiB: the whole built-in buffer
    B2, B2d = _case(gpu, 300, 129, 2)         # smaller problem, 5 slabs, right behind it on the same stream
    assert b.spinner_sketch_gram_workspace_bytes(2048, 512) == b.spinner_sketch_gram_static_limit() == 16 << 20
    assert 0 < b.spinner_sketch_gram_workspace_bytes(300, 129) < 16 << 20
    G1 = t.empty((512, 512), dtype=t.float32, device=gpu.dev)
    G2 = t.empty((129, 129), dtype=t.float32, device=gpu.dev)
    b.spinner_sketch_gram_static(B1d, G1)
    b.spinner_sketch_gram_static(B2d, G2)
    t.cuda.synchronize()
    R1 = b.spinner_sketch_gram(B1d)
    R2 = b.spinner_sketch_gram(B2d)
    t.cuda.synchronize()
    assert t.equal(G1, R1) and t.equal(G2, R2)
    for G, B in ((G1, B1), (G2, B2)):
        want = oracle.sketched_gram(B)
        assert np.linalg.norm(G.cpu().numpy().astype(np.float64) - want) <= 1e-5 * np.linalg.norm(want)
    # a third call, larger again: what the smaller call left in the buffer does not leak into the result
    b.spinner_sketch_gram_static(B1d, G1)
    t.cuda.synchronize()
    assert t.equal(G1, R1)


def test_static_scratch_gram_limit_and_errors(gpu):
    b = gpu.b
    f = b.lib.spinner_sketch_gram_static
    # d = 384 with many rows wants 29 slabs of 576 KiB: above the 16 MiB built in
    assert b.spinner_sketch_gram_workspace_bytes(4096, 384) > b.spinner_sketch_gram_static_limit()
    assert f(64, 4096, 384, 64, None) == b.SPINNER_ERR_SCRATCH_LIMIT
    assert "scratch" in b.spinner_strerror(b.SPINNER_ERR_SCRATCH_LIMIT)
    assert f(None, 64, 64, 64, None) == b.SPINNER_ERR_NULL_PTR
    assert f(64, 64, 64, 72, None) == b.SPINNER_ERR_ALIGNMENT
    assert f(None, 0, 64, None, None) == b.SPINNER_OK
    assert f(64, -1, 64, 64, None) == b.SPINNER_ERR_BAD_BATCH
