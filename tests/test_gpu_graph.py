"""The entry points a serving loop would capture into a HIP graph: projection from sign words (plain, features,
stacked blocks), hashing, sign codes, and the Gram entry point that allocates nothing.  Every replay, with the
program's own eager work and synchronisations in between, must give the bits of the eager calls.  (The library records
no memset nodes: it clears nothing with hipMemsetAsync.)"""
import sys

import numpy as np
import pytest

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


def test_projection_hash_codes_and_gram_as_a_captured_graph(gpu):
    print("\n[gpu-case] graph capture of apply_signs / apply_blocks / hash_signs / sign_codes_signs / sketch_gram_static",
          file=sys.stderr, flush=True)
    t, b = gpu.torch, gpu.b
    n, batch, L = 1024, 300, 3
    rng = np.random.default_rng(31)
    x = t.from_numpy(rng.standard_normal((batch, n)).astype(np.float32)).to(gpu.dev)
    ds = t.from_numpy(W.rademacher_diagonals(n, 3 * L, 32).reshape(L, 3, n)).to(gpu.dev)
    signs = b.spinner_pack_signs(ds)
    Bm = t.from_numpy(rng.standard_normal((700, 129)).astype(np.float32)).to(gpu.dev)

    # eager results (each call allocates its own output here)
    y0 = b.spinner_apply_signs(x, signs)
    f0 = b.spinner_apply_signs(x, signs, 512, "cossin", 3.0, triple=1)
    k0 = b.spinner_apply_blocks(x, ds, 256, "cossin", 2.0)
    h0 = b.spinner_hash_signs(x, signs, L)
    c0 = b.spinner_sign_codes_signs(x, signs, n)
    G0 = b.spinner_sketch_gram(Bm)
    t.cuda.synchronize()

    y, f, k, h, c = (t.zeros_like(a) for a in (y0, f0, k0, h0, c0))
    Gs = t.zeros_like(G0)

    def step():
        b.spinner_apply_signs(x, signs, out=y)
        b.spinner_apply_signs(x, signs, 512, "cossin", 3.0, triple=1, out=f)
        b.spinner_apply_blocks(x, ds, 256, "cossin", 2.0, out=k)
        b.spinner_hash_signs(x, signs, L, out_idx=h)
        b.spinner_sign_codes_signs(x, signs, n, codes=c)
        b.spinner_sketch_gram_static(Bm, Gs)          # no workspace, no allocation: the library's built-in scratch

    side = t.cuda.Stream()
    side.wait_stream(t.cuda.current_stream())
    with t.cuda.stream(side):
        step()
    t.cuda.current_stream().wait_stream(side)
    t.cuda.synchronize()
    graph = t.cuda.CUDAGraph()
    with t.cuda.graph(graph):
        step()
        step()
    for rep in range(3):
        for buf in (y, f, k, Gs):
            buf.fill_(float(rep + 1))                  # eager work between replays
        h.fill_(-1)
        c.zero_()
        t.cuda.synchronize()
        graph.replay()
        t.cuda.synchronize()
        assert t.equal(y, y0) and t.equal(f, f0) and t.equal(k, k0), rep
        assert t.equal(h, h0) and t.equal(c, c0) and t.equal(Gs, G0), rep
