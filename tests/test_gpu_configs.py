"""Full-size parity on the five benchmark configurations, in the launch
configuration the benchmark times: the library runs on the whole batch, the
O(n^2) oracle checks a seeded sample of rows copied back from the buffer the
GPU consumed, and size-independent properties are checked on the whole output.
"""
import math
import sys

import numpy as np
import pytest

from helpers import REL_L2_TOL, check_hash_against_projection, rel_l2_per_vector
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
    import torch

    torch.cuda.empty_cache()


def _setup(g, name):
    w = W.CONFIGS[name]
    x = W.make_x_torch(w, g.dev)
    ds = W.diag_sets(w)
    dsd = g.torch.from_numpy(ds).to(g.dev)
    rows = W.sample_rows(w.batch, w.oracle_rows, w.seed)
    xs = x[g.torch.from_numpy(rows).to(g.dev)].cpu().numpy()
    return w, x, ds, dsd, rows, xs


def _norms(t):
    return t.double().pow(2).sum(dim=1).sqrt()


def test_cfg1_plain_n256(gpu, oracle):
    w, x, ds, dsd, rows, xs = _setup(gpu, "cfg1_plain_n256")
    y = gpu.b.spinner_apply(x, dsd[0, 0], dsd[0, 1], dsd[0, 2], w.m, w.epilogue, w.scale)
    want = oracle.apply(xs, ds[0, 0], ds[0, 1], ds[0, 2], w.m, "none", w.scale)
    err = rel_l2_per_vector(y.cpu().numpy()[rows], want)
    assert err.max() <= REL_L2_TOL, err.max()
    assert bool(((_norms(y) / _norms(x) - 1).abs() < 1e-5).all())          # isometry, whole batch
    # the form the benchmark times: +-1 diagonals as packed sign words
    ys = gpu.b.spinner_apply_signs(x, gpu.b.spinner_pack_signs(dsd), w.m, w.epilogue, w.scale)
    assert rel_l2_per_vector(ys.cpu().numpy()[rows], want).max() <= REL_L2_TOL
    assert bool(((_norms(ys) / _norms(x) - 1).abs() < 1e-5).all())


def test_cfg2_lsh_n1024(gpu, oracle):
    w, x, ds, dsd, rows, xs = _setup(gpu, "cfg2_lsh_n1024")
    h = gpu.b.spinner_hash(x, dsd)
    assert h.shape == (w.batch, w.L)
    _, ys = oracle.hash(xs, ds, return_y=True)
    exact, banded = check_hash_against_projection(h.cpu().numpy()[rows], ys)
    assert exact + banded == len(rows) * w.L
    assert banded <= 2
    # whole batch: range, antipodal symmetry, roughly uniform buckets, independent triples
    assert int(h.min()) >= 0 and int(h.max()) < 2 * w.n
    hn = gpu.b.spinner_hash(-x, dsd)
    assert bool(((h + w.n) % (2 * w.n) == hn).all())
    counts = gpu.torch.bincount(h[:, 0].long(), minlength=2 * w.n).double()
    expect = w.batch / (2 * w.n)
    chi2 = float(((counts - expect) ** 2 / expect).sum())
    assert chi2 < 2 * w.n + 8 * math.sqrt(4 * w.n)          # mean 2n-1, std sqrt(2(2n-1))
    assert float((h[:, 0] == h[:, 1]).double().mean()) < 5.0 / (2 * w.n)
    # the form the benchmark times: packed sign words (a kernel of its own at this size); sampled rows against the
    # oracle, and the whole batch against the fp32-diagonal kernel (they may part only where two coordinates tie)
    hs = gpu.b.spinner_hash_signs(x, gpu.b.spinner_pack_signs(dsd), w.L)
    exact, banded = check_hash_against_projection(hs.cpu().numpy()[rows], ys)
    assert exact + banded == len(rows) * w.L
    assert banded <= 2
    assert float((hs != h).double().mean()) < 1e-3


def test_cfg3_rff_n4096(gpu, oracle):
    w, x, ds, dsd, rows, xs = _setup(gpu, "cfg3_rff_n4096")
    f = gpu.b.spinner_apply(x, dsd[0, 0], dsd[0, 1], dsd[0, 2], w.m, w.epilogue, w.scale)
    assert f.shape == (w.batch, 2 * w.m)
    want = oracle.apply(xs, ds[0, 0], ds[0, 1], ds[0, 2], w.m, "cossin", w.scale)
    got = f[gpu.torch.from_numpy(rows).to(gpu.dev)].cpu().numpy()
    err = rel_l2_per_vector(got, want)
    assert err.max() <= REL_L2_TOL, err.max()
    step = 16384
    for s in range(0, w.batch, step):                       # ||features|| = 1 on the whole batch
        assert bool(((_norms(f[s:s + step]) - 1).abs() < 2e-6).all())
    # the form the benchmark times: +-1 diagonals as packed sign words (a kernel of its own at this size)
    del f
    signs = gpu.b.spinner_pack_signs(dsd)
    f = gpu.b.spinner_apply_signs(x, signs, w.m, w.epilogue, w.scale)
    got = f[gpu.torch.from_numpy(rows).to(gpu.dev)].cpu().numpy()
    err = rel_l2_per_vector(got, want)
    assert err.max() <= REL_L2_TOL, err.max()
    for s in range(0, w.batch, step):
        assert bool(((_norms(f[s:s + step]) - 1).abs() < 2e-6).all())


def test_cfg4_jl_n16384(gpu, oracle):
    w, x, ds, dsd, rows, xs = _setup(gpu, "cfg4_jl_n16384")
    f = gpu.b.spinner_apply(x, dsd[0, 0], dsd[0, 1], dsd[0, 2], w.m, w.epilogue, w.scale)
    assert f.shape == (w.batch, w.m)
    want = oracle.apply(xs, ds[0, 0], ds[0, 1], ds[0, 2], w.m, "none", w.scale)
    err = rel_l2_per_vector(f.cpu().numpy()[rows], want)
    assert err.max() <= REL_L2_TOL, err.max()
    # the form the benchmark times: packed sign words (wide exchanges, pruned last round)
    fs = gpu.b.spinner_apply_signs(x, gpu.b.spinner_pack_signs(dsd), w.m, w.epilogue, w.scale)
    assert rel_l2_per_vector(fs.cpu().numpy()[rows], want).max() <= REL_L2_TOL
    assert float(((fs - f).double().norm(dim=1) / f.double().norm(dim=1)).max()) <= REL_L2_TOL
    del fs
    # pairwise distances of 1000 seeded pairs, on the full-batch GPU output
    rng = np.random.default_rng(4)
    i = rng.integers(0, w.batch, 1000)
    j = (i + 1 + rng.integers(0, w.batch - 1, 1000)) % w.batch
    it, jt = (gpu.torch.from_numpy(a).to(gpu.dev) for a in (i, j))
    r = (_norms(f[it] - f[jt]) / _norms(x[it] - x[jt])).cpu().numpy()
    assert np.mean(np.abs(r - 1)) <= 0.03 and np.max(np.abs(r - 1)) <= 0.15, (np.mean(np.abs(r - 1)), np.max(np.abs(r - 1)))
    # the same statistic on the oracle's rows
    fo, xo = want, xs.astype(np.float64)
    ro = np.linalg.norm(fo[:-1] - fo[1:], axis=1) / np.linalg.norm(xo[:-1] - xo[1:], axis=1)
    assert np.max(np.abs(ro - 1)) <= 0.15


def test_cfg5_large_n2p20(gpu, oracle):
    w, x, ds, dsd, rows, xs = _setup(gpu, "cfg5_large_n2p20")
    y = gpu.b.spinner_apply(x, dsd[0, 0], dsd[0, 1], dsd[0, 2], w.m, w.epilogue, w.scale)
    want = oracle.apply(xs, ds[0, 0], ds[0, 1], ds[0, 2], w.m, "none", w.scale)
    err = rel_l2_per_vector(y.cpu().numpy()[rows], want)
    assert err.max() <= REL_L2_TOL, err.max()
    assert bool(((_norms(y) / _norms(x) - 1).abs() < 1e-5).all())
    # balancedness of the first block at this size (Remark 1): every |y_i| of a unit vector
    # stays below log(n)/sqrt(n); the full spinner output is balanced as well
    ymax = (y.abs().max(dim=1).values.double() / _norms(x)).max()
    assert float(ymax) <= math.log(w.n) / math.sqrt(w.n)
    # the form the benchmark times: packed sign words in all three diagonal passes, several slices
    ys = gpu.b.spinner_apply_signs(x, gpu.b.spinner_pack_signs(dsd), w.m, w.epilogue, w.scale)
    assert rel_l2_per_vector(ys.cpu().numpy()[rows], want).max() <= REL_L2_TOL
    assert float(((ys - y).double().norm(dim=1) / _norms(y)).max()) <= REL_L2_TOL


# ------------------------------------------------------------------ the rows beyond the five configurations, at the sizes bench.py times
def test_next_angular_n4096_full_size(gpu, oracle):
    from helpers import check_sign_bits, unpack_sign_codes

    w = W.NEXT["next_angular_n4096"]
    x = W.make_x_torch(w, gpu.dev)
    ds = W.diag_sets(w)
    signs = gpu.b.spinner_pack_signs(gpu.torch.from_numpy(ds).to(gpu.dev))
    codes = gpu.b.spinner_sign_codes_signs(x, signs, w.m)
    gpu.torch.cuda.synchronize()
    assert tuple(codes.shape) == (w.batch, w.m // 64)
    rows = W.sample_rows(w.batch, w.oracle_rows, w.seed)
    idx = gpu.torch.from_numpy(rows).to(gpu.dev)
    xs = x[idx].cpu().numpy()
    y = oracle.spinner(xs, ds[0, 0], ds[0, 1], ds[0, 2])
    check_sign_bits(unpack_sign_codes(codes[idx].cpu().numpy(), w.m), y, w.m)
    # size-independent property on the whole output: about half the bits are set in every code (balanced rows)
    v = codes.view(gpu.torch.int32)
    v = v - ((v >> 1) & 0x55555555)
    v = (v & 0x33333333) + ((v >> 2) & 0x33333333)
    v = (v + (v >> 4)) & 0x0F0F0F0F
    ones = ((v * 0x01010101) >> 24) & 0xFF            # popcount of every 32-bit half word
    frac = ones.sum(dim=1).double() / w.m
    assert float((frac - 0.5).abs().max()) < 0.06       # binomial: 4 sigma = 4 * 0.5 / sqrt(4096) = 0.031


def test_angular_gram_bench_size(gpu, oracle):
    # the shape bench.py times: 16384 x 16384 codes of 4096 bits (1 GiB of estimates); a sampled block of rows and
    # columns against the oracle, exact Hamming distances, and properties of the whole table
    from helpers import unpack_sign_codes

    t, b = gpu.torch, gpu.b
    rows, m = 16384, 4096
    g = t.Generator(device=gpu.dev)
    g.manual_seed(4096 + rows)
    codes = t.randint(-2**62, 2**62, (rows, m // 64), dtype=t.int64, device=gpu.dev, generator=g)
    codes[5] = codes[4]                              # a pair at distance 0 off the diagonal
    codes[7] = ~codes[6]                             # and one at distance m
    out = b.spinner_angular_gram(codes, codes, m)
    t.cuda.synchronize()
    assert tuple(out.shape) == (rows, rows)
    ri = W.sample_rows(rows, 48, 11)
    ci = W.sample_rows(rows, 48, 12)
    ri[:4] = [4, 5, 6, 7]
    ci[:4] = [5, 4, 7, 6]
    got = out[t.from_numpy(ri).to(gpu.dev)][:, t.from_numpy(ci).to(gpu.dev)].cpu().numpy()
    ba = unpack_sign_codes(codes[t.from_numpy(ri).to(gpu.dev)].cpu().numpy(), m)
    bb = unpack_sign_codes(codes[t.from_numpy(ci).to(gpu.dev)].cpu().numpy(), m)
    want = oracle.angular_estimate(ba, bb)
    assert np.array_equal(np.rint((1.0 - got.astype(np.float64)) * m), np.rint((1.0 - want) * m))
    assert got[0, 0] == 1.0 and got[1, 1] == 1.0 and got[2, 2] == 0.0 and got[3, 3] == 0.0
    # whole table: symmetric (a = b), ones on the diagonal, estimates of independent codes near 1/2
    assert bool((out.diagonal() == 1.0).all())
    step = 2048
    for s0 in range(0, rows, step):
        blk = out[s0:s0 + step]
        assert t.equal(blk, out[:, s0:s0 + step].t())
        assert float(blk.min()) >= 0.0 and float(blk.max()) <= 1.0
    off = out[8:, 8:].double()
    n_off = off.numel() - off.shape[0]
    mean = (off.sum() - off.diagonal().sum()) / n_off
    assert abs(float(mean) - 0.5) < 1e-3             # sd of one estimate 0.5 / sqrt(4096), averaged over 2.7e8 pairs
    del out, off


def test_adaptive_layer_full_size(gpu, oracle):
    # the shape bench.py times: n = 4096, batch 65536; sampled rows for y and dx, all of dd through linearity
    t, b = gpu.torch, gpu.b
    n, batch = 4096, 65536
    g = t.Generator(device=gpu.dev)
    g.manual_seed(20260)
    x = t.randn((batch, n), generator=g, device=gpu.dev, dtype=t.float32)
    dy = t.randn((batch, n), generator=g, device=gpu.dev, dtype=t.float32)
    d = 1.0 + 0.5 * t.randn((3, n), generator=g, device=gpu.dev, dtype=t.float32)
    y, saved = b.spinner_layer_forward(x, d[0], d[1], d[2], 1.0)
    dx, dd = b.spinner_layer_backward(dy, x, saved, d[0], d[1], d[2], 1.0)
    t.cuda.synchronize()
    rows = W.sample_rows(batch, 16, 99)
    idx = t.from_numpy(rows).to(gpu.dev)
    dn = d.cpu().numpy()
    xs, dys = x[idx].cpu().numpy(), dy[idx].cpu().numpy()
    wy, _, _ = oracle.layer_forward(xs, dn[0], dn[1], dn[2], 1.0)
    wdx, _ = oracle.layer_backward(xs, dn[0], dn[1], dn[2], dys, 1.0)
    assert rel_l2_per_vector(y[idx].cpu().numpy(), wy).max() <= REL_L2_TOL
    assert rel_l2_per_vector(dx[idx].cpu().numpy(), wdx).max() <= REL_L2_TOL
    # the layer is linear in each diagonal, so sum_i d_k[i] dd_k[i] = <dy, y> over the whole batch, for every k
    inner = float((dy.double() * y.double()).sum())
    for k in range(3):
        got = float((d[k].double() * dd[k].double()).sum())
        assert abs(got - inner) <= 1e-5 * abs(inner) + 1e-2 * math.sqrt(batch * n), (k, got, inner)
    # and the batch sum is additive: the gradient of the whole batch is the sum of the gradients of its two halves
    h = batch // 2
    _, dd_a = b.spinner_layer_backward(dy[:h], x[:h], saved.view(2, batch, n)[:, :h].contiguous(), d[0], d[1], d[2], 1.0)
    _, dd_b = b.spinner_layer_backward(dy[h:], x[h:], saved.view(2, batch, n)[:, h:].contiguous(), d[0], d[1], d[2], 1.0)
    t.cuda.synchronize()
    num = (dd_a.double() + dd_b.double() - dd.double()).norm(dim=1)
    assert float((num / dd.double().norm(dim=1)).max()) <= REL_L2_TOL


def test_newton_sketch_bench_size(gpu, oracle):
    # n = 2^16, d = 512, m = 2048 as in bench.py; the O(n^2) oracle checks a few columns, the Gram matrix all of B
    n, d, m = 1 << 16, 512, 2048
    A, wts = W.newton_sketch_problem(n, d, 31337)
    dg = W.rademacher_diagonals(n, 3, 31338)
    scale = math.sqrt(n / m)
    At = gpu.torch.from_numpy(A).to(gpu.dev)
    B = gpu.b.spinner_sketch(At, gpu.torch.from_numpy(wts).to(gpu.dev), *[gpu.torch.from_numpy(dg[k]).to(gpu.dev) for k in range(3)],
                             m, scale)
    G = gpu.b.spinner_sketch_gram(B)
    gpu.torch.cuda.synchronize()
    cols = np.array([0, 1, 255, 300, 511])
    want = oracle.sketch(A[:, cols], wts, dg[0], dg[1], dg[2], m, scale)
    Bn = B.cpu().numpy()
    assert rel_l2_per_vector(Bn[:, cols].T, want.T).max() <= REL_L2_TOL
    Gw = oracle.sketched_gram(Bn)
    assert np.linalg.norm(G.cpu().numpy() - Gw) <= 1e-5 * np.linalg.norm(Gw)
    # the sketched Hessian approximates A^T W A: relative error of order sqrt(d / m) (loose bound)
    WA = (A * wts[:, None]).astype(np.float64)
    exact = WA.T @ WA
    assert np.linalg.norm(Gw - exact) / np.linalg.norm(exact) < 0.5


def test_more_than_2_to_32_elements(gpu, oracle):
    # 64-bit indexing: 5 * 2^20 vectors of 1024 floats are 5.4e9 elements (20 GiB in, 20 GiB out); sampled rows
    # against the oracle, among them the last rows, whose element offsets do not fit 32 bits
    t, b = gpu.torch, gpu.b
    n, batch = 1024, 5 << 20
    g = t.Generator(device=gpu.dev)
    g.manual_seed(77)
    x = t.empty((batch, n), dtype=t.float32, device=gpu.dev)
    step = 1 << 20
    for s in range(0, batch, step):
        x[s:s + step] = t.randn((step, n), generator=g, device=gpu.dev, dtype=t.float32)
    ds = W.rademacher_diagonals(n, 3, 78)
    dsd = t.from_numpy(ds).to(gpu.dev)
    signs = b.spinner_pack_signs(dsd[None].contiguous())
    out = b.spinner_apply_signs(x, signs, n, "none", 1.0)
    t.cuda.synchronize()
    rows = np.array([0, 1, (1 << 21) - 1, 1 << 21, (1 << 22) + 5, batch - 2, batch - 1])
    idx = t.from_numpy(rows).to(gpu.dev)
    want = oracle.apply(x[idx].cpu().numpy(), ds[0], ds[1], ds[2], n, "none", 1.0)
    assert rel_l2_per_vector(out[idx].cpu().numpy(), want).max() <= REL_L2_TOL
    # isometry on the whole output, in chunks
    for s in range(0, batch, step):
        a, c = _norms(out[s:s + step]), _norms(x[s:s + step])
        assert float(((a - c).abs() / c).max()) < 1e-5
    del out
    t.cuda.empty_cache()
    idx_out = b.spinner_hash_signs(x, signs, 1)
    t.cuda.synchronize()
    hw = oracle.hash(x[idx].cpu().numpy(), ds[None])
    assert np.array_equal(idx_out[idx].cpu().numpy(), hw)
