"""TEST INFRASTRUCTURE - NOT PART OF THE PRODUCT PATH.

Python face of the dense-matrix CPU oracle (``spinner_oracle.c``) for the
structured spinner ``y = H D3 H D2 H D1 x`` and the three downstream steps the
paper attaches to it.  Only ``tests/``, the smoke check and the benchmark's
``cpu_baseline`` leg may import this module; it imports nothing from the HIP
package and shares no code with it.

What each function follows:

* ``spinner``            - Section 1 / Section 3 (the HD3HD2HD1 member of the
  family; H is the L2-normalised Hadamard matrix, D_i diagonal).
* ``spinner_by_products`` - the same product for the largest n, where the plain loops of ``spinner`` take minutes per
  vector: H_n = H_a (x) H_b is applied as the two dense matrix products H_a T H_b on the a x b view of the vector,
  with the materialised factors and numpy's fp64 matrix product as the step.
* ``epilogue_none``      - Section 3.2: an m x n spinner is the first m rows of
  the n x n one; ``scale`` is the caller's extra factor (sqrt(n) in Lemma 1,
  sqrt(n/m) for a norm-preserving embedding).
* ``epilogue_cossin``    - Section 5 (kernel approximation): features
  ``s(Ax) = exp(-i A x / sigma)`` scaled by ``1/sqrt(d')``; written in its real
  form ``(1/sqrt(m)) [cos w ; sin w]`` whose dot product is the Hermitian
  product of the complex features.
* ``epilogue_hash``      - Section 4, Theorem 4 and its proof: the hash of a
  vector is the signed canonical direction closest to its projection, i.e.
  ``argmax_i |y_i|`` together with the sign of that coordinate.
* ``layer_forward`` / ``layer_backward`` - the adaptive setting (Section 1, Section 3.2 "adaptive"
  diagonals, Section 5 neural networks): the HD3HD2HD1 block as a layer with learned diagonals.
  The backward pass is the transpose of the layer's Jacobian written out with dense matrices:
  ``dx = scale * D1 H D2 H D3 H dy`` (H is symmetric) and, for each diagonal, the sum over the batch of
  (signal arriving at the diagonal from the output side) times (activation entering it from the input side).
* ``struct_matrix`` / ``struct_apply`` - the members G_struct D2 H D1 of the family (Lemma 1 and the remark after
  it; Theorem 3; Section 5 experiments): G_struct a Gaussian circulant, skew-circulant, Toeplitz or Hankel matrix,
  written out densely from its generating vector.
* ``struct_rows`` / ``struct_apply_rows`` - the same members for n too large for the dense matrix: selected rows of
  G_struct written out from the generating vector, and the matching outputs.
* ``apply_blocks``       - Section 3.2: independently constructed m x n blocks stacked vertically.
* ``sketch`` / ``sketched_gram`` - the Newton-sketch use of the Supplement ("Additional experiments"):
  an m x n sketching matrix S (the first m rows of a spinner, scaled) applied to the columns of a
  weighted data matrix diag(w) A, and the d x d matrix (S diag(w) A)^T (S diag(w) A) that replaces the Hessian.
* ``epilogue_signbits`` / ``angular_estimate`` - Section 5 (angular kernel):
  the pointwise sign of the projection, and the kernel estimate
  ``1 - d_H / d'`` from the Hamming distance of two such sign vectors.

Readings where the paper is silent: Sylvester row order; bucket ``i`` for
``+e_i`` and ``i + n`` for ``-e_i``; lowest index wins exact ties; a zero
coordinate counts as positive (hash and sign bits alike); features are
concatenated (cos block, then sin block), not interleaved.

Parity status: every function here is pinned by the CPU tests (``tests/
test_oracle_*.py``) against closed forms, library constructions of the Hadamard
matrix, invariants and brute force; nothing is "parity unpinned".
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "spinner_oracle.c")
_LIB = os.path.join(_HERE, "liboracle_spinner.so")
_lib = None

# n above which the dense n x n Hadamard matrix is not materialised and the
# two explicit Kronecker factors are used instead.
DENSE_MAX_N = 1 << 14


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP over vectors). Returns the .so path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c11", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.oracle_hadamard_sign.restype = ctypes.c_int
        lib.oracle_hadamard_sign.argtypes = [ctypes.c_uint64, ctypes.c_uint64]
        lib.oracle_hadamard_dense.restype = None
        lib.oracle_hadamard_dense.argtypes = [ctypes.c_int, ctypes.c_void_p]
        lib.oracle_max_threads.restype = ctypes.c_int
        lib.oracle_hadamard_apply.restype = ctypes.c_int
        lib.oracle_hadamard_apply.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_long,
                                              ctypes.c_int, ctypes.c_void_p]
        lib.oracle_spinner.restype = ctypes.c_int
        lib.oracle_spinner.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_long,
                                       ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                       ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
        _lib = lib
    return _lib


def max_threads() -> int:
    return int(_load().oracle_max_threads())


def _is_pow2(v: int) -> bool:
    return v > 0 and (v & (v - 1)) == 0


def default_kron_a(n: int) -> int:
    """0 (dense H_n) up to DENSE_MAX_N, else the larger factor of a balanced split."""
    if n <= DENSE_MAX_N:
        return 0
    log2n = n.bit_length() - 1
    return 1 << ((log2n + 1) // 2)


def hadamard_sign(i: int, j: int) -> int:
    return int(_load().oracle_hadamard_sign(i, j))


def hadamard_dense(n: int) -> np.ndarray:
    """Unnormalised Sylvester Hadamard matrix, int8 [n][n]."""
    assert _is_pow2(n)
    H = np.empty((n, n), dtype=np.int8)
    _load().oracle_hadamard_dense(n, H.ctypes.data)
    return H


def hadamard_apply(t: np.ndarray, kron_a: int = 0) -> np.ndarray:
    """(H_n / sqrt(n)) t for each row of fp64 ``t`` [batch][n] (dense or Kronecker route)."""
    t = np.ascontiguousarray(t, dtype=np.float64)
    squeeze = t.ndim == 1
    if squeeze:
        t = t[None, :]
    batch, n = t.shape
    out = np.empty_like(t)
    rc = _load().oracle_hadamard_apply(t.ctypes.data, n, batch, kron_a, out.ctypes.data)
    if rc != 0:
        raise ValueError("oracle_hadamard_apply: bad arguments")
    return out[0] if squeeze else out


def spinner(x: np.ndarray, d1: np.ndarray, d2: np.ndarray, d3: np.ndarray,
            kron_a: int | None = None, nthreads: int = 0) -> np.ndarray:
    """y = H D3 H D2 H D1 x in fp64 for each row of fp32 ``x`` [batch][n]."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    squeeze = x.ndim == 1
    if squeeze:
        x = x[None, :]
    batch, n = x.shape
    ds = [np.ascontiguousarray(d, dtype=np.float32) for d in (d1, d2, d3)]
    for d in ds:
        if d.shape != (n,):
            raise ValueError("diagonal must have shape (n,)")
    if kron_a is None:
        kron_a = default_kron_a(n)
    y = np.empty((batch, n), dtype=np.float64)
    rc = _load().oracle_spinner(x.ctypes.data, n, batch, ds[0].ctypes.data, ds[1].ctypes.data,
                                ds[2].ctypes.data, kron_a, nthreads, y.ctypes.data)
    if rc != 0:
        raise ValueError("oracle_spinner: bad arguments or out of memory")
    return y[0] if squeeze else y


def spinner_by_products(x: np.ndarray, d1: np.ndarray, d2: np.ndarray, d3: np.ndarray) -> np.ndarray:
    """y = H D3 H D2 H D1 x in fp64 for each row of fp32 ``x`` [batch][n], n >= 4, for the largest n.

    Section 1 / Section 3, with the Sylvester matrix written as H_n = H_a (x) H_b (a b = n): entry (i, j) of H_n is
    H_a[ia][ja] H_b[ib][jb] for i = ia b + ib, j = ja b + jb, so H_n t is the matrix H_a T H_b for the row-major a x b
    view T of t (both factors are symmetric).  The factors are materialised and multiplied with numpy's fp64 matrix
    product: 2 n (a + b) multiply-adds per round instead of n^2.
    """
    x = np.ascontiguousarray(x, dtype=np.float32)
    squeeze = x.ndim == 1
    if squeeze:
        x = x[None, :]
    batch, n = x.shape
    assert _is_pow2(n) and n >= 4
    log2n = n.bit_length() - 1
    a = 1 << ((log2n + 1) // 2)
    b = n // a
    Ha = hadamard_dense(a).astype(np.float64)
    Hb = hadamard_dense(b).astype(np.float64)
    t = x.astype(np.float64)
    for d in (d1, d2, d3):
        d = np.asarray(d, dtype=np.float32)
        if d.shape != (n,):
            raise ValueError("diagonal must have shape (n,)")
        t = t * d.astype(np.float64)[None, :]
        t = (Ha @ t.reshape(batch, a, b) @ Hb).reshape(batch, n) / np.sqrt(float(n))
    return t[0] if squeeze else t


def epilogue_none(y: np.ndarray, m: int, scale: float) -> np.ndarray:
    """First m coordinates of ``scale * y`` (Section 3.2: first m rows of the spinner)."""
    return float(scale) * y[..., :m]


def epilogue_cossin(y: np.ndarray, m: int, scale: float) -> np.ndarray:
    """(1/sqrt(m)) [cos(w_0..w_{m-1}), sin(w_0..w_{m-1})] with w = scale * y (Section 5)."""
    w = float(scale) * y[..., :m]
    return np.concatenate([np.cos(w), np.sin(w)], axis=-1) / np.sqrt(float(m))


def epilogue_hash(y: np.ndarray) -> np.ndarray:
    """Cross-polytope bucket per row: i* = argmax |y_i| (lowest index on ties),
    bucket = i* if y_{i*} >= 0 else i* + n (Section 4, Theorem 4)."""
    n = y.shape[-1]
    istar = np.argmax(np.abs(y), axis=-1)            # numpy returns the first maximum
    ystar = np.take_along_axis(y, istar[..., None], axis=-1)[..., 0]
    return (istar + n * (ystar < 0)).astype(np.int32)


def epilogue_signbits(y: np.ndarray, m: int) -> np.ndarray:
    """uint8 [..., m]: 1 where the coordinate is negative, 0 otherwise (zero counts as
    positive): s = sign applied pointwise to the first m coordinates (Section 5)."""
    return (y[..., :m] < 0).astype(np.uint8)


def angular_estimate(bits_a: np.ndarray, bits_b: np.ndarray) -> np.ndarray:
    """[Ba][Bb] estimates 1 - d_H(s(Ax_i), s(Ax_j)) / d' of the angular kernel from two
    sets of sign vectors (Section 5)."""
    bits_a = np.asarray(bits_a, dtype=np.uint8)
    bits_b = np.asarray(bits_b, dtype=np.uint8)
    m = bits_a.shape[-1]
    dh = (bits_a[:, None, :] != bits_b[None, :, :]).sum(axis=-1)
    return 1.0 - dh.astype(np.float64) / float(m)


def layer_forward(x, d1, d2, d3, scale: float = 1.0, nthreads: int = 0):
    """y = scale * H D3 H D2 H D1 x together with the activations that enter D2 and D3:
    b1 = H D1 x and b2 = H D2 b1 (all fp64, [batch][n])."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    d1, d2, d3 = (np.asarray(d, dtype=np.float64) for d in (d1, d2, d3))
    ka = default_kron_a(x.shape[-1])              # dense H_n up to DENSE_MAX_N, its two Kronecker factors above
    b1 = hadamard_apply(x * d1, ka)
    b2 = hadamard_apply(b1 * d2, ka)
    y = float(scale) * hadamard_apply(b2 * d3, ka)
    return y, b1, b2


def layer_backward(x, d1, d2, d3, dy, scale: float = 1.0):
    """Gradients of L with respect to x and to the three diagonals, given dy = dL/dy for
    y = scale * H D3 H D2 H D1 x.  Returns (dx [batch][n], dd [3][n]); dd sums over the batch."""
    d1, d2, d3 = (np.asarray(d, dtype=np.float64) for d in (d1, d2, d3))
    x = np.ascontiguousarray(x, dtype=np.float64)
    dy = np.ascontiguousarray(dy, dtype=np.float64)
    _, b1, b2 = layer_forward(x, d1, d2, d3, scale)
    ka = default_kron_a(x.shape[-1])
    g3 = float(scale) * hadamard_apply(dy, ka)    # dL/d(D3 b2): H^T = H
    dd3 = (g3 * b2).sum(axis=0)
    g2 = hadamard_apply(g3 * d3, ka)              # dL/d(D2 b1)
    dd2 = (g2 * b1).sum(axis=0)
    g1 = hadamard_apply(g2 * d2, ka)              # dL/d(D1 x)
    dd1 = (g1 * x).sum(axis=0)
    dx = g1 * d1
    return dx, np.stack([dd1, dd2, dd3])


def sketch(A, w, d1, d2, d3, m: int, scale: float, nthreads: int = 0) -> np.ndarray:
    """B = S diag(w) A, fp64 [m][d], for A fp32 [n][d], row weights w fp32 [n] (None: all ones) and
    S = scale * (first m rows of H D3 H D2 H D1).  The spinner acts on each column of diag(w) A."""
    A = np.asarray(A, dtype=np.float64)
    if w is not None:
        A = A * np.asarray(w, dtype=np.float64)[:, None]                           # diag(w) A, no intermediate rounding
    cols = np.ascontiguousarray(A.T)                                               # [d][n]: one vector per column
    ka = default_kron_a(cols.shape[1])
    d1, d2, d3 = (np.asarray(d, dtype=np.float64) for d in (d1, d2, d3))
    t = hadamard_apply(cols * d1, ka)                                              # H D1 (diag(w) a) for every column a
    t = hadamard_apply(t * d2, ka)
    y = hadamard_apply(t * d3, ka)
    return float(scale) * np.ascontiguousarray(y[:, :m].T)


def sketched_gram(B) -> np.ndarray:
    """(S diag(w) A)^T (S diag(w) A), fp64 [d][d]."""
    B = np.asarray(B, dtype=np.float64)
    return B.T @ B


def apply(x, d1, d2, d3, m: int, epilogue: str, scale: float,
          kron_a: int | None = None, nthreads: int = 0) -> np.ndarray:
    """Whole path for one diagonal triple: spinner then the named epilogue, fp64."""
    y = spinner(x, d1, d2, d3, kron_a=kron_a, nthreads=nthreads)
    if epilogue == "none":
        return epilogue_none(y, m, scale)
    if epilogue == "cossin":
        return epilogue_cossin(y, m, scale)
    if epilogue == "signbits":
        return epilogue_signbits(y, m)
    raise ValueError("unknown epilogue %r" % (epilogue,))


STRUCT_KINDS = ("circulant", "skew_circulant", "toeplitz", "hankel")


def struct_matrix(kind: str, params, n: int) -> np.ndarray:
    """Dense n x n structured matrix from its generating vector (fp64).

    circulant       params g[n]:     row 0 is g, each next row is the previous one shifted right cyclically
                                     (Section 3, notation): G[i][j] = g[(j - i) mod n]
    skew_circulant  params g[n]:     the same, but an entry that wraps around changes sign
    toeplitz        params t[2n-1]:  constant along diagonals, G[i][j] = t[j - i + n - 1]
    hankel          params h[2n-1]:  constant along anti-diagonals, G[i][j] = h[i + j]"""
    p = np.asarray(params, dtype=np.float64)
    i, j = np.meshgrid(np.arange(n), np.arange(n), indexing="ij")
    if kind == "circulant":
        assert p.shape == (n,)
        return p[(j - i) % n]
    if kind == "skew_circulant":
        assert p.shape == (n,)
        return np.where(j >= i, 1.0, -1.0) * p[(j - i) % n]
    if kind == "toeplitz":
        assert p.shape == (2 * n - 1,)
        return p[j - i + n - 1]
    if kind == "hankel":
        assert p.shape == (2 * n - 1,)
        return p[i + j]
    raise ValueError("unknown structured matrix %r" % (kind,))


def struct_apply(x, kind: str, params, d1, d2, m: int, scale: float) -> np.ndarray:
    """scale * (first m rows of G_struct D2 H D1 x), fp64 [batch][m]."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    n = x.shape[-1]
    t = hadamard_apply(x * np.asarray(d1, dtype=np.float64)) * np.asarray(d2, dtype=np.float64)
    G = struct_matrix(kind, params, n)
    return float(scale) * (t @ G[:m].T)


def struct_rows(kind: str, params, n: int, rows) -> np.ndarray:
    """The listed rows of the n x n structured matrix, fp64 [len(rows)][n], written out from the generating vector by
    the definitions in ``struct_matrix`` (for n where the whole matrix would not fit in memory)."""
    p = np.asarray(params, dtype=np.float64)
    i = np.asarray(rows, dtype=np.int64)[:, None]
    j = np.arange(n, dtype=np.int64)[None, :]
    if kind == "circulant":
        assert p.shape == (n,)
        return p[(j - i) % n]
    if kind == "skew_circulant":
        assert p.shape == (n,)
        return np.where(j >= i, 1.0, -1.0) * p[(j - i) % n]
    if kind == "toeplitz":
        assert p.shape == (2 * n - 1,)
        return p[j - i + n - 1]
    if kind == "hankel":
        assert p.shape == (2 * n - 1,)
        return p[i + j]
    raise ValueError("unknown structured matrix %r" % (kind,))


def struct_apply_rows(x, kind: str, params, d1, d2, rows, scale: float) -> np.ndarray:
    """scale * (the listed rows of G_struct D2 H D1 x), fp64 [batch][len(rows)]; H through its two Kronecker factors
    above DENSE_MAX_N."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    n = x.shape[-1]
    t = hadamard_apply(x * np.asarray(d1, dtype=np.float64), default_kron_a(n)) * np.asarray(d2, dtype=np.float64)
    return float(scale) * (t @ struct_rows(kind, params, n, rows).T)


def apply_blocks(x, diag_sets: np.ndarray, m: int, epilogue: str, scale: float, nthreads: int = 0) -> np.ndarray:
    """Section 3.2: L independently constructed m x n blocks stacked vertically (k = L m rows).  Returns the
    k coordinates, block after block ("none"), or (1/sqrt(k)) [cos of all k ; sin of all k] ("cossin")."""
    diag_sets = np.ascontiguousarray(diag_sets, dtype=np.float32)
    ys = [spinner(x, t[0], t[1], t[2], nthreads=nthreads)[:, :m] for t in diag_sets]
    w = float(scale) * np.concatenate(ys, axis=-1)
    if epilogue == "none":
        return w
    if epilogue == "cossin":
        return np.concatenate([np.cos(w), np.sin(w)], axis=-1) / np.sqrt(float(w.shape[-1]))
    raise ValueError("unknown epilogue %r" % (epilogue,))


def hash(x, diag_sets: np.ndarray, nthreads: int = 0, return_y: bool = False):
    """Buckets for L independently drawn triples (Section 3.2: independently
    constructed blocks).  diag_sets: fp32 [L][3][n].  Returns int32 [batch][L]
    (and the fp64 projections [L][batch][n] when ``return_y``)."""
    diag_sets = np.ascontiguousarray(diag_sets, dtype=np.float32)
    L = diag_sets.shape[0]
    cols, ys = [], []
    for l in range(L):
        y = spinner(x, diag_sets[l, 0], diag_sets[l, 1], diag_sets[l, 2], nthreads=nthreads)
        cols.append(epilogue_hash(y))
        if return_y:
            ys.append(y)
    idx = np.stack(cols, axis=-1).astype(np.int32)
    return (idx, np.stack(ys, axis=0)) if return_y else idx
