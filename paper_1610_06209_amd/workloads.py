"""Seeded synthetic inputs for the structured-spinner path.

This module holds input recipes only - shapes, value distributions and seeds of
the five benchmark configurations and of the plain-spinner size sweep.  It
contains none of the method's arithmetic (no Hadamard transform, no diagonal
product, no epilogue), so both the CPU oracle's tests and the HIP path's tests
can draw their inputs from it without sharing any computation.

The data stand in for the paper's workloads (Section 5: cross-polytope LSH
collision experiment; Gaussian-kernel random features on G50C / USPST; the
dimensionality-reduction use of Section 1), none of whose datasets are
available here.  Random +-1 diagonals follow Section 3 (D has independent
uniform +-1 entries on its diagonal); Gaussian third diagonals follow Lemma 1.

Generation happens on the CPU with numpy (small cases) or directly on the GPU
with torch's seeded generator (full-size cases, so that no multi-GiB host
buffer crosses PCIe).  A parity test always copies the rows it checks back
from the buffer the GPU consumed, so the two never need to agree bit for bit.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np

BASE_SEED = 0x5EED161006209000


@dataclass(frozen=True)
class Workload:
    name: str
    kind: str          # "apply" or "hash"
    n: int
    batch: int
    m: int             # rows kept (apply); n for hash
    epilogue: str      # "none" | "cossin" | "hash"
    scale: float       # caller's extra factor on top of the normalised spinner
    L: int             # number of independent (D1,D2,D3) triples (hash), else 1
    dist: str          # input distribution recipe
    seed: int
    oracle_rows: int   # how many rows the O(n^2) oracle checks at full size


CONFIGS = {
    # Plain spinner, full output.
    "cfg1_plain_n256": Workload("cfg1_plain_n256", "apply", 256, 1024, 256, "none", 1.0, 1,
                                "normal", BASE_SEED + 1, 1024),
    # Cross-polytope LSH, 16 independent triples on unit vectors.
    "cfg2_lsh_n1024": Workload("cfg2_lsh_n1024", "hash", 1024, 65536, 1024, "hash", 1.0, 16,
                               "unit_normal", BASE_SEED + 2, 256),
    # Gaussian-kernel random features, sigma_k = 1 -> scale = sqrt(n).
    "cfg3_rff_n4096": Workload("cfg3_rff_n4096", "apply", 4096, 131072, 4096, "cossin", 64.0, 1,
                               "mixture64", BASE_SEED + 3, 128),
    # JL reduction to m = 1024 rows, scale sqrt(n/m).
    "cfg4_jl_n16384": Workload("cfg4_jl_n16384", "apply", 16384, 32768, 1024, "none", 4.0, 1,
                               "normal_heavy", BASE_SEED + 4, 32),
    # Large-n multi-pass spinner.
    "cfg5_large_n2p20": Workload("cfg5_large_n2p20", "apply", 1 << 20, 256, 1 << 20, "none", 1.0, 1,
                                 "normal", BASE_SEED + 5, 4),
}
CONFIG_ORDER = list(CONFIGS)

# Rows beyond the five benchmark configurations (measured beside them, same recipe style).
NEXT = {
    # Angular-kernel sign codes (Section 5) on the shape of the random-feature configuration.
    "next_angular_n4096": Workload("next_angular_n4096", "codes", 4096, 131072, 4096, "signbits", 1.0, 1,
                                   "mixture64", BASE_SEED + 6, 128),
    # k = 4 n random features from four stacked independent blocks (Section 3.2, Section 5), on the mixture of cfg3.
    "next_blocks_n4096_L4": Workload("next_blocks_n4096_L4", "blocks", 4096, 32768, 4096, "cossin", 64.0, 4,
                                     "mixture64", BASE_SEED + 7, 64),
}


def sweep_workload(log2n: int, total_elems_log2: int = 28) -> Workload:
    """Plain spinner, full output, batch = 2^total / n (the size sweep of the metric)."""
    n = 1 << log2n
    batch = max(1, (1 << total_elems_log2) // n)
    return Workload("sweep_plain_n2p%d" % log2n, "apply", n, batch, n, "none", 1.0, 1,
                    "normal", BASE_SEED + 100 + log2n, 4)


# ----------------------------------------------------------------------------
# diagonals
# ----------------------------------------------------------------------------
def rademacher_diagonals(n: int, count: int, seed: int) -> np.ndarray:
    """fp32 [count][n] of independent +-1 entries."""
    rng = np.random.Generator(np.random.PCG64(seed ^ 0xD1A6))
    bits = rng.integers(0, 2, size=(count, n), dtype=np.int8)
    return (1.0 - 2.0 * bits).astype(np.float32)


def gaussian_diagonal(n: int, seed: int) -> np.ndarray:
    """fp32 [n] of N(0,1) entries (the D_{g_1..g_n} of Lemma 1 / learned diagonals)."""
    rng = np.random.Generator(np.random.PCG64(seed ^ 0x6A55))
    return rng.standard_normal(n).astype(np.float32)


def diag_sets(w: Workload) -> np.ndarray:
    """fp32 [L][3][n] Rademacher triples for a workload (L = 1 for apply)."""
    return rademacher_diagonals(w.n, 3 * w.L, w.seed).reshape(w.L, 3, w.n)


# ----------------------------------------------------------------------------
# data
# ----------------------------------------------------------------------------
def heavy_coordinates(n: int, seed: int) -> np.ndarray:
    """The fixed set of floor(0.05 n) coordinates that are scaled x10 in every vector."""
    rng = np.random.Generator(np.random.PCG64(seed ^ 0x4EA7))
    return np.sort(rng.choice(n, size=int(0.05 * n), replace=False))


def make_x_numpy(w: Workload, batch: int | None = None) -> np.ndarray:
    """fp32 [batch][n] on the host, numpy generator."""
    b = w.batch if batch is None else batch
    rng = np.random.Generator(np.random.PCG64(w.seed))
    if w.dist == "normal":
        x = rng.standard_normal((b, w.n), dtype=np.float32)
    elif w.dist == "unit_normal":
        x = rng.standard_normal((b, w.n), dtype=np.float32)
        x /= np.linalg.norm(x.astype(np.float64), axis=1, keepdims=True).astype(np.float32)
    elif w.dist == "mixture64":
        centres = rng.standard_normal((64, w.n), dtype=np.float32)
        comp = rng.integers(0, 64, size=b)
        x = centres[comp] + np.float32(0.5) * rng.standard_normal((b, w.n), dtype=np.float32)
    elif w.dist == "normal_heavy":
        x = rng.standard_normal((b, w.n), dtype=np.float32)
        x[:, heavy_coordinates(w.n, w.seed)] *= np.float32(10.0)
    else:
        raise ValueError(w.dist)
    return np.ascontiguousarray(x, dtype=np.float32)


def make_x_torch(w: Workload, device, batch: int | None = None):
    """fp32 [batch][n] generated directly on ``device`` with torch's seeded generator."""
    import torch

    b = w.batch if batch is None else batch
    g = torch.Generator(device=device)
    g.manual_seed(w.seed & 0x7FFFFFFFFFFFFFFF)
    if w.dist == "normal":
        x = torch.randn((b, w.n), generator=g, device=device, dtype=torch.float32)
    elif w.dist == "unit_normal":
        x = torch.randn((b, w.n), generator=g, device=device, dtype=torch.float32)
        x /= torch.linalg.vector_norm(x, dim=1, keepdim=True)
    elif w.dist == "mixture64":
        centres = torch.randn((64, w.n), generator=g, device=device, dtype=torch.float32)
        comp = torch.randint(0, 64, (b,), generator=g, device=device)
        x = torch.randn((b, w.n), generator=g, device=device, dtype=torch.float32)
        x *= 0.5
        # add the chosen centre in chunks so no second full-size temporary is made
        step = 8192
        for s in range(0, b, step):
            x[s:s + step] += centres[comp[s:s + step]]
    elif w.dist == "normal_heavy":
        x = torch.randn((b, w.n), generator=g, device=device, dtype=torch.float32)
        idx = torch.from_numpy(heavy_coordinates(w.n, w.seed)).to(device)
        x[:, idx] *= 10.0
    else:
        raise ValueError(w.dist)
    return x.contiguous()


def newton_sketch_problem(n: int, d: int, seed: int):
    """Data of the Supplement's logistic-regression experiment: rows a_i ~ N(0, Sigma) with
    Sigma_jk = 0.99^|j-k| (generated as a stationary AR(1) sequence along each row), and the row weights
    w_i = sqrt(p_i (1 - p_i)), p_i = 1 / (1 + exp(-a_i^T x)), at a seeded iterate x.  Returns (A fp32 [n][d], w fp32 [n])."""
    rng = np.random.Generator(np.random.PCG64(seed ^ 0x4E5754))
    rho = 0.99
    eps = rng.standard_normal((n, d), dtype=np.float32)
    A = np.empty((n, d), dtype=np.float32)
    A[:, 0] = eps[:, 0]
    c = np.float32(math.sqrt(1.0 - rho * rho))
    for j in range(1, d):
        A[:, j] = np.float32(rho) * A[:, j - 1] + c * eps[:, j]
    x = (rng.standard_normal(d) / math.sqrt(d)).astype(np.float32)
    p = 1.0 / (1.0 + np.exp(-(A.astype(np.float64) @ x.astype(np.float64))))
    w = np.sqrt(p * (1.0 - p)).astype(np.float32)
    return A, w


def sample_rows(batch: int, count: int, seed: int) -> np.ndarray:
    """Row indices a full-size parity check looks at: first, last and a seeded draw."""
    count = min(count, batch)
    if count >= batch:
        return np.arange(batch)
    rng = np.random.Generator(np.random.PCG64(seed ^ 0x5A3B1E))
    mid = rng.choice(np.arange(1, batch - 1), size=count - 2, replace=False)
    return np.sort(np.concatenate([[0, batch - 1], mid])).astype(np.int64)


def fused_max_n(epilogue: str) -> int:
    """Largest n one fused kernel handles: 2^16 for the plain / first-m-rows epilogue (fp32
    butterflies), 2^14 for the fp64 feature map and for hashing."""
    return (1 << 16) if epilogue == "none" else (1 << 14)


def algorithmic_bytes_per_vector(w: Workload) -> int:
    """Bytes the method must move per vector at any n: x once, the epilogue's output once
    (diagonals are shared by the batch and amortise to zero)."""
    n = w.n
    if w.kind == "hash":
        return 4 * n + 4 * w.L
    if w.kind == "codes":                       # one bit per kept coordinate leaves the chip
        return 4 * n + w.m // 8
    out = 8 * w.m if w.epilogue == "cossin" else 4 * w.m
    if w.kind == "blocks":                      # x once, L blocks of output
        return 4 * n + out * w.L
    return 4 * n + out


def schedule_bytes_per_vector(w: Workload) -> int:
    """Bytes the kernels themselves read and write per vector, memory-side cache and HBM together.  The same as
    the algorithmic bytes while one fused kernel serves n; above that the four-pass schedule moves the vector four
    times (three of the trips are meant to stay in the memory-side cache), and sign codes take a fifth read."""
    n = w.n
    if w.kind in ("hash", "blocks") or n <= fused_max_n("none" if w.kind == "codes" else w.epilogue):
        return algorithmic_bytes_per_vector(w)
    if w.kind == "codes":
        return 4 * 8 * n + 4 * n + w.m // 8
    out = 8 * w.m if w.epilogue == "cossin" else 4 * w.m
    return 3 * 8 * n + 4 * n + out


PRUNE_BITS = 4      # the kernels drop the four highest index bits of the last round when m <= n / 16


def adds_per_vector(w: Workload) -> int:
    """fp32 additions of the butterfly network per vector (3 rounds, per triple).  When at most n/16 leading
    coordinates are kept, the last round only forms the sums on its four highest index bits
    (n/2 + n/4 + n/8 + n/16 additions) and log2(n) - 4 full stages on the n/16 values that are left."""
    N = int(math.log2(w.n))
    full = N * w.n
    if w.kind == "apply" and w.epilogue == "none" and 8 <= N <= 16 and w.m <= (w.n >> PRUNE_BITS):
        last = (w.n - (w.n >> PRUNE_BITS)) + (N - PRUNE_BITS) * (w.n >> PRUNE_BITS)
        return (2 * full + last) * w.L
    return 3 * full * w.L
