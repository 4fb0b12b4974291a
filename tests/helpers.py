"""Shared comparison rules for GPU-vs-oracle parity tests."""
import numpy as np

REL_L2_TOL = 1e-5          # per output vector, fp32 path vs fp64 oracle
HASH_BAND = 1e-5           # relative band inside which near-ties may resolve either way


def rel_l2_per_vector(got: np.ndarray, want: np.ndarray) -> np.ndarray:
    got = got.astype(np.float64)
    num = np.linalg.norm(got - want, axis=-1)
    den = np.linalg.norm(want, axis=-1)
    return num / np.where(den == 0, 1.0, den)


def rel_l2_first_m(got: np.ndarray, want: np.ndarray, x: np.ndarray, n: int, m: int, scale: float) -> np.ndarray:
    """Error of a first-m-rows output per vector.  With m > 8 coordinates kept this is the plain rule
    (error norm over the norm of the kept part).  A handful of kept coordinates can cancel to next to
    nothing, and fp32 cannot hold 1e-5 of that: for m <= 8 the error is measured against the kept part's
    norm or its expected size sqrt(m / n) * scale * |x| (the spinner is an isometry), whichever is larger."""
    if m > 8:
        return rel_l2_per_vector(got, want)
    num = np.linalg.norm(got.astype(np.float64) - want, axis=-1)
    ref = np.maximum(np.linalg.norm(want, axis=-1),
                     np.sqrt(m / n) * scale * np.linalg.norm(x.astype(np.float64), axis=-1))
    return num / np.where(ref == 0, 1.0, ref)


def check_hash_against_projection(idx_gpu: np.ndarray, y: np.ndarray, band: float = HASH_BAND):
    """idx_gpu int32 [batch][L]; y fp64 [L][batch][n] (the oracle's projections).

    Exact agreement with the oracle bucket is required wherever the oracle's two
    largest |y_i| differ by more than `band` relative; inside the band any index
    whose |y_i| is within the band of the maximum is accepted, with its own sign.
    Returns (number of exact matches, number accepted through the band)."""
    L, batch, n = y.shape
    exact = banded = 0
    for l in range(L):
        ay = np.abs(y[l])
        istar = np.argmax(ay, axis=1)
        top = ay[np.arange(batch), istar]
        want = istar + n * (y[l][np.arange(batch), istar] < 0)
        got = idx_gpu[:, l].astype(np.int64)
        same = got == want
        exact += int(same.sum())
        for v in np.nonzero(~same)[0]:
            g = int(got[v])
            assert 0 <= g < 2 * n, (v, l, g)
            i = g % n
            # the GPU's choice must be a near-tie of the maximum and carry the right sign
            assert ay[v, i] >= top[v] * (1.0 - band), (v, l, g, int(want[v]), ay[v, i], top[v])
            assert (g >= n) == (y[l][v, i] < 0), (v, l, g)
            banded += 1
    return exact, banded


SIGN_BAND = 1e-5           # coordinates with |y_i| <= SIGN_BAND * max|y| may take either sign bit


def unpack_sign_codes(codes: np.ndarray, m: int) -> np.ndarray:
    """codes: integer array [batch][m/64] of 64-bit words -> uint8 [batch][m], bit of coordinate e taken from
    bit (e >> 2) & 63 of word ((e >> 8) << 2) | (e & 3) (the layout documented in include/spinner.h)."""
    words = codes.view(np.uint64)
    e = np.arange(m)
    w = ((e >> 8) << 2) | (e & 3)
    b = ((e >> 2) & 63).astype(np.uint64)
    return ((words[:, w] >> b) & np.uint64(1)).astype(np.uint8)


def check_sign_bits(bits_gpu: np.ndarray, y: np.ndarray, m: int, band: float = SIGN_BAND) -> int:
    """bits_gpu uint8 [batch][m] against the oracle's fp64 projection y [batch][n]: exact wherever |y_i| exceeds
    band * max|y| of its vector (an fp32 path cannot resolve the sign of a coordinate that is zero to rounding).
    Returns the number of coordinates that fell inside the band."""
    want = (y[:, :m] < 0).astype(np.uint8)
    clear = np.abs(y[:, :m]) > band * np.abs(y).max(axis=1, keepdims=True)
    bad = (bits_gpu != want) & clear
    assert not bad.any(), np.argwhere(bad)[:5]
    return int((~clear).sum())
