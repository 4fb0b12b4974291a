"""Thin ctypes binding of ``libspinner.so`` (the C ABI in ``include/spinner.h``).

Argument marshalling only: every step of the path runs in the library's HIP
kernels.  PyTorch is used for device memory and streams, nothing else.  There
is no fallback: if the library has not been built, importing this module
raises.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
# SPINNER_LIB lets a tuning run point the binding at another build of the same library
LIB_PATH = os.environ.get("SPINNER_LIB") or os.path.join(_HERE, "libspinner.so")

SPINNER_OK = 0
SPINNER_ERR_BAD_N = -1
SPINNER_ERR_BAD_M = -2
SPINNER_ERR_NULL_PTR = -3
SPINNER_ERR_BAD_EPILOGUE = -4
SPINNER_ERR_BAD_BATCH = -5
SPINNER_ERR_WORKSPACE = -6
SPINNER_ERR_HIP = -7
SPINNER_ERR_BAD_L = -8
SPINNER_ERR_ALIGNMENT = -9
SPINNER_ERR_UNSUPPORTED = -10

SPINNER_EPI_NONE = 0
SPINNER_EPI_COSSIN = 1
EPILOGUES = {"none": SPINNER_EPI_NONE, "cossin": SPINNER_EPI_COSSIN}

EXPORTS = ["spinner_apply", "spinner_hash", "spinner_workspace_bytes", "spinner_strerror",
           "spinner_version", "spinner_stream_copy", "spinner_signs_bytes", "spinner_pack_signs",
           "spinner_apply_signs", "spinner_hash_signs"]

if not os.path.exists(LIB_PATH):
    raise ImportError(
        "libspinner.so is not built: run `python -m paper_1610_06209_amd.build` "
        "(or __graft_entry__.build()); there is no fallback path")

lib = ctypes.CDLL(LIB_PATH)
_vp = ctypes.c_void_p
lib.spinner_apply.restype = ctypes.c_int
lib.spinner_apply.argtypes = [_vp, ctypes.c_int, ctypes.c_long, _vp, _vp, _vp, ctypes.c_int, ctypes.c_int,
                              ctypes.c_float, _vp, _vp, _vp]
lib.spinner_hash.restype = ctypes.c_int
lib.spinner_hash.argtypes = [_vp, ctypes.c_int, ctypes.c_long, ctypes.c_int, _vp, _vp, _vp]
lib.spinner_workspace_bytes.restype = ctypes.c_size_t
lib.spinner_workspace_bytes.argtypes = [ctypes.c_int, ctypes.c_long, ctypes.c_int, ctypes.c_int]
lib.spinner_strerror.restype = ctypes.c_char_p
lib.spinner_strerror.argtypes = [ctypes.c_int]
lib.spinner_version.restype = ctypes.c_int
lib.spinner_version.argtypes = []
lib.spinner_signs_bytes.restype = ctypes.c_size_t
lib.spinner_signs_bytes.argtypes = [ctypes.c_int, ctypes.c_int]
lib.spinner_pack_signs.restype = ctypes.c_int
lib.spinner_pack_signs.argtypes = [_vp, ctypes.c_int, ctypes.c_int, _vp, _vp]
lib.spinner_apply_signs.restype = ctypes.c_int
lib.spinner_apply_signs.argtypes = [_vp, ctypes.c_int, ctypes.c_long, _vp, ctypes.c_int, ctypes.c_int,
                                    ctypes.c_float, _vp, _vp, _vp]
lib.spinner_hash_signs.restype = ctypes.c_int
lib.spinner_hash_signs.argtypes = [_vp, ctypes.c_int, ctypes.c_long, ctypes.c_int, _vp, _vp, _vp]
lib.spinner_stream_copy.restype = ctypes.c_int
lib.spinner_stream_copy.argtypes = [_vp, _vp, ctypes.c_size_t, _vp]


class SpinnerError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__("spinner: %s (status %d)" % (spinner_strerror(status), status))


def spinner_strerror(status: int) -> str:
    return lib.spinner_strerror(int(status)).decode()


def spinner_version() -> int:
    return int(lib.spinner_version())


def spinner_workspace_bytes(n: int, batch: int, m: int, epilogue) -> int:
    return int(lib.spinner_workspace_bytes(int(n), int(batch), int(m), _epi(epilogue)))


def _epi(e) -> int:
    return EPILOGUES[e] if isinstance(e, str) else int(e)


def _stream_handle(stream):
    import torch

    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _check_tensor(t, name, dtype):
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise ValueError("%s must be a contiguous %s CUDA tensor" % (name, dtype))


def spinner_apply(x, d1, d2, d3, m=None, epilogue="none", scale=1.0, out=None, workspace=None, stream=None):
    """out = epilogue(scale * first m coordinates of H D3 H D2 H D1 x) for each row of x.

    x: fp32 CUDA tensor [batch][n]; d1..d3: fp32 CUDA tensors [n].  Allocates
    ``out`` (and the workspace when one is needed) unless given.  Asynchronous
    on ``stream`` (default: torch's current stream).
    """
    import torch

    _check_tensor(x, "x", torch.float32)
    for name, d in (("d1", d1), ("d2", d2), ("d3", d3)):
        _check_tensor(d, name, torch.float32)
    batch, n = x.shape
    for d in (d1, d2, d3):
        if d.numel() != n:
            raise ValueError("diagonal length must equal n")
    m = n if m is None else int(m)
    epi = _epi(epilogue)
    width = 2 * m if epi == SPINNER_EPI_COSSIN else m
    if out is None:
        out = torch.empty((batch, width), dtype=torch.float32, device=x.device)
    else:
        _check_tensor(out, "out", torch.float32)
        if out.numel() != batch * width:
            raise ValueError("out has the wrong size")
    need = spinner_workspace_bytes(n, batch, m, epi)
    if need and workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    if workspace is not None and workspace.numel() * workspace.element_size() < need:
        raise ValueError("workspace too small")
    rc = lib.spinner_apply(x.data_ptr(), n, batch, d1.data_ptr(), d2.data_ptr(), d3.data_ptr(), m, epi,
                           ctypes.c_float(scale), out.data_ptr(),
                           workspace.data_ptr() if workspace is not None else None, _stream_handle(stream))
    if rc != SPINNER_OK:
        raise SpinnerError(rc)
    return out


def spinner_hash(x, diag_sets, out_idx=None, stream=None):
    """Cross-polytope buckets, int32 [batch][L], for L diagonal triples diag_sets fp32 [L][3][n]."""
    import torch

    _check_tensor(x, "x", torch.float32)
    _check_tensor(diag_sets, "diag_sets", torch.float32)
    batch, n = x.shape
    if diag_sets.dim() != 3 or diag_sets.shape[1] != 3 or diag_sets.shape[2] != n:
        raise ValueError("diag_sets must be [L][3][n]")
    L = diag_sets.shape[0]
    if out_idx is None:
        out_idx = torch.empty((batch, L), dtype=torch.int32, device=x.device)
    else:
        _check_tensor(out_idx, "out_idx", torch.int32)
        if out_idx.numel() != batch * L:
            raise ValueError("out_idx has the wrong size")
    rc = lib.spinner_hash(x.data_ptr(), n, batch, L, diag_sets.data_ptr(), out_idx.data_ptr(), _stream_handle(stream))
    if rc != SPINNER_OK:
        raise SpinnerError(rc)
    return out_idx


def spinner_signs_bytes(n: int, L: int) -> int:
    return int(lib.spinner_signs_bytes(int(n), int(L)))


def spinner_pack_signs(diag_sets, stream=None):
    """Pack fp32 +-1 diagonals [L][3][n] into the library's sign words (uint8 CUDA tensor, opaque)."""
    import torch

    _check_tensor(diag_sets, "diag_sets", torch.float32)
    if diag_sets.dim() != 3 or diag_sets.shape[1] != 3:
        raise ValueError("diag_sets must be [L][3][n]")
    L, _, n = diag_sets.shape
    nbytes = spinner_signs_bytes(n, L)
    if nbytes == 0:
        raise SpinnerError(SPINNER_ERR_BAD_N)
    signs = torch.empty(nbytes, dtype=torch.uint8, device=diag_sets.device)
    rc = lib.spinner_pack_signs(diag_sets.data_ptr(), n, L, signs.data_ptr(), _stream_handle(stream))
    if rc != SPINNER_OK:
        raise SpinnerError(rc)
    return signs


def spinner_apply_signs(x, signs, m=None, epilogue="none", scale=1.0, out=None, workspace=None, stream=None,
                        triple=0):
    """spinner_apply for +-1 diagonals given as packed sign words (see spinner_pack_signs)."""
    import torch

    _check_tensor(x, "x", torch.float32)
    batch, n = x.shape
    m = n if m is None else int(m)
    epi = _epi(epilogue)
    width = 2 * m if epi == SPINNER_EPI_COSSIN else m
    if out is None:
        out = torch.empty((batch, width), dtype=torch.float32, device=x.device)
    else:
        _check_tensor(out, "out", torch.float32)
        if out.numel() != batch * width:
            raise ValueError("out has the wrong size")
    one = spinner_signs_bytes(n, 1)
    if signs.numel() < (triple + 1) * one:
        raise ValueError("signs buffer too small for this n / triple")
    need = spinner_workspace_bytes(n, batch, m, epi)
    if need and workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    if workspace is not None and workspace.numel() * workspace.element_size() < need:
        raise ValueError("workspace too small")
    rc = lib.spinner_apply_signs(x.data_ptr(), n, batch, signs.data_ptr() + triple * one, m, epi,
                                 ctypes.c_float(scale), out.data_ptr(),
                                 workspace.data_ptr() if workspace is not None else None, _stream_handle(stream))
    if rc != SPINNER_OK:
        raise SpinnerError(rc)
    return out


def spinner_hash_signs(x, signs, L, out_idx=None, stream=None):
    """spinner_hash for +-1 diagonals given as packed sign words of L triples."""
    import torch

    _check_tensor(x, "x", torch.float32)
    batch, n = x.shape
    if signs.numel() < spinner_signs_bytes(n, L):
        raise ValueError("signs buffer too small")
    if out_idx is None:
        out_idx = torch.empty((batch, L), dtype=torch.int32, device=x.device)
    else:
        _check_tensor(out_idx, "out_idx", torch.int32)
        if out_idx.numel() != batch * L:
            raise ValueError("out_idx has the wrong size")
    rc = lib.spinner_hash_signs(x.data_ptr(), n, batch, L, signs.data_ptr(), out_idx.data_ptr(), _stream_handle(stream))
    if rc != SPINNER_OK:
        raise SpinnerError(rc)
    return out_idx


def spinner_stream_copy(src, dst, stream=None):
    """dst[:] = src with the library's plain copy kernel (measurement aid)."""
    import torch

    _check_tensor(src, "src", torch.float32)
    _check_tensor(dst, "dst", torch.float32)
    if src.numel() != dst.numel():
        raise ValueError("size mismatch")
    rc = lib.spinner_stream_copy(src.data_ptr(), dst.data_ptr(), src.numel(), _stream_handle(stream))
    if rc != SPINNER_OK:
        raise SpinnerError(rc)
    return dst
