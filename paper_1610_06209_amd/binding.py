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
LIB_PATH = os.path.join(_HERE, "libspinner.so")

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
SPINNER_ERR_SCRATCH_LIMIT = -11

SPINNER_EPI_NONE = 0
SPINNER_EPI_COSSIN = 1
EPILOGUES = {"none": SPINNER_EPI_NONE, "cossin": SPINNER_EPI_COSSIN}

EXPORTS = ["spinner_apply", "spinner_hash", "spinner_workspace_bytes", "spinner_strerror",
           "spinner_version", "spinner_stream_copy", "spinner_signs_bytes", "spinner_pack_signs",
           "spinner_apply_signs", "spinner_hash_signs", "spinner_hash_workspace_bytes", "spinner_hash_ws", "spinner_hash_signs_ws", "spinner_code_bytes", "spinner_codes_workspace_bytes",
           "spinner_code_position", "spinner_sign_codes", "spinner_sign_codes_signs", "spinner_angular_gram",
           "spinner_layer_saved_bytes", "spinner_layer_workspace_bytes", "spinner_layer_forward",
           "spinner_layer_backward", "spinner_sketch_workspace_bytes", "spinner_sketch", "spinner_sketch_gram",
           "spinner_sketch_gram_workspace_bytes", "spinner_sketch_gram_static", "spinner_sketch_gram_static_limit",
           "spinner_blocks_workspace_bytes", "spinner_apply_blocks",
           "spinner_struct_params", "spinner_struct_spectrum_bytes", "spinner_struct_prepare", "spinner_struct_apply",
           "spinner_struct_workspace_bytes", "spinner_struct_apply_ws"]

if not os.path.exists(LIB_PATH):
    raise ImportError(
        "libspinner.so is not built: run `python -m paper_1610_06209_amd.build` "
        "(or __graft_entry__.build()); there is no fallback path")

# PyTorch ships its own HIP runtime and loads it by path; the library must bind to that same copy (it owns
# the device memory and the streams handed in here), so torch is loaded first and the library's
# dependency on libamdhip64 then resolves to the runtime already in the process.
import torch  # noqa: E402,F401

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
lib.spinner_hash_workspace_bytes.restype = ctypes.c_size_t
lib.spinner_hash_workspace_bytes.argtypes = [ctypes.c_int, ctypes.c_long]
lib.spinner_hash_ws.restype = ctypes.c_int
lib.spinner_hash_ws.argtypes = [_vp, ctypes.c_int, ctypes.c_long, ctypes.c_int, _vp, _vp, _vp, _vp]
lib.spinner_hash_signs_ws.restype = ctypes.c_int
lib.spinner_hash_signs_ws.argtypes = [_vp, ctypes.c_int, ctypes.c_long, ctypes.c_int, _vp, _vp, _vp, _vp]
lib.spinner_stream_copy.restype = ctypes.c_int
lib.spinner_stream_copy.argtypes = [_vp, _vp, ctypes.c_size_t, _vp]
lib.spinner_code_bytes.restype = ctypes.c_size_t
lib.spinner_code_bytes.argtypes = [ctypes.c_int]
lib.spinner_codes_workspace_bytes.restype = ctypes.c_size_t
lib.spinner_codes_workspace_bytes.argtypes = [ctypes.c_int, ctypes.c_long]
lib.spinner_code_position.restype = ctypes.c_int
lib.spinner_code_position.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int)]
lib.spinner_sign_codes.restype = ctypes.c_int
lib.spinner_sign_codes.argtypes = [_vp, ctypes.c_int, ctypes.c_long, _vp, _vp, _vp, ctypes.c_int, _vp, _vp, _vp]
lib.spinner_sign_codes_signs.restype = ctypes.c_int
lib.spinner_sign_codes_signs.argtypes = [_vp, ctypes.c_int, ctypes.c_long, _vp, ctypes.c_int, _vp, _vp, _vp]
lib.spinner_angular_gram.restype = ctypes.c_int
lib.spinner_angular_gram.argtypes = [_vp, ctypes.c_long, _vp, ctypes.c_long, ctypes.c_int, _vp, _vp]
lib.spinner_layer_saved_bytes.restype = ctypes.c_size_t
lib.spinner_layer_saved_bytes.argtypes = [ctypes.c_int, ctypes.c_long]
lib.spinner_layer_workspace_bytes.restype = ctypes.c_size_t
lib.spinner_layer_workspace_bytes.argtypes = [ctypes.c_int, ctypes.c_long]
lib.spinner_layer_forward.restype = ctypes.c_int
lib.spinner_layer_forward.argtypes = [_vp, ctypes.c_int, ctypes.c_long, _vp, _vp, _vp, ctypes.c_float, _vp, _vp, _vp]
lib.spinner_layer_backward.restype = ctypes.c_int
lib.spinner_layer_backward.argtypes = [_vp, _vp, _vp, ctypes.c_int, ctypes.c_long, _vp, _vp, _vp, ctypes.c_float, _vp, _vp,
                                       _vp, _vp]
lib.spinner_sketch_workspace_bytes.restype = ctypes.c_size_t
lib.spinner_sketch_workspace_bytes.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int]
lib.spinner_sketch.restype = ctypes.c_int
lib.spinner_sketch.argtypes = [_vp, ctypes.c_int, ctypes.c_int, _vp, _vp, _vp, _vp, ctypes.c_int, ctypes.c_float, _vp, _vp, _vp]
lib.spinner_sketch_gram.restype = ctypes.c_int
lib.spinner_sketch_gram.argtypes = [_vp, ctypes.c_int, ctypes.c_int, _vp, _vp, _vp]
lib.spinner_sketch_gram_workspace_bytes.restype = ctypes.c_size_t
lib.spinner_sketch_gram_workspace_bytes.argtypes = [ctypes.c_int, ctypes.c_int]
lib.spinner_sketch_gram_static.restype = ctypes.c_int
lib.spinner_sketch_gram_static.argtypes = [_vp, ctypes.c_int, ctypes.c_int, _vp, _vp]
lib.spinner_sketch_gram_static_limit.restype = ctypes.c_size_t
lib.spinner_sketch_gram_static_limit.argtypes = []
lib.spinner_blocks_workspace_bytes.restype = ctypes.c_size_t
lib.spinner_blocks_workspace_bytes.argtypes = [ctypes.c_int, ctypes.c_long, ctypes.c_int, ctypes.c_int]
lib.spinner_apply_blocks.restype = ctypes.c_int
lib.spinner_apply_blocks.argtypes = [_vp, ctypes.c_int, ctypes.c_long, ctypes.c_int, _vp, ctypes.c_int, ctypes.c_int,
                                     ctypes.c_float, _vp, _vp, _vp]
lib.spinner_struct_params.restype = ctypes.c_size_t
lib.spinner_struct_params.argtypes = [ctypes.c_int, ctypes.c_int]
lib.spinner_struct_spectrum_bytes.restype = ctypes.c_size_t
lib.spinner_struct_spectrum_bytes.argtypes = [ctypes.c_int, ctypes.c_int]
lib.spinner_struct_prepare.restype = ctypes.c_int
lib.spinner_struct_prepare.argtypes = [ctypes.c_int, _vp, ctypes.c_int, _vp, _vp]
lib.spinner_struct_workspace_bytes.restype = ctypes.c_size_t
lib.spinner_struct_workspace_bytes.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_long]
lib.spinner_struct_apply_ws.restype = ctypes.c_int
lib.spinner_struct_apply_ws.argtypes = [_vp, ctypes.c_int, ctypes.c_long, ctypes.c_int, _vp, _vp, _vp, ctypes.c_int, ctypes.c_float,
                                        _vp, _vp, _vp]
lib.spinner_struct_apply.restype = ctypes.c_int
lib.spinner_struct_apply.argtypes = [_vp, ctypes.c_int, ctypes.c_long, ctypes.c_int, _vp, _vp, _vp, ctypes.c_int, ctypes.c_float,
                                     _vp, _vp]
STRUCT_KINDS = {"circulant": 0, "skew_circulant": 1, "toeplitz": 2, "hankel": 3}


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


def spinner_hash_workspace_bytes(n: int, batch: int) -> int:
    return int(lib.spinner_hash_workspace_bytes(int(n), int(batch)))


def _hash_workspace(x, n, batch, workspace):
    import torch

    need = spinner_hash_workspace_bytes(n, batch)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    if workspace is not None and workspace.numel() * workspace.element_size() < need:
        raise ValueError("workspace too small")
    return workspace


def spinner_hash_ws(x, diag_sets, out_idx=None, workspace=None, stream=None):
    """spinner_hash for every n up to 2^24 (a workspace tensor is made when none is given and one is needed)."""
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
    workspace = _hash_workspace(x, n, batch, workspace)
    rc = lib.spinner_hash_ws(x.data_ptr(), n, batch, L, diag_sets.data_ptr(), out_idx.data_ptr(),
                             workspace.data_ptr() if workspace is not None else None, _stream_handle(stream))
    if rc != SPINNER_OK:
        raise SpinnerError(rc)
    return out_idx


def spinner_hash_signs_ws(x, signs, L, out_idx=None, workspace=None, stream=None):
    """spinner_hash_signs for every n up to 2^24."""
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
    workspace = _hash_workspace(x, n, batch, workspace)
    rc = lib.spinner_hash_signs_ws(x.data_ptr(), n, batch, L, signs.data_ptr(), out_idx.data_ptr(),
                                   workspace.data_ptr() if workspace is not None else None, _stream_handle(stream))
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


def spinner_code_bytes(m: int) -> int:
    return int(lib.spinner_code_bytes(int(m)))


def spinner_codes_workspace_bytes(n: int, batch: int) -> int:
    return int(lib.spinner_codes_workspace_bytes(int(n), int(batch)))


def spinner_code_position(coordinate: int):
    """(word, bit) of a coordinate inside a row of sign codes."""
    w, b = ctypes.c_int(), ctypes.c_int()
    rc = lib.spinner_code_position(int(coordinate), ctypes.byref(w), ctypes.byref(b))
    if rc != SPINNER_OK:
        raise SpinnerError(rc)
    return w.value, b.value


def _codes_out(x, m, codes):
    import torch

    batch = x.shape[0]
    nbytes = spinner_code_bytes(m)
    if nbytes == 0:
        raise SpinnerError(SPINNER_ERR_BAD_M)
    if codes is None:
        codes = torch.empty((batch, nbytes // 8), dtype=torch.int64, device=x.device)
    else:
        _check_tensor(codes, "codes", torch.int64)
        if codes.numel() != batch * (nbytes // 8):
            raise ValueError("codes has the wrong size")
    return codes


def _codes_workspace(x, workspace):
    import torch

    batch, n = x.shape
    need = spinner_codes_workspace_bytes(n, batch)
    if need and workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    if workspace is not None and workspace.numel() * workspace.element_size() < need:
        raise ValueError("workspace too small")
    return workspace


def spinner_sign_codes(x, d1, d2, d3, m=None, codes=None, workspace=None, stream=None):
    """Sign bits of the first m coordinates of H D3 H D2 H D1 x, int64 CUDA tensor [batch][m/64]."""
    import torch

    _check_tensor(x, "x", torch.float32)
    for name, d in (("d1", d1), ("d2", d2), ("d3", d3)):
        _check_tensor(d, name, torch.float32)
    batch, n = x.shape
    m = n if m is None else int(m)
    codes = _codes_out(x, m, codes)
    workspace = _codes_workspace(x, workspace)
    rc = lib.spinner_sign_codes(x.data_ptr(), n, batch, d1.data_ptr(), d2.data_ptr(), d3.data_ptr(), m, codes.data_ptr(),
                                workspace.data_ptr() if workspace is not None else None, _stream_handle(stream))
    if rc != SPINNER_OK:
        raise SpinnerError(rc)
    return codes


def spinner_sign_codes_signs(x, signs, m=None, codes=None, workspace=None, stream=None, triple=0):
    """spinner_sign_codes for +-1 diagonals given as packed sign words (see spinner_pack_signs)."""
    import torch

    _check_tensor(x, "x", torch.float32)
    batch, n = x.shape
    m = n if m is None else int(m)
    codes = _codes_out(x, m, codes)
    workspace = _codes_workspace(x, workspace)
    one = spinner_signs_bytes(n, 1)
    if signs.numel() < (triple + 1) * one:
        raise ValueError("signs buffer too small for this n / triple")
    rc = lib.spinner_sign_codes_signs(x.data_ptr(), n, batch, signs.data_ptr() + triple * one, m, codes.data_ptr(),
                                      workspace.data_ptr() if workspace is not None else None, _stream_handle(stream))
    if rc != SPINNER_OK:
        raise SpinnerError(rc)
    return codes


def spinner_angular_gram(codes_a, codes_b, m, out=None, stream=None):
    """out[i][j] = 1 - Hamming(codes_a[i], codes_b[j]) / m, fp32 CUDA tensor [na][nb]."""
    import torch

    _check_tensor(codes_a, "codes_a", torch.int64)
    _check_tensor(codes_b, "codes_b", torch.int64)
    words = spinner_code_bytes(m) // 8
    if words == 0:
        raise SpinnerError(SPINNER_ERR_BAD_M)
    if codes_a.shape[-1] != words or codes_b.shape[-1] != words:
        raise ValueError("codes do not have m / 64 words per row")
    na, nb = codes_a.shape[0], codes_b.shape[0]
    if out is None:
        out = torch.empty((na, nb), dtype=torch.float32, device=codes_a.device)
    else:
        _check_tensor(out, "out", torch.float32)
        if out.numel() != na * nb:
            raise ValueError("out has the wrong size")
    rc = lib.spinner_angular_gram(codes_a.data_ptr(), na, codes_b.data_ptr(), nb, int(m), out.data_ptr(),
                                  _stream_handle(stream))
    if rc != SPINNER_OK:
        raise SpinnerError(rc)
    return out


def spinner_layer_saved_bytes(n: int, batch: int) -> int:
    return int(lib.spinner_layer_saved_bytes(int(n), int(batch)))


def spinner_layer_workspace_bytes(n: int, batch: int) -> int:
    return int(lib.spinner_layer_workspace_bytes(int(n), int(batch)))


def spinner_layer_forward(x, d1, d2, d3, scale=1.0, y=None, saved=None, stream=None):
    """y = scale * H D3 H D2 H D1 x and the opaque activations the backward pass needs: returns (y, saved)."""
    import torch

    _check_tensor(x, "x", torch.float32)
    for name, d in (("d1", d1), ("d2", d2), ("d3", d3)):
        _check_tensor(d, name, torch.float32)
    batch, n = x.shape
    if y is None:
        y = torch.empty_like(x)
    else:
        _check_tensor(y, "y", torch.float32)
    if saved is None:
        saved = torch.empty((2, batch, n), dtype=torch.float32, device=x.device)
    else:
        _check_tensor(saved, "saved", torch.float32)
        if saved.numel() != 2 * batch * n:
            raise ValueError("saved has the wrong size")
    rc = lib.spinner_layer_forward(x.data_ptr(), n, batch, d1.data_ptr(), d2.data_ptr(), d3.data_ptr(),
                                   ctypes.c_float(scale), y.data_ptr(), saved.data_ptr(), _stream_handle(stream))
    if rc != SPINNER_OK:
        raise SpinnerError(rc)
    return y, saved


def spinner_layer_backward(dy, x, saved, d1, d2, d3, scale=1.0, dx=None, dd=None, workspace=None, stream=None):
    """Gradients for x ([batch][n]) and for the three diagonals ([3][n], summed over the batch): returns (dx, dd)."""
    import torch

    for name, t in (("dy", dy), ("x", x), ("saved", saved), ("d1", d1), ("d2", d2), ("d3", d3)):
        _check_tensor(t, name, torch.float32)
    batch, n = x.shape
    if dy.shape != x.shape or saved.numel() != 2 * batch * n:
        raise ValueError("dy / saved do not match x")
    if dx is None:
        dx = torch.empty_like(x)
    if dd is None:
        dd = torch.empty((3, n), dtype=torch.float32, device=x.device)
    need = spinner_layer_workspace_bytes(n, batch)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=x.device)
    if workspace.numel() * workspace.element_size() < need:
        raise ValueError("workspace too small")
    rc = lib.spinner_layer_backward(dy.data_ptr(), x.data_ptr(), saved.data_ptr(), n, batch, d1.data_ptr(), d2.data_ptr(),
                                    d3.data_ptr(), ctypes.c_float(scale), dx.data_ptr(), dd.data_ptr(), workspace.data_ptr(),
                                    _stream_handle(stream))
    if rc != SPINNER_OK:
        raise SpinnerError(rc)
    return dx, dd


def spinner_sketch_workspace_bytes(n: int, d: int, m: int) -> int:
    return int(lib.spinner_sketch_workspace_bytes(int(n), int(d), int(m)))


def spinner_sketch(A, w, d1, d2, d3, m, scale=1.0, out=None, workspace=None, stream=None):
    """B = scale * (first m rows of H D3 H D2 H D1) diag(w) A for A fp32 [n][d]; w may be None.  Returns B [m][d]."""
    import torch

    _check_tensor(A, "A", torch.float32)
    for name, t in (("d1", d1), ("d2", d2), ("d3", d3)):
        _check_tensor(t, name, torch.float32)
    if w is not None:
        _check_tensor(w, "w", torch.float32)
    n, d = A.shape
    if out is None:
        out = torch.empty((int(m), d), dtype=torch.float32, device=A.device)
    else:
        _check_tensor(out, "out", torch.float32)
        if out.numel() != int(m) * d:
            raise ValueError("out has the wrong size")
    need = spinner_sketch_workspace_bytes(n, d, m)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=A.device)
    if workspace.numel() * workspace.element_size() < need:
        raise ValueError("workspace too small")
    rc = lib.spinner_sketch(A.data_ptr(), n, d, w.data_ptr() if w is not None else None, d1.data_ptr(), d2.data_ptr(),
                            d3.data_ptr(), int(m), ctypes.c_float(scale), out.data_ptr(), workspace.data_ptr(),
                            _stream_handle(stream))
    if rc != SPINNER_OK:
        raise SpinnerError(rc)
    return out


def spinner_sketch_gram_static_limit() -> int:
    return int(lib.spinner_sketch_gram_static_limit())


def spinner_sketch_gram_static(B, out, stream=None):
    """G = B^T B into the caller's `out` [d][d]; the call allocates nothing (the library's built-in scratch)."""
    import torch

    _check_tensor(B, "B", torch.float32)
    _check_tensor(out, "out", torch.float32)
    m, d = B.shape
    if out.numel() != d * d:
        raise ValueError("out has the wrong size")
    rc = lib.spinner_sketch_gram_static(B.data_ptr(), m, d, out.data_ptr(), _stream_handle(stream))
    if rc != SPINNER_OK:
        raise SpinnerError(rc)
    return out


def spinner_sketch_gram_workspace_bytes(m: int, d: int) -> int:
    return int(lib.spinner_sketch_gram_workspace_bytes(int(m), int(d)))


def spinner_sketch_gram(B, out=None, workspace=None, stream=None):
    """G = B^T B, fp32 CUDA tensor [d][d]."""
    import torch

    _check_tensor(B, "B", torch.float32)
    m, d = B.shape
    if out is None:
        out = torch.empty((d, d), dtype=torch.float32, device=B.device)
    else:
        _check_tensor(out, "out", torch.float32)
        if out.numel() != d * d:
            raise ValueError("out has the wrong size")
    need = spinner_sketch_gram_workspace_bytes(m, d)
    if need and workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=B.device)
    if workspace is not None and workspace.numel() * workspace.element_size() < need:
        raise ValueError("workspace too small")
    rc = lib.spinner_sketch_gram(B.data_ptr(), m, d, out.data_ptr(), workspace.data_ptr() if workspace is not None else None,
                                 _stream_handle(stream))
    if rc != SPINNER_OK:
        raise SpinnerError(rc)
    return out


def spinner_apply_blocks(x, diag_sets, m=None, epilogue="none", scale=1.0, out=None, workspace=None, stream=None):
    """L independent triples (diag_sets fp32 [L][3][n]) applied to the same x, their m-row blocks side by side:
    out [batch][L m] (epilogue none) or [batch][2 L m] (cos block | sin block)."""
    import torch

    _check_tensor(x, "x", torch.float32)
    _check_tensor(diag_sets, "diag_sets", torch.float32)
    batch, n = x.shape
    if diag_sets.dim() != 3 or diag_sets.shape[1] != 3 or diag_sets.shape[2] != n:
        raise ValueError("diag_sets must be [L][3][n]")
    L = diag_sets.shape[0]
    m = n if m is None else int(m)
    epi = _epi(epilogue)
    width = (2 * m if epi == SPINNER_EPI_COSSIN else m) * L
    if out is None:
        out = torch.empty((batch, width), dtype=torch.float32, device=x.device)
    else:
        _check_tensor(out, "out", torch.float32)
        if out.numel() != batch * width:
            raise ValueError("out has the wrong size")
    need = int(lib.spinner_blocks_workspace_bytes(n, batch, m, epi))
    if need and workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    if workspace is not None and workspace.numel() * workspace.element_size() < need:
        raise ValueError("workspace too small")
    rc = lib.spinner_apply_blocks(x.data_ptr(), n, batch, L, diag_sets.data_ptr(), m, epi, ctypes.c_float(scale),
                                  out.data_ptr(), workspace.data_ptr() if workspace is not None else None,
                                  _stream_handle(stream))
    if rc != SPINNER_OK:
        raise SpinnerError(rc)
    return out


def spinner_struct_prepare(kind, params, n, stream=None):
    """Opaque spectrum (uint8 CUDA tensor) of a structured third block from its generating vector (fp32 CUDA tensor)."""
    import torch

    k = STRUCT_KINDS[kind] if isinstance(kind, str) else int(kind)
    _check_tensor(params, "params", torch.float32)
    nbytes = int(lib.spinner_struct_spectrum_bytes(k, int(n)))
    if nbytes == 0:
        raise SpinnerError(SPINNER_ERR_UNSUPPORTED)
    if params.numel() != int(lib.spinner_struct_params(k, int(n))):
        raise ValueError("generating vector has the wrong length")
    spec = torch.empty(nbytes, dtype=torch.uint8, device=params.device)
    rc = lib.spinner_struct_prepare(k, params.data_ptr(), int(n), spec.data_ptr(), _stream_handle(stream))
    if rc != SPINNER_OK:
        raise SpinnerError(rc)
    return spec


def spinner_struct_apply(x, kind, spectrum, d1, d2, m=None, scale=1.0, out=None, stream=None):
    """out [batch][m] = scale * (first m rows of G_struct D2 H D1 x)."""
    import torch

    k = STRUCT_KINDS[kind] if isinstance(kind, str) else int(kind)
    for name, t in (("x", x), ("d1", d1), ("d2", d2)):
        _check_tensor(t, name, torch.float32)
    batch, n = x.shape
    m = n if m is None else int(m)
    if out is None:
        out = torch.empty((batch, m), dtype=torch.float32, device=x.device)
    else:
        _check_tensor(out, "out", torch.float32)
        if out.numel() != batch * m:
            raise ValueError("out has the wrong size")
    rc = lib.spinner_struct_apply(x.data_ptr(), n, batch, k, spectrum.data_ptr(), d1.data_ptr(), d2.data_ptr(), m,
                                  ctypes.c_float(scale), out.data_ptr(), _stream_handle(stream))
    if rc != SPINNER_OK:
        raise SpinnerError(rc)
    return out


def spinner_struct_workspace_bytes(kind, n: int, batch: int) -> int:
    k = STRUCT_KINDS[kind] if isinstance(kind, str) else int(kind)
    return int(lib.spinner_struct_workspace_bytes(k, int(n), int(batch)))


def spinner_struct_apply_ws(x, kind, spectrum, d1, d2, m=None, scale=1.0, out=None, workspace=None, stream=None):
    """spinner_struct_apply for every supported n (a workspace tensor is made when none is given and one is needed)."""
    import torch

    k = STRUCT_KINDS[kind] if isinstance(kind, str) else int(kind)
    for name, t in (("x", x), ("d1", d1), ("d2", d2)):
        _check_tensor(t, name, torch.float32)
    batch, n = x.shape
    m = n if m is None else int(m)
    if out is None:
        out = torch.empty((batch, m), dtype=torch.float32, device=x.device)
    else:
        _check_tensor(out, "out", torch.float32)
        if out.numel() != batch * m:
            raise ValueError("out has the wrong size")
    need = spinner_struct_workspace_bytes(k, n, batch)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    if workspace is not None and workspace.numel() * workspace.element_size() < need:
        raise ValueError("workspace too small")
    rc = lib.spinner_struct_apply_ws(x.data_ptr(), n, batch, k, spectrum.data_ptr(), d1.data_ptr(), d2.data_ptr(), m,
                                     ctypes.c_float(scale), out.data_ptr(),
                                     workspace.data_ptr() if workspace is not None else None, _stream_handle(stream))
    if rc != SPINNER_OK:
        raise SpinnerError(rc)
    return out
