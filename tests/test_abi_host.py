"""Host-only checks of the C-ABI library: it loads, exports every entry point the
header declares, and turns invalid arguments into status codes before any launch
(no GPU work is issued by these tests)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "spinner.h")


@pytest.fixture(scope="module")
def b():
    from paper_1610_06209_amd import binding

    return binding


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(spinner_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(b):
    names = _declared_functions()
    assert names == sorted(b.EXPORTS)
    for name in names:
        assert getattr(b.lib, name) is not None


def test_version_and_messages(b):
    assert b.spinner_version() >= 100
    assert b.spinner_strerror(0) == "success"
    for code in range(-11, 0):
        msg = b.spinner_strerror(code)
        assert msg and msg != "unknown status"
    assert b.spinner_strerror(-99) == "unknown status"


def test_workspace_bytes(b):
    assert b.spinner_workspace_bytes(1 << 14, 32768, 1024, "none") == 0
    assert b.spinner_workspace_bytes(1 << 16, 64, 1024, "none") == 0            # still one fused kernel
    assert b.spinner_workspace_bytes(1 << 15, 64, 1024, "cossin") == 64 * (1 << 15) * 4
    assert b.spinner_workspace_bytes(1 << 20, 256, 1 << 20, "none") == 0          # in place in out
    assert b.spinner_workspace_bytes(1 << 20, 256, 1024, "none") == 256 * (1 << 20) * 4
    assert b.spinner_workspace_bytes(1 << 20, 256, 1 << 20, "cossin") == 256 * (1 << 20) * 4
    assert b.spinner_workspace_bytes(1000, 4, 10, "none") == 0                    # invalid -> 0


def _apply(b, n=256, batch=4, m=256, epi=0, x=64, d1=64, d2=64, d3=64, out=64, ws=None):
    return b.lib.spinner_apply(x, n, batch, d1, d2, d3, m, epi, ctypes.c_float(1.0), out, ws, None)


def test_apply_rejects_bad_arguments_before_launch(b):
    # pointers are fake but aligned; every call below must return before touching them
    assert _apply(b, n=100) == b.SPINNER_ERR_BAD_N
    assert _apply(b, n=8) == b.SPINNER_ERR_BAD_N
    assert _apply(b, n=1 << 25) == b.SPINNER_ERR_BAD_N
    assert _apply(b, n=0) == b.SPINNER_ERR_BAD_N
    assert _apply(b, m=0) == b.SPINNER_ERR_BAD_M
    assert _apply(b, m=257) == b.SPINNER_ERR_BAD_M
    assert _apply(b, epi=2) == b.SPINNER_ERR_BAD_EPILOGUE
    assert _apply(b, batch=-1) == b.SPINNER_ERR_BAD_BATCH
    assert _apply(b, x=None) == b.SPINNER_ERR_NULL_PTR
    assert _apply(b, d2=None) == b.SPINNER_ERR_NULL_PTR
    assert _apply(b, out=None) == b.SPINNER_ERR_NULL_PTR
    assert _apply(b, d3=8) == b.SPINNER_ERR_ALIGNMENT
    assert _apply(b, out=68) == b.SPINNER_ERR_ALIGNMENT
    assert _apply(b, n=1 << 20, m=1024) == b.SPINNER_ERR_WORKSPACE
    assert _apply(b, batch=0, x=None, out=None) == b.SPINNER_OK                    # empty batch: no-op


def test_hash_rejects_bad_arguments_before_launch(b):
    h = b.lib.spinner_hash
    assert h(64, 1000, 4, 2, 64, 64, None) == b.SPINNER_ERR_BAD_N
    assert h(64, 1024, 4, 0, 64, 64, None) == b.SPINNER_ERR_BAD_L
    assert h(64, 1024, -2, 2, 64, 64, None) == b.SPINNER_ERR_BAD_BATCH
    assert h(None, 1024, 4, 2, 64, 64, None) == b.SPINNER_ERR_NULL_PTR
    assert h(64, 1024, 4, 2, 64, None, None) == b.SPINNER_ERR_NULL_PTR
    assert h(4, 1024, 4, 2, 64, 64, None) == b.SPINNER_ERR_ALIGNMENT
    assert h(64, 1 << 17, 4, 2, 64, 64, None) == b.SPINNER_ERR_UNSUPPORTED
    assert h(None, 1024, 0, 2, None, None, None) == b.SPINNER_OK
    # the variant with a workspace serves every n; above 2^16 the workspace holds the projection and the candidates
    hw = b.lib.spinner_hash_ws
    assert b.spinner_hash_workspace_bytes(1 << 16, 8) == 0 and b.spinner_hash_workspace_bytes(1000, 8) == 0
    assert b.spinner_hash_workspace_bytes(1 << 17, 3) == 3 * (1 << 17) * 4 + 3 * 2 * 8
    assert b.spinner_hash_workspace_bytes(1 << 24, 1) == (1 << 26) + 256 * 8
    assert hw(64, 1 << 17, 4, 2, 64, 64, None, None) == b.SPINNER_ERR_WORKSPACE
    assert hw(64, 1 << 17, 4, 2, 64, 64, 72, None) == b.SPINNER_ERR_ALIGNMENT
    assert hw(64, 1 << 17, 4, 0, 64, 64, 64, None) == b.SPINNER_ERR_BAD_L
    assert hw(64, 1 << 25, 4, 2, 64, 64, 64, None) == b.SPINNER_ERR_BAD_N
    assert hw(None, 1 << 17, 4, 2, 64, 64, 64, None) == b.SPINNER_ERR_NULL_PTR
    assert hw(None, 1 << 17, 0, 2, None, None, None, None) == b.SPINNER_OK
    assert b.lib.spinner_hash_signs_ws(64, 1 << 17, 4, 2, None, 64, 64, None) == b.SPINNER_ERR_NULL_PTR


def test_sign_word_entry_points_reject_bad_arguments(b):
    assert b.spinner_signs_bytes(2048, 1) == 3 * 32 * 8
    # n = 1024 also carries the lane masks of its hash kernel's two layouts: [3][2][32] words per triple
    assert b.spinner_signs_bytes(1024, 1) == 3 * 16 * 8 + 3 * 2 * 32 * 8
    assert b.spinner_signs_bytes(1024, 5) == 5 * b.spinner_signs_bytes(1024, 1)
    # sign words, lane masks of the all-register feature kernel, lane masks of the second layout of the wide exchange
    assert b.spinner_signs_bytes(4096, 1) == 3 * 64 * 8 + 3 * 2 * 64 * 8 + 3 * 64 * 8
    assert b.spinner_signs_bytes(16384, 2) == 2 * (3 * 256 * 8 + 3 * 256 * 8)
    assert b.spinner_signs_bytes(64, 2) == 2 * 3 * 4 * 8
    assert b.spinner_signs_bytes(256, 1) == 3 * 4 * 8 + 3 * 2 * 16 * 8
    # above 2^14: sign words, lane masks of the four-pass schedule's column pass; at 2^15 also the fp32 diagonals
    assert b.spinner_signs_bytes(1 << 15, 1) == 4 * 512 * 8 + 3 * (1 << 15) * 4
    assert b.spinner_signs_bytes(1 << 16, 1) == 4 * 1024 * 8
    assert b.spinner_signs_bytes(1 << 17, 1) == 4 * 2048 * 8
    assert b.spinner_signs_bytes(1 << 24, 2) == 2 * 4 * (1 << 18) * 8
    assert b.spinner_signs_bytes(1000, 1) == 0 and b.spinner_signs_bytes(1024, 0) == 0
    pk = b.lib.spinner_pack_signs
    assert pk(64, 1000, 1, 64, None) == b.SPINNER_ERR_BAD_N
    assert pk(64, 1024, 0, 64, None) == b.SPINNER_ERR_BAD_L
    assert pk(None, 1024, 1, 64, None) == b.SPINNER_ERR_NULL_PTR
    assert pk(64, 1024, 1, 72, None) == b.SPINNER_ERR_ALIGNMENT
    ap = b.lib.spinner_apply_signs
    assert ap(64, 1024, 4, None, 1024, 0, ctypes.c_float(1.0), 64, None, None) == b.SPINNER_ERR_NULL_PTR
    assert ap(64, 1024, 4, 64, 2000, 0, ctypes.c_float(1.0), 64, None, None) == b.SPINNER_ERR_BAD_M
    assert ap(64, 1024, 4, 8, 1024, 0, ctypes.c_float(1.0), 64, None, None) == b.SPINNER_ERR_ALIGNMENT
    hs = b.lib.spinner_hash_signs
    assert hs(64, 1024, 4, 2, None, 64, None) == b.SPINNER_ERR_NULL_PTR
    assert hs(64, 1 << 17, 4, 2, 64, 64, None) == b.SPINNER_ERR_UNSUPPORTED


def test_sign_code_entry_points_host_side(b):
    assert b.spinner_code_bytes(256) == 32 and b.spinner_code_bytes(4096) == 512
    assert b.spinner_code_bytes(0) == 0 and b.spinner_code_bytes(320) == 0 and b.spinner_code_bytes(128) == 0
    assert b.spinner_codes_workspace_bytes(1 << 16, 100) == 0
    assert b.spinner_codes_workspace_bytes(1 << 17, 100) == 100 * (1 << 17) * 4
    # the documented layout: 64 consecutive multiples-of-four offsets share a word; every (word, bit) is hit once
    assert b.spinner_code_position(0) == (0, 0) and b.spinner_code_position(1) == (1, 0)
    assert b.spinner_code_position(4) == (0, 1) and b.spinner_code_position(255) == (3, 63)
    assert b.spinner_code_position(256) == (4, 0) and b.spinner_code_position(1023) == (15, 63)
    seen = {b.spinner_code_position(e) for e in range(2048)}
    assert len(seen) == 2048 and max(w for w, _ in seen) == 2048 // 64 - 1
    sc = b.lib.spinner_sign_codes
    assert sc(64, 1000, 4, 64, 64, 64, 256, 64, None, None) == b.SPINNER_ERR_BAD_N
    assert sc(64, 128, 4, 64, 64, 64, 128, 64, None, None) == b.SPINNER_ERR_UNSUPPORTED
    assert sc(64, 1024, 4, 64, 64, 64, 300, 64, None, None) == b.SPINNER_ERR_BAD_M
    assert sc(64, 1024, 4, 64, 64, 64, 2048, 64, None, None) == b.SPINNER_ERR_BAD_M
    assert sc(64, 1024, 4, None, 64, 64, 1024, 64, None, None) == b.SPINNER_ERR_NULL_PTR
    assert sc(64, 1024, 4, 64, 64, 64, 1024, None, None, None) == b.SPINNER_ERR_NULL_PTR
    assert sc(64, 1024, 4, 64, 64, 64, 1024, 72, None, None) == b.SPINNER_ERR_ALIGNMENT
    assert sc(64, 1 << 17, 4, 64, 64, 64, 1024, 64, None, None) == b.SPINNER_ERR_WORKSPACE
    assert sc(64, 1024, 0, None, None, None, 1024, None, None, None) == b.SPINNER_OK       # empty batch: nothing to do
    ss = b.lib.spinner_sign_codes_signs
    assert ss(64, 1024, 4, None, 1024, 64, None, None) == b.SPINNER_ERR_NULL_PTR
    assert ss(64, 1024, 4, 64, 100, 64, None, None) == b.SPINNER_ERR_BAD_M
    ag = b.lib.spinner_angular_gram
    assert ag(64, 4, 64, 4, 100, 64, None) == b.SPINNER_ERR_BAD_M
    assert ag(None, 4, 64, 4, 256, 64, None) == b.SPINNER_ERR_NULL_PTR
    assert ag(64, 4, 64, 4, 256, 68, None) == b.SPINNER_ERR_ALIGNMENT
    assert ag(64, -1, 64, 4, 256, 64, None) == b.SPINNER_ERR_BAD_BATCH
    assert ag(None, 0, None, 4, 256, None, None) == b.SPINNER_OK


def test_layer_entry_points_host_side(b):
    assert b.spinner_layer_saved_bytes(1024, 10) == 2 * 10 * 1024 * 4
    assert b.spinner_layer_saved_bytes(1 << 15, 10) == 2 * 10 * (1 << 15) * 4 and b.spinner_layer_saved_bytes(1000, 10) == 0
    # one partial row of 3 n floats per tile slot: small batches take one slot per vector (rounded up to whole workgroups)
    assert b.spinner_layer_workspace_bytes(4096, 8) == 8 * 3 * 4096 * 4
    # large batches: as many slots as tiles are resident on the chip (four workgroups per compute unit, or what the
    # backward kernel of that size is compiled for)
    assert b.spinner_layer_workspace_bytes(1024, 1 << 20) == 4096 * 3 * 1024 * 4
    assert b.spinner_layer_workspace_bytes(2048, 1 << 20) == 1536 * 3 * 2048 * 4
    assert b.spinner_layer_workspace_bytes(4096, 1 << 20) == 768 * 3 * 4096 * 4
    assert b.spinner_layer_workspace_bytes(8192, 1 << 20) == 512 * 3 * 8192 * 4
    assert b.spinner_layer_workspace_bytes(16, 1 << 20) == 8192 * 3 * 16 * 4          # bounded number of partial rows
    # above 2^14: two signal buffers and one partial row per slab of the batch sums (never more slabs than vectors)
    assert b.spinner_layer_workspace_bytes(1 << 15, 8) == (2 * 8 + 8) * (1 << 15) * 4
    assert b.spinner_layer_workspace_bytes(1 << 15, 1000) == (2 * 1000 + 64) * (1 << 15) * 4
    assert b.spinner_layer_workspace_bytes(1 << 24, 3) == (2 * 3 + 1) * (1 << 24) * 4
    f = b.lib.spinner_layer_forward
    one = ctypes.c_float(1.0)
    assert f(64, 1000, 4, 64, 64, 64, one, 64, 64, None) == b.SPINNER_ERR_BAD_N
    assert f(64, 1 << 25, 4, 64, 64, 64, one, 64, 64, None) == b.SPINNER_ERR_BAD_N
    assert f(64, 1 << 15, 4, 64, 64, 64, one, 64, None, None) == b.SPINNER_ERR_NULL_PTR
    assert f(64, 1024, -1, 64, 64, 64, one, 64, 64, None) == b.SPINNER_ERR_BAD_BATCH
    assert f(64, 1024, 4, 64, None, 64, one, 64, 64, None) == b.SPINNER_ERR_NULL_PTR
    assert f(64, 1024, 4, 64, 64, 64, one, 64, None, None) == b.SPINNER_ERR_NULL_PTR
    assert f(64, 1024, 4, 64, 64, 64, one, 72, 64, None) == b.SPINNER_ERR_ALIGNMENT
    assert f(None, 1024, 0, None, None, None, one, None, None, None) == b.SPINNER_OK
    g = b.lib.spinner_layer_backward
    assert g(64, 64, 64, 1000, 4, 64, 64, 64, one, 64, 64, 64, None) == b.SPINNER_ERR_BAD_N
    assert g(64, 64, 64, 1024, 4, 64, 64, 64, one, 64, 64, None, None) == b.SPINNER_ERR_WORKSPACE
    assert g(64, 64, 64, 1 << 17, 4, 64, 64, 64, one, 64, 64, None, None) == b.SPINNER_ERR_WORKSPACE
    assert g(64, None, 64, 1024, 4, 64, 64, 64, one, 64, 64, 64, None) == b.SPINNER_ERR_NULL_PTR
    assert g(64, 64, 64, 1024, 4, 64, 64, 64, one, 64, 68, 64, None) == b.SPINNER_ERR_ALIGNMENT
    assert g(None, None, None, 1024, 0, None, None, None, one, None, None, None, None) == b.SPINNER_OK


def test_stream_copy_rejects_bad_arguments(b):
    c = b.lib.spinner_stream_copy
    assert c(None, 64, 16, None) == b.SPINNER_ERR_NULL_PTR
    assert c(64, 68, 16, None) == b.SPINNER_ERR_ALIGNMENT
    assert c(64, 64, 6, None) == b.SPINNER_ERR_ALIGNMENT
    assert c(64, 64, 0, None) == b.SPINNER_OK


def test_workloads_module_is_independent():
    # the shared input recipes import neither side and carry none of the method's arithmetic
    src = open(os.path.join(ROOT, "paper_1610_06209_amd", "workloads.py")).read()
    code = "\n".join(l for l in src.splitlines() if not l.lstrip().startswith("#"))
    for word in ("import oracle", "from oracle", "binding", "popcount", "argmax", "np.cos", "np.sin", "ctypes"):
        assert word not in code.split('"""', 2)[2], word
    osrc = open(os.path.join(ROOT, "oracle", "spinner_oracle.py")).read()
    assert "paper_1610_06209_amd" not in osrc
