"""The C boundary: the shared library loads and exports every symbol include/lsrm.h
declares (no compute calls here: this runs without a GPU)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "lsrm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lsrm_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_entry_points():
    names = _declared()
    for must in ("lsrm_route_blocks", "lsrm_route_blocks_static", "lsrm_route_blocks_3d", "lsrm_nsa_compress", "lsrm_nsa_forward",
                 "lsrm_nsa_backward", "lsrm_workspace_bytes", "lsrm_strerror"):
        assert must in names


def test_library_exports_every_declared_symbol():
    path = os.path.join(ROOT, "paper_2604_05182_amd", "liblsrm.so")
    assert os.path.exists(path), "build first: python -m paper_2604_05182_amd.build"
    lib = ctypes.CDLL(path)
    for name in _declared():
        assert hasattr(lib, name), name


def test_host_side_argument_checks():
    """Validation happens on the host before any HIP call, so it can be exercised here."""
    from paper_2604_05182_amd import binding as B
    ok = B.make_params(512, 2, 16, 2, 64, 3, 128)
    assert B.lsrm_workspace_bytes(ok, B.LSRM_WS_ROUTE) >= 8 * 2 * 8
    assert B.lsrm_workspace_bytes(ok, B.LSRM_WS_FORWARD) >= 1024 * 2 * 64 * 2
    for bad in (B.make_params(500, 2, 16, 2, 64, 3, 128), B.make_params(512, 2, 12, 2, 64, 3, 128),
                B.make_params(512, 2, 16, 2, 64, 3, 127), B.make_params(512, 2, 16, 2, 96, 3, 128),
                B.make_params(512, 2, 16, 2, 64, 129, 128), B.make_params(512, 2, 16, 3, 64, 3, 128, h_kv=2)):
        assert B.lsrm_workspace_bytes(bad, B.LSRM_WS_FORWARD) == 0
    assert B.strerror(B.LSRM_ERR_WORKSPACE).startswith("workspace")
    # null pointers are rejected before anything is launched
    rc = B._lib.lsrm_nsa_compress(__import__("ctypes").byref(ok), None, None, None, None, None)
    assert rc == B.LSRM_ERR_INVALID_ARG
    # the backward takes every head dimension the forward does; null pointers are rejected
    assert B.lsrm_workspace_bytes(ok, B.LSRM_WS_BACKWARD) > 0
    wide = B.make_params(512, 2, 16, 2, 128, 3, 128)
    assert B.lsrm_workspace_bytes(wide, B.LSRM_WS_BACKWARD) > 0
    rc = B._lib.lsrm_nsa_backward(__import__("ctypes").byref(wide), *([None] * 14), 0, None, None, None)
    assert rc == B.LSRM_ERR_INVALID_ARG
    rc = B._lib.lsrm_nsa_backward(__import__("ctypes").byref(ok), *([None] * 14), 0, None, None, None)
    assert rc == B.LSRM_ERR_INVALID_ARG
    # four-rule routing: budgets must fit the row width; the budget struct is required
    r_bad, r_ok = B.lsrm_route3d_params(2, 3, 1, 1, 1), B.lsrm_route3d_params(2, 2, 1, 1, 1)
    assert B.lsrm_workspace_bytes(ok, B.LSRM_WS_ROUTE_3D) >= 16 * 16
    call = B._lib.lsrm_route_blocks_3d
    assert call(__import__("ctypes").byref(ok), __import__("ctypes").byref(r_bad), *([None] * 6), 0, None) \
        == B.LSRM_ERR_INVALID_ARG
    assert call(__import__("ctypes").byref(ok), None, *([None] * 6), 0, None) == B.LSRM_ERR_INVALID_ARG
    assert call(__import__("ctypes").byref(ok), __import__("ctypes").byref(r_ok), *([None] * 6), 0, None) \
        == B.LSRM_ERR_INVALID_ARG          # null output table
    # grouped-query heads and per-channel gates: forward and backward
    gqa = B.make_params(512, 2, 16, 4, 64, 3, 128, h_kv=2)
    chan = B.make_params(512, 2, 16, 2, 64, 3, 128, gate_channels=True)
    for p in (gqa, chan):
        assert B.lsrm_workspace_bytes(p, B.LSRM_WS_FORWARD) > 0
        assert B.lsrm_workspace_bytes(p, B.LSRM_WS_BACKWARD) > 0
    # fewer key/value heads need less room for the packed tiles
    assert B.lsrm_workspace_bytes(gqa, B.LSRM_WS_FORWARD) < B.lsrm_workspace_bytes(
        B.make_params(512, 2, 16, 4, 64, 3, 128), B.LSRM_WS_FORWARD)
    # own-block window and active counts: everywhere
    own = B.make_params(512, 2, 16, 2, 64, 3, 128, window_mode=1)
    assert B.lsrm_workspace_bytes(own, B.LSRM_WS_BACKWARD) > 0
    assert B.lsrm_workspace_bytes(B.make_params(512, 2, 16, 2, 64, 3, 128, window_mode=2), B.LSRM_WS_FORWARD) == 0
    cnt = B.make_params(512, 2, 16, 2, 64, 3, 128)
    cnt.d_block_count = 256            # any non-null device address: only looked at on the device
    assert B.lsrm_workspace_bytes(cnt, B.LSRM_WS_FORWARD) > 0
    assert B.lsrm_workspace_bytes(cnt, B.LSRM_WS_BACKWARD) > 0
