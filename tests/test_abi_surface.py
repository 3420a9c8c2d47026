"""CPU-side checks of the boundary: the built library loads and exports every symbol the header
declares; pure host functions behave.  No compute call is made."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    names = []
    for fn in os.listdir(os.path.join(ROOT, "include")):
        if fn.endswith(".h"):
            src = open(os.path.join(ROOT, "include", fn)).read()
            names += re.findall(r"S3GD_API\s+[\w\s\*]+?\b(s3gd_\w+)\s*\(", src)
    return sorted(set(names))


def test_library_exports_every_declared_symbol(lib):
    decl = _declared()
    assert len(decl) >= 11
    so = ctypes.CDLL(lib.LIB_PATH)
    for name in decl:
        assert hasattr(so, name), name
    assert sorted(lib.EXPORTS) == decl


def test_named_entry_points_present(lib):
    for name in ("s3gd_topk_sign_encode", "s3gd_majority_vote", "s3gd_apply_update"):
        assert name in lib.EXPORTS


def test_workspace_bytes_is_pure_and_monotone(lib):
    a = lib.workspace_bytes(4, 1_000_000, 1000)
    b = lib.workspace_bytes(8, 1_000_000, 1000)
    c = lib.workspace_bytes(8, 4_000_000, 1000)
    assert 0 < a < b < c
    assert lib.workspace_bytes(0, 10, 1) == 0
    assert lib.workspace_bytes(1, (1 << 31) - 1, 1) == 0  # above the index limit
    # scratch stays a small fraction of the gradients it serves
    M, N = 4, 1_200_000_000
    assert lib.workspace_bytes(M, N, N // 1000) < 0.025 * 4 * M * N


def test_strerror(lib):
    assert lib.strerror(0) == "ok"
    for code in (lib.E_INVAL, lib.E_RANGE, lib.E_HIP, lib.E_NOMEM, lib.E_NAN):
        assert lib.strerror(code) not in ("ok", "unknown error")
    assert lib.strerror(-99) == "unknown error"


def test_create_rejects_bad_arguments_without_touching_a_device(lib):
    h = ctypes.c_void_p()
    assert lib.raw.s3gd_create(None, 0, 1, 10, 1) == lib.E_INVAL
    assert lib.raw.s3gd_create(ctypes.byref(h), 0, 0, 10, 1) == lib.E_INVAL
    assert lib.raw.s3gd_create(ctypes.byref(h), 0, 65536, 10, 1) == lib.E_INVAL  # above S3GD_M_LIMIT, as the header says
    assert lib.raw.s3gd_create(ctypes.byref(h), 0, 1, 0, 1) == lib.E_INVAL
    assert lib.raw.s3gd_create(ctypes.byref(h), 0, 1, (1 << 31) - 1, 1) == lib.E_RANGE
    assert lib.raw.s3gd_create(ctypes.byref(h), -1, 1, 10, 1) == lib.E_INVAL
    assert lib.raw.s3gd_destroy(None) == lib.E_INVAL
