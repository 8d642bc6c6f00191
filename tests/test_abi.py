"""The C-ABI library loads and exports every symbol include/attnpack.h declares
(no compute calls: runs without a GPU)."""
import ctypes
import os
import re

import torch  # noqa: F401  (first: its HIP runtime must be the one the library binds to)

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2603_23914_amd", "libattnpack.so")


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "attnpack.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ap_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    assert os.path.exists(LIB), "build first: python -m paper_2603_23914_amd.build"
    lib = ctypes.CDLL(LIB)
    syms = declared_symbols()
    assert {"ap_compact", "ap_select_ranks", "ap_decode_attn"} <= set(syms)
    for s in syms:
        assert hasattr(lib, s), f"{s} declared in attnpack.h but not exported"


def test_host_only_entry_points():
    lib = ctypes.CDLL(LIB)
    lib.ap_status_string.restype = ctypes.c_char_p
    lib.ap_last_error.restype = ctypes.c_char_p
    assert lib.ap_status_string(0) == b"AP_OK"
    assert lib.ap_status_string(3) == b"AP_ERR_WORKSPACE"
    assert lib.ap_version() >= 100
    lib.ap_decode_workspace_bytes.restype = ctypes.c_size_t
    assert lib.ap_decode_workspace_bytes(1, 4, 32, 64, 16, 0) > 0
    assert lib.ap_decode_workspace_bytes(0, 4, 32, 64, 16, 0) == 0          # invalid shape
    assert lib.ap_decode_workspace_bytes(1, 40, 128, 64, 100, 2) == 0        # r % 64 != 0: unsupported


def test_argument_validation_without_gpu():
    """Host-checkable violations are rejected before any launch (NULL pointers here,
    so nothing could run anyway)."""
    lib = ctypes.CDLL(LIB)
    lib.ap_last_error.restype = ctypes.c_char_p
    vp = ctypes.c_void_p
    lib.ap_decode_attn.argtypes = ([vp] * 7 + [ctypes.c_int64] + [vp] * 4 + [ctypes.c_int] +
                                   [vp, vp, vp] + [ctypes.c_int] * 7 +
                                   [ctypes.c_float, ctypes.c_int, ctypes.c_int, ctypes.c_int, vp, ctypes.c_size_t, vp])
    st = lib.ap_decode_attn(None, None, None, None, None, None, None, 0, None, None, None, None, 0,
                            None, None, None, 1, 4, 4, 32, 64, 64, 16, 0.1, 0, 0, 0, None, 0, None)
    assert st == 1 and b"NULL" in lib.ap_last_error()
    gr = (ctypes.c_int32 * 2)(64, 128)                                     # increasing: invalid
    cn = (ctypes.c_int32 * 2)(1, 2)
    lib.ap_select_ranks.argtypes = [vp, ctypes.c_int, ctypes.c_int, ctypes.c_int, vp, vp,
                                    ctypes.c_int32, vp, vp, vp, vp, ctypes.c_size_t, vp]
    one = ctypes.c_void_p(16)                                               # never dereferenced
    st = lib.ap_select_ranks(one, 1, 8, 2, ctypes.cast(gr, vp), ctypes.cast(cn, vp), 2, one, one,
                             one, one, 1 << 20, None)
    assert st == 1 and b"non-increasing" in lib.ap_last_error()
    lib.ap_update_importance.argtypes = [vp, vp, vp] + [ctypes.c_int] * 4 + [ctypes.c_int64, ctypes.c_float, vp]
    assert lib.ap_update_importance(None, one, one, 1, 4, 8, 8, 8, 0.5, None) == 1
    assert lib.ap_update_importance(one, one, one, 1, 4, 9, 8, 9, 0.5, None) == 1     # T > T_cap
    assert lib.ap_update_importance(one, one, one, 1, 4, 8, 8, 8, 1.5, None) == 1     # alpha > 1
    assert b"alpha" in lib.ap_last_error()
