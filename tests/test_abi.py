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


def test_validation_of_the_later_entry_points_without_gpu():
    """Shape and size rules of the compression step, the allocation-free decode entry and the
    group selection's workspace are checked on the host, before anything touches the GPU."""
    lib = ctypes.CDLL(LIB)
    lib.ap_last_error.restype = ctypes.c_char_p
    vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_size_t
    one = ctypes.c_void_p(4096)                                             # aligned, never dereferenced
    # compression step: hidden width must be a multiple of 64, the sketch no wider than the rows are many
    lib.ap_compute_bases.argtypes = [vp, vp, i64, vp, vp] + [i32] * 7 + [vp, sz, vp]
    st = lib.ap_compute_bases(one, one, 0, one, None, 1, 512, 500, 64, 32, 2, 1, one, 1 << 30, None)
    assert st != 0 and b"HD % 64" in lib.ap_last_error()
    st = lib.ap_compute_bases(one, one, 0, one, None, 1, 64, 512, 64, 32, 2, 1, one, 1 << 30, None)
    assert st != 0 and b"l <= n" in lib.ap_last_error()
    lib.ap_bases_workspace_bytes.restype = sz
    need = lib.ap_bases_workspace_bytes(1, 512, 512, 64, 32)
    assert need > 0
    st = lib.ap_compute_bases(one, one, 0, one, None, 1, 512, 512, 64, 32, 2, 1, one, need - 1, None)
    assert st == 3 and b"workspace" in lib.ap_last_error()
    # allocation-free decode: a shape whose scratch exceeds the static buffer is refused with its size
    lib.ap_decode_workspace_bytes.restype = sz
    assert lib.ap_decode_workspace_bytes(64, 64, 128, 4352, 640, 2) > (64 << 20)
    lib.ap_decode_attn_static.argtypes = ([vp] * 7 + [i64] + [vp] * 4 + [i32] + [vp, vp, vp] + [i32] * 7 +
                                          [ctypes.c_float, i32, i32, i32, vp])
    st = lib.ap_decode_attn_static(one, one, one, None, None, one, one, 0, None, None, None, None, 0,
                                   one, None, None, 64, 64, 64, 128, 4352, 4352, 640, 0.1, 2, 2, 0, None)
    assert st == 3 and b"scratch" in lib.ap_last_error()
    # group selection: few long rows are split over workgroups and need room to meet
    lib.ap_select_workspace_bytes.restype = sz
    short = lib.ap_select_workspace_bytes(64, 4224, 4)
    long_ = lib.ap_select_workspace_bytes(1, 32768, 4)
    assert short <= 4096 and long_ > 16 * 4096 * 4
    lib.ap_select_ranks.argtypes = [vp, i32, i32, i32, vp, vp, ctypes.c_int32, vp, vp, vp, vp, sz, vp]
    st = lib.ap_select_ranks(one, 1, 32768, 2, ctypes.cast((ctypes.c_int32 * 2)(128, 64), vp),
                             ctypes.cast((ctypes.c_int32 * 2)(1, 2), vp), 2, one, one, one, one, short, None)
    assert st == 3 and b"workspace" in lib.ap_last_error()
