"""ctypes binding of libattnpack.so: argument marshalling only.

Every function has the name and the argument order of the C entry point it
calls (see include/attnpack.h); tensors are torch tensors on the GPU whose
data_ptr() is passed through.  No step of the computation happens in Python,
and there is no CPU fallback: if the shared library is missing, importing this
module raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libattnpack.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} not found: build it with `python -m paper_2603_23914_amd.build` "
        "(there is no fallback implementation)")

_lib = ctypes.CDLL(LIB_PATH)

AP_OK, AP_ERR_INVALID_ARG, AP_ERR_UNSUPPORTED, AP_ERR_WORKSPACE, AP_ERR_HIP = range(5)
AP_F32, AP_F16, AP_BF16, AP_I8, AP_I4 = range(5)
AP_QBLOCK = 64

_c = ctypes
_vp, _i, _i64, _sz, _f = _c.c_void_p, _c.c_int, _c.c_int64, _c.c_size_t, _c.c_float

_lib.ap_compact.restype = _i
_lib.ap_compact.argtypes = [_vp] * 8 + [_i] * 6 + [_i64, _i, _i, _vp]
_lib.ap_bases_workspace_bytes.restype = _sz
_lib.ap_bases_workspace_bytes.argtypes = [_i] * 5
_lib.ap_compute_bases.restype = _i
_lib.ap_compute_bases.argtypes = [_vp, _vp, _i64, _vp, _vp] + [_i] * 7 + [_vp, _sz, _vp]
_lib.ap_decompress_workspace_bytes.restype = _sz
_lib.ap_decompress_workspace_bytes.argtypes = [_i] * 5
_lib.ap_decompress.restype = _i
_lib.ap_decompress.argtypes = [_vp, _vp, _i64, _vp, _vp] + [_i] * 6 + [_vp, _sz, _vp]
_lib.ap_quantize_i8.restype = _i
_lib.ap_quantize_i8.argtypes = [_vp, _vp, _vp, _i, _i, _i, _i, _vp]
_lib.ap_quantize_i4.restype = _i
_lib.ap_quantize_i4.argtypes = [_vp, _vp, _vp, _i, _i, _i, _i, _vp]
_lib.ap_select_ranks.restype = _i
_lib.ap_select_ranks.argtypes = [_vp, _i, _i, _i, _vp, _vp, _c.c_int32, _vp, _vp, _vp, _vp, _sz, _vp]
_lib.ap_select_workspace_bytes.restype = _sz
_lib.ap_select_workspace_bytes.argtypes = [_i, _i, _i]
_lib.ap_decode_attn.restype = _i
_lib.ap_decode_attn.argtypes = ([_vp] * 7 + [_i64] + [_vp] * 4 + [_i] + [_vp, _vp, _vp] + [_i] * 7 +
                                [_f, _i, _i, _i, _vp, _sz, _vp])
_lib.ap_decode_attn_static.restype = _i
_lib.ap_decode_attn_static.argtypes = ([_vp] * 7 + [_i64] + [_vp] * 4 + [_i] + [_vp, _vp, _vp] + [_i] * 7 +
                                       [_f, _i, _i, _i, _vp])
_lib.ap_decode_step.restype = _i
_lib.ap_decode_step.argtypes = ([_vp] * 7 + [_i64] + [_vp] * 4 + [_i] + [_vp, _vp, _vp] + [_i] * 7 +
                                [_f, _i, _i, _vp, _sz, _vp])
_lib.ap_update_importance.restype = _i
_lib.ap_update_importance.argtypes = [_vp, _vp, _vp, _i, _i, _i, _i, _i64, _f, _vp]
_lib.ap_raw_workspace_bytes.restype = _sz
_lib.ap_raw_workspace_bytes.argtypes = [_i] * 4
_lib.ap_raw_attn.restype = _i
_lib.ap_raw_attn.argtypes = [_vp] * 5 + [_i] * 6 + [_f, _i, _vp, _sz, _vp]
_lib.ap_merge_segments.restype = _i
_lib.ap_merge_segments.argtypes = [_vp] * 6 + [_i] * 4 + [_vp]
_lib.ap_keyonly_workspace_bytes.restype = _sz
_lib.ap_keyonly_workspace_bytes.argtypes = [_i] * 6
_lib.ap_keyonly_attn.restype = _i
_lib.ap_keyonly_attn.argtypes = [_vp] * 3 + [_c.c_int64] + [_vp] * 3 + [_i] * 7 + [_f, _i, _vp, _sz, _vp]
_lib.ap_valueonly_workspace_bytes.restype = _sz
_lib.ap_valueonly_workspace_bytes.argtypes = [_i] * 6
_lib.ap_valueonly_attn.restype = _i
_lib.ap_valueonly_attn.argtypes = [_vp] * 4 + [_c.c_int64] + [_vp] * 2 + [_i] * 7 + [_f, _i, _vp, _sz, _vp]
_lib.ap_raw_append.restype = _i
_lib.ap_raw_append.argtypes = [_vp] * 4 + [_i] * 5 + [_vp]
_lib.ap_decode_workspace_bytes.restype = _sz
_lib.ap_decode_workspace_bytes.argtypes = [_i] * 6
_lib.ap_status_string.restype = _c.c_char_p
_lib.ap_status_string.argtypes = [_i]
_lib.ap_last_error.restype = _c.c_char_p
_lib.ap_last_error.argtypes = []
_lib.ap_version.restype = _i
_lib.ap_version.argtypes = []
_lib.ap_probe_read_granule.restype = _sz
_lib.ap_probe_read_granule.argtypes = []
_lib.ap_probe_read.restype = _i
_lib.ap_probe_read.argtypes = [_vp, _sz, _vp, _vp]
_lib.ap_probe_read_stream.restype = _i
_lib.ap_probe_read_stream.argtypes = [_vp, _sz, _vp, _vp]
_lib.ap_prof_enable.restype = None
_lib.ap_prof_enable.argtypes = [_i]
_lib.ap_set_fused_value_min_bytes.restype = None
_lib.ap_set_fused_value_min_bytes.argtypes = [_c.c_int64]
_lib.ap_prof_read.restype = _i
_lib.ap_prof_read.argtypes = [_c.POINTER(_c.c_float), _c.POINTER(_c.c_int)]
_lib.ap_prof_read_launches.restype = _i
_lib.ap_prof_read_launches.argtypes = [_c.POINTER(_c.c_float), _i, _c.POINTER(_c.c_int)]

EXPORTS = ("ap_compact", "ap_bases_workspace_bytes", "ap_compute_bases", "ap_decompress_workspace_bytes",
           "ap_decompress", "ap_quantize_i4", "ap_quantize_i8", "ap_select_ranks", "ap_select_workspace_bytes",
           "ap_decode_attn", "ap_decode_attn_static", "ap_decode_step", "ap_update_importance", "ap_decode_workspace_bytes",
           "ap_raw_workspace_bytes", "ap_raw_attn", "ap_keyonly_workspace_bytes", "ap_keyonly_attn",
           "ap_valueonly_workspace_bytes", "ap_valueonly_attn", "ap_merge_segments", "ap_raw_append", "ap_status_string", "ap_last_error",
           "ap_version", "ap_set_fused_value_min_bytes", "ap_prof_enable", "ap_prof_read", "ap_prof_read_launches", "ap_probe_read_granule", "ap_probe_read", "ap_probe_read_stream")

# coefficient tensors: int8 = one code per byte, uint8 = 4-bit codes, two per byte
_DT = {torch.float32: AP_F32, torch.float16: AP_F16, torch.bfloat16: AP_BF16, torch.int8: AP_I8,
       torch.uint8: AP_I4}


class AttnPackError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"{_lib.ap_status_string(status).decode()}: {_lib.ap_last_error().decode()}")


def _check(status: int) -> None:
    if status != AP_OK:
        raise AttnPackError(status)


def _p(t: Optional[torch.Tensor]):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "tensors must be contiguous GPU tensors"
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def _bstride(Bm: torch.Tensor) -> int:
    return 0 if Bm.dim() == 2 else Bm.stride(0)


def ap_version() -> int:
    return _lib.ap_version()


def ap_status_string(status: int) -> str:
    return _lib.ap_status_string(status).decode()


def ap_last_error() -> str:
    return _lib.ap_last_error().decode()


def ap_decode_workspace_bytes(B: int, H: int, d: int, T: int, r: int, dt: int) -> int:
    return _lib.ap_decode_workspace_bytes(B, H, d, T, r, dt)


def ap_select_workspace_bytes(B: int, T: int, F: int) -> int:
    return _lib.ap_select_workspace_bytes(B, T, F)


def ap_compact(K, V, Bk, Bv, Ck, Cv, scale_k=None, scale_v=None, *, n: int, row0: int,
               stream=None) -> None:
    """K, V [B, n, HD] (either may be None); Bk, Bv [r, HD] or [B, r, HD];
    Ck, Cv [B, T_cap, r] (int8 => scale_k/scale_v [B, T_cap, r/64] fp16)."""
    X = K if K is not None else V
    Cx = Ck if K is not None else Cv
    Bx = Bk if K is not None else Bv
    B, HD = X.shape[0], X.shape[-1]
    T_cap, r = Cx.shape[1], Cx.shape[2]
    _check(_lib.ap_compact(_p(K), _p(V), _p(Bk), _p(Bv), _p(Ck), _p(Cv), _p(scale_k), _p(scale_v),
                           B, n, row0, T_cap, HD, r, _bstride(Bx), _DT[X.dtype], _DT[Cx.dtype],
                           _stream(stream)))


def ap_bases_workspace_bytes(B: int, n: int, HD: int, r: int, oversample: int) -> int:
    return _lib.ap_bases_workspace_bytes(B, n, HD, r, oversample)


def ap_compute_bases(X, Omega, Bm, workspace, *, power_iters: int = 2, sigma=None, stream=None) -> None:
    """X [B, n, HD]; Omega [l, HD] or [B, l, HD] start block (l = r + oversampling); Bm [B, r, HD] out;
    sigma [B, r] fp32 out (optional)."""
    B, n, HD = X.shape
    r = Bm.shape[1]
    l = Omega.shape[-2]
    _check(_lib.ap_compute_bases(_p(X), _p(Omega), 0 if Omega.dim() == 2 else Omega.stride(0), _p(Bm), _p(sigma),
                                 B, n, HD, r, l - r, int(power_iters), _DT[X.dtype], _p(workspace),
                                 workspace.numel() * workspace.element_size(), _stream(stream)))


def ap_decompress_workspace_bytes(B: int, T: int, HD: int, r: int, with_ranks: bool) -> int:
    return _lib.ap_decompress_workspace_bytes(B, T, HD, r, int(with_ranks))


def ap_decompress(C, Bm, X, workspace, *, T: int, rank=None, stream=None) -> None:
    """C [B, T_cap, r], Bm [r, HD] or [B, r, HD] -> X [B, T, HD] = C[:, :T, :rank] Bm[:rank]."""
    B, T_cap, r = C.shape
    HD = Bm.shape[-1]
    _check(_lib.ap_decompress(_p(C), _p(Bm), _bstride(Bm), _p(rank), _p(X), B, T, T_cap, HD, r, _DT[C.dtype],
                              _p(workspace), workspace.numel() * workspace.element_size(), _stream(stream)))


def ap_quantize_i8(C, codes, scales, *, T: int, stream=None) -> None:
    B, T_cap, r = C.shape
    _check(_lib.ap_quantize_i8(_p(C), _p(codes), _p(scales), B, T, T_cap, r, _stream(stream)))


def ap_quantize_i4(C, codes, scales, *, T: int, stream=None) -> None:
    """C [B, T_cap, r] fp16 -> codes [B, T_cap, r/2] uint8 (two 4-bit codes per byte), scales fp16."""
    B, T_cap, r = C.shape
    _check(_lib.ap_quantize_i4(_p(C), _p(codes), _p(scales), B, T, T_cap, r, _stream(stream)))


def ap_select_ranks(mass, group_rank, cum_num, den: int, rank_out, bucket_off, bucket_idx,
                    workspace, *, stream=None) -> None:
    """mass [B, T] fp32 (GPU); group_rank, cum_num: host sequences of ints."""
    B, T = mass.shape
    F = len(group_rank)
    gr = (_c.c_int32 * F)(*[int(x) for x in group_rank])
    cn = (_c.c_int32 * F)(*[int(x) for x in cum_num])
    _check(_lib.ap_select_ranks(_p(mass), B, T, F, _c.cast(gr, _vp), _c.cast(cn, _vp), int(den),
                                _p(rank_out), _p(bucket_off), _p(bucket_idx), _p(workspace),
                                workspace.numel() * workspace.element_size(), _stream(stream)))


def ap_decode_attn(q, Ck, Cv, Bk, Bv, out, workspace, *, T: int, sm_scale: float,
                   scale_k=None, scale_v=None, rank_k=None, rank_v=None, bucket_off=None,
                   bucket_idx=None, F: int = 0, lse=None, scores=None, stream=None) -> None:
    """q, out [B, H, d] (out in q's dtype or fp32); Ck, Cv [B, T_cap, r];
    Bk, Bv [r, H_kv*d] or [B, r, H_kv*d] (H_kv is read off their width);
    scores [B, T_cap, H] fp32 (optional output)."""
    B, H, d = q.shape
    T_cap, r = Ck.shape[1], Ck.shape[2] * (2 if Ck.dtype == torch.uint8 else 1)
    H_kv = Bk.shape[-1] // d
    _check(_lib.ap_decode_attn(_p(q), _p(Ck), _p(Cv), _p(scale_k), _p(scale_v), _p(Bk), _p(Bv),
                               _bstride(Bk), _p(rank_k), _p(rank_v), _p(bucket_off),
                               _p(bucket_idx), F, _p(out), _p(lse), _p(scores), B, H, H_kv, d, T, T_cap, r,
                               float(sm_scale), _DT[q.dtype], _DT[Ck.dtype], _DT[out.dtype],
                               _p(workspace),
                               workspace.numel() * workspace.element_size(), _stream(stream)))


AP_STATIC_SCRATCH_BYTES = 64 << 20


def ap_decode_attn_static(q, Ck, Cv, Bk, Bv, out, *, T: int, sm_scale: float,
                          scale_k=None, scale_v=None, rank_k=None, rank_v=None, bucket_off=None,
                          bucket_idx=None, F: int = 0, lse=None, scores=None, stream=None) -> None:
    """ap_decode_attn on the library's own scratch buffer (no workspace argument, no allocation)."""
    B, H, d = q.shape
    T_cap, r = Ck.shape[1], Ck.shape[2] * (2 if Ck.dtype == torch.uint8 else 1)
    H_kv = Bk.shape[-1] // d
    _check(_lib.ap_decode_attn_static(_p(q), _p(Ck), _p(Cv), _p(scale_k), _p(scale_v), _p(Bk), _p(Bv),
                                      _bstride(Bk), _p(rank_k), _p(rank_v), _p(bucket_off),
                                      _p(bucket_idx), F, _p(out), _p(lse), _p(scores), B, H, H_kv, d, T, T_cap,
                                      r, float(sm_scale), _DT[q.dtype], _DT[Ck.dtype], _DT[out.dtype],
                                      _stream(stream)))


def ap_decode_step(q, k_new, v_new, Ck, Cv, Bk, Bv, out, workspace, *, T: int, sm_scale: float,
                   rank_k=None, rank_v=None, bucket_off=None, bucket_idx=None, F: int = 0,
                   lse=None, scores=None, stream=None) -> None:
    """Append k_new, v_new [B, H_kv*d] at row T-1, then attend over T rows (one fused call)."""
    B, H, d = q.shape
    T_cap, r = Ck.shape[1], Ck.shape[2]
    H_kv = Bk.shape[-1] // d
    _check(_lib.ap_decode_step(_p(q), _p(k_new), _p(v_new), _p(Ck), _p(Cv), _p(Bk), _p(Bv),
                               _bstride(Bk), _p(rank_k), _p(rank_v), _p(bucket_off),
                               _p(bucket_idx), F, _p(out), _p(lse), _p(scores), B, H, H_kv, d, T, T_cap, r,
                               float(sm_scale), _DT[q.dtype], _DT[out.dtype], _p(workspace),
                               workspace.numel() * workspace.element_size(), _stream(stream)))


def ap_update_importance(scores, lse, mass, *, T: int, alpha: float, stream=None) -> None:
    """mass [B, >=T] fp32 <- alpha*mass + (1-alpha)*mean_h exp(scores - lse) (Eq. 1, one query);
    scores [B, T_cap, H] as the decode entry points write them."""
    B, T_cap, H = scores.shape
    _check(_lib.ap_update_importance(_p(scores), _p(lse), _p(mass), B, H, T, T_cap, mass.stride(0),
                                     float(alpha), _stream(stream)))


def ap_raw_workspace_bytes(B: int, H: int, d: int, T_u: int) -> int:
    return _lib.ap_raw_workspace_bytes(B, H, d, T_u)


def ap_raw_attn(q, K, V, out, workspace, *, T_u: int, sm_scale: float, lse=None, stream=None) -> None:
    """q [B, H, d]; K, V [B, T_u_cap, H_kv*d] (same 16-bit dtype); out [B, H, d] fp32."""
    B, H, d = q.shape
    _check(_lib.ap_raw_attn(_p(q), _p(K), _p(V), _p(out), _p(lse), B, H, K.shape[2] // d, d, T_u, K.shape[1],
                            float(sm_scale), _DT[q.dtype], _p(workspace),
                            workspace.numel() * workspace.element_size(), _stream(stream)))


def ap_keyonly_workspace_bytes(B: int, H: int, H_kv: int, d: int, T: int, r: int) -> int:
    return _lib.ap_keyonly_workspace_bytes(B, H, H_kv, d, T, r)


def ap_keyonly_attn(q, Ck, Bk, V, out, workspace, *, T: int, sm_scale: float, lse=None, stream=None) -> None:
    """Compressed keys, raw values.  q [B, H, d]; Ck [B, T_cap, r]; Bk [r, H_kv*d] or
    [B, r, H_kv*d]; V [B, T_cap, H_kv*d]; out [B, H, d] fp32."""
    B, H, d = q.shape
    r = Ck.shape[2]
    _check(_lib.ap_keyonly_attn(_p(q), _p(Ck), _p(Bk), _bstride(Bk), _p(V), _p(out), _p(lse), B, H, V.shape[2] // d, d,
                                T, Ck.shape[1], r, float(sm_scale), _DT[q.dtype], _p(workspace),
                                workspace.numel() * workspace.element_size(), _stream(stream)))


def ap_valueonly_workspace_bytes(B: int, H: int, H_kv: int, d: int, T: int, r: int) -> int:
    return _lib.ap_valueonly_workspace_bytes(B, H, H_kv, d, T, r)


def ap_valueonly_attn(q, K, Cv, Bv, out, workspace, *, T: int, sm_scale: float, lse=None, stream=None) -> None:
    """Raw keys, compressed values.  q [B, H, d]; K [B, T_cap, H_kv*d]; Cv [B, T_cap, r];
    Bv [r, H_kv*d] or [B, r, H_kv*d]; out [B, H, d] fp32."""
    B, H, d = q.shape
    _check(_lib.ap_valueonly_attn(_p(q), _p(K), _p(Cv), _p(Bv), _bstride(Bv), _p(out), _p(lse), B, H,
                                  K.shape[2] // d, d, T, K.shape[1], Cv.shape[2], float(sm_scale), _DT[q.dtype],
                                  _p(workspace), workspace.numel() * workspace.element_size(), _stream(stream)))


def ap_merge_segments(out_a, lse_a, out_b, lse_b, out, *, lse=None, stream=None) -> None:
    """out_a, out_b [B, H, d] fp32 with lse_a, lse_b [B, H] -> out (any supported dtype)."""
    B, H, d = out_a.shape
    _check(_lib.ap_merge_segments(_p(out_a), _p(lse_a), _p(out_b), _p(lse_b), _p(out), _p(lse), B, H, d,
                                  _DT[out.dtype], _stream(stream)))


def ap_raw_append(k_new, v_new, K, V, *, row: int, stream=None) -> None:
    """k_new, v_new [B, HD] -> row `row` of K, V [B, T_u_cap, HD]."""
    X = K if K is not None else V
    B, T_cap, HD = X.shape
    _check(_lib.ap_raw_append(_p(k_new), _p(v_new), _p(K), _p(V), B, HD, row, T_cap, _DT[X.dtype],
                              _stream(stream)))


def ap_probe_read_granule() -> int:
    return _lib.ap_probe_read_granule()


def ap_probe_read(src, nbytes: int, sink, *, stream=None) -> None:
    """Plain streaming read of the first nbytes of src (measurement aid); sink: 8192 int32."""
    _check(_lib.ap_probe_read(_p(src), nbytes, _p(sink), _stream(stream)))


def ap_probe_read_stream(src, nbytes: int, sink, *, stream=None) -> None:
    """Plain streaming read of the first nbytes of src (measurement aid); sink: 8192 int32."""
    _check(_lib.ap_probe_read_stream(_p(src), nbytes, _p(sink), _stream(stream)))


def ap_set_fused_value_min_bytes(min_bytes: int) -> None:
    """Fused steps produce the new value row inside the expansion pass when the value bases
    streamed per step are at least min_bytes; negative: the library's own rule."""
    _lib.ap_set_fused_value_min_bytes(int(min_bytes))


def ap_prof_enable(on) -> None:
    """False / 0: off; True / 1: time every launch; n > 1: every n-th launch."""
    _lib.ap_prof_enable(int(on))


def ap_prof_read():
    """-> (summed milliseconds of the coefficient-streaming kernel, launches recorded)."""
    ms, cnt = _c.c_float(0), _c.c_int(0)
    _check(_lib.ap_prof_read(_c.byref(ms), _c.byref(cnt)))
    return ms.value, cnt.value


def ap_prof_read_launches(cap: int = 4096):
    """-> list of the timed launches' kernel times in microseconds, in launch order."""
    buf, cnt = (_c.c_float * cap)(), _c.c_int(0)
    _check(_lib.ap_prof_read_launches(buf, cap, _c.byref(cnt)))
    return [buf[i] for i in range(min(cnt.value, cap))]


def raw():
    """The ctypes library handle (tests use it to exercise error paths)."""
    return _lib
