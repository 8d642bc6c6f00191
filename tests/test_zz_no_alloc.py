"""GPU: the allocation-free decode entry point (ap_decode_attn_static: the decode workspace is a
device array of the library) against ap_decode_attn on a caller's workspace, two calls in a row,
the second on a smaller input, and both against the fp64 oracle."""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2603_23914_amd import workloads as wl
from gpu_util import TORCH_DT, assert_close, to_dev, to_host64, workspace

pytestmark = pytest.mark.gpu


def _both_ways(dtype, B, H, d, r, T, seed, ragged=False):
    from paper_2603_23914_amd import binding as ap
    case = wl.decode_case(dtype, B, H, d, r, T, steps=0, seed=seed, append=False)
    q = wl.step_query(case, 0)
    dq, dCk, dCv, dBk, dBv = (to_dev(x, dtype) for x in (q, case.Ck, case.Cv, case.Bk, case.Bv))
    kw = {}
    rk = None
    if ragged:
        mass = torch.rand(B, T, device="cuda")
        rank = torch.empty(B, T, dtype=torch.int32, device="cuda")
        off = torch.empty(B, 3, dtype=torch.int32, device="cuda")
        idx = torch.empty(B, T, dtype=torch.int32, device="cuda")
        ap.ap_select_ranks(mass, (r, 64), (1, 3), 3, rank, off, idx, workspace(ap.ap_select_workspace_bytes(B, T, 2)))
        kw = dict(rank_k=rank, rank_v=rank, bucket_off=off, bucket_idx=idx, F=2)
        rk = rank.cpu().numpy()
    out_ws = torch.empty((B, H, d), dtype=torch.float32, device="cuda")
    out_st = torch.full((B, H, d), float("nan"), dtype=torch.float32, device="cuda")
    lse_ws = torch.empty((B, H), dtype=torch.float32, device="cuda")
    lse_st = torch.full((B, H), float("nan"), dtype=torch.float32, device="cuda")
    scale = 1.0 / math.sqrt(d)
    ws = workspace(ap.ap_decode_workspace_bytes(B, H, d, T, r, ap._DT[TORCH_DT[dtype]]))
    print(f"static vs workspace: {dtype} B={B} H={H} d={d} r={r} T={T} ragged={ragged}", flush=True)
    ap.ap_decode_attn(dq, dCk, dCv, dBk, dBv, out_ws, ws, T=T, sm_scale=scale, lse=lse_ws, **kw)
    ap.ap_decode_attn_static(dq, dCk, dCv, dBk, dBv, out_st, T=T, sm_scale=scale, lse=lse_st, **kw)
    torch.cuda.synchronize()
    # same kernels, same layout of the scratch: the two agree bit for bit
    assert torch.equal(out_ws, out_st)
    assert torch.equal(lse_ws, lse_st)
    P = lambda x: oracle.promote(x, dtype)
    ref = oracle.decode_attn_batched(P(q), P(case.Ck), P(case.Cv), P(case.Bk), P(case.Bv), T,
                                     rank_k=rk, rank_v=rk, absorbed=True)
    assert_close(to_host64(out_st), ref, dtype, "ap_decode_attn_static")


def test_static_scratch_two_calls_second_smaller():
    _both_ways("bf16", 8, 40, 128, 640, 1500, seed=31)            # 32 splits, merged by their own kernel
    _both_ways("f16", 3, 16, 64, 128, 333, seed=32)               # smaller: the small-rank kernel
    _both_ways("f16", 2, 32, 128, 512, 700, seed=33, ragged=True)  # per-token ranks
    _both_ways("f32", 1, 4, 32, 16, 64, seed=34)                  # the fp32 kernels use the same buffer


def test_static_scratch_rejects_what_does_not_fit():
    from paper_2603_23914_amd import binding as ap
    B, H, d, r, T = 64, 64, 128, 640, 200000
    assert ap.ap_decode_workspace_bytes(B, H, d, T, r, ap.AP_BF16) > ap.AP_STATIC_SCRATCH_BYTES
    t = torch.zeros(16, dtype=torch.bfloat16, device="cuda")      # never read: the call is refused first
    lib = ap.raw()
    st = lib.ap_decode_attn_static(t.data_ptr(), t.data_ptr(), t.data_ptr(), None, None, t.data_ptr(),
                                   t.data_ptr(), 0, None, None, None, None, 0, t.data_ptr(), None, None,
                                   B, H, H, d, T, T, r, 0.1, ap.AP_BF16, ap.AP_BF16, ap.AP_F32, None)
    assert st == ap.AP_ERR_WORKSPACE
    assert "scratch" in ap.ap_last_error()
    # the five benchmark shapes fit
    for (b, h, t_, r_, dt) in ((1, 4, 64, 16, ap.AP_F32), (8, 32, 1216, 512, ap.AP_F16), (64, 40, 4288, 640, ap.AP_BF16),
                               (1, 32, 32768, 512, ap.AP_F16), (16, 32, 4224, 512, ap.AP_F16)):
        dd = 32 if dt == ap.AP_F32 else 128
        assert 0 < ap.ap_decode_workspace_bytes(b, h, dd, t_, r_, dt) <= ap.AP_STATIC_SCRATCH_BYTES
