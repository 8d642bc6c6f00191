"""GPU parity: grouped-query attention (H query heads share H_kv key/value heads; the cache and
the bases have H_kv*d hidden columns) against the fp64 oracle, on every decode entry point."""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2603_23914_amd import workloads as wl
from gpu_util import TORCH_DT, assert_close, to_dev, to_host64, workspace

pytestmark = pytest.mark.gpu


def gqa_case(dtype, B, H, Hkv, d, r, T, steps, seed, append):
    """Cache and bases of Hkv*d hidden columns; queries for H heads."""
    case = wl.decode_case(dtype, B, Hkv, d, r, T, steps=steps, seed=seed, append=append)
    qs = [wl.store(wl.rng_for(seed, 77, s).standard_normal((B, H, d)), dtype) for s in range(max(steps, 1))]
    return case, qs


@pytest.mark.parametrize("dtype,B,H,Hkv,d,r,T", [
    ("bf16", 2, 32, 8, 128, 256, 301),      # Qwen3-VL-8B-like head layout
    ("f16", 2, 40, 10, 128, 512, 200),
    ("f16", 3, 16, 2, 64, 128, 97),
    ("bf16", 1, 8, 1, 128, 64, 130),        # multi-query: one key/value head
    ("f16", 1, 12, 4, 256, 192, 64),
    ("bf16", 2, 48, 16, 32, 128, 77),
])
def test_decode_attn_grouped_queries(dtype, B, H, Hkv, d, r, T):
    from paper_2603_23914_amd import binding as ap
    case, qs = gqa_case(dtype, B, H, Hkv, d, r, T, 0, 51, False)
    q = qs[0]
    print(f"gqa {dtype} B={B} H={H} Hkv={Hkv} d={d} r={r} T={T}", flush=True)
    dq, dCk, dCv, dBk, dBv = (to_dev(x, dtype) for x in (q, case.Ck, case.Cv, case.Bk, case.Bv))
    out = torch.empty((B, H, d), dtype=torch.float32, device="cuda")
    lse = torch.empty((B, H), dtype=torch.float32, device="cuda")
    ws = workspace(ap.ap_decode_workspace_bytes(B, H, d, T, r, ap._DT[TORCH_DT[dtype]]))
    ap.ap_decode_attn(dq, dCk, dCv, dBk, dBv, out, ws, T=T, sm_scale=1.0 / math.sqrt(d), lse=lse)
    torch.cuda.synchronize()
    P = lambda x: oracle.promote(x, dtype)
    ref = oracle.decode_attn_batched(P(q), P(case.Ck), P(case.Cv), P(case.Bk), P(case.Bv), T, absorbed=True,
                                     kv_heads=Hkv)
    assert_close(to_host64(out), ref, dtype, "grouped queries")
    ref_def, ref_lse = oracle.decode_attn(P(q)[0], P(case.Ck)[0, :T], P(case.Cv)[0, :T], P(case.Bk)[0],
                                          P(case.Bv)[0], return_lse=True, kv_heads=Hkv)
    assert np.abs(ref_def - ref[0]).max() < 1e-9
    assert np.abs(to_host64(lse[0]) - ref_lse).max() <= 2e-3 * max(1.0, np.abs(ref_lse).max())


def test_decode_attn_grouped_queries_fp32():
    from paper_2603_23914_amd import binding as ap
    B, H, Hkv, d, r, T = 2, 6, 2, 16, 24, 50
    rng = wl.rng_for(52)
    q = rng.standard_normal((B, H, d)).astype(np.float32)
    Ck = rng.standard_normal((B, T, r)).astype(np.float32)
    Cv = rng.standard_normal((B, T, r)).astype(np.float32)
    Bk = (rng.standard_normal((B, r, Hkv * d)) / math.sqrt(Hkv * d)).astype(np.float32)
    Bv = (rng.standard_normal((B, r, Hkv * d)) / math.sqrt(Hkv * d)).astype(np.float32)
    rank = rng.integers(0, r + 1, size=(B, T)).astype(np.int32)
    rank[:, 0] = r
    dq, dCk, dCv, dBk, dBv = (torch.from_numpy(x).cuda() for x in (q, Ck, Cv, Bk, Bv))
    dr = torch.from_numpy(rank).cuda()
    out = torch.empty((B, H, d), dtype=torch.float32, device="cuda")
    ws = workspace(ap.ap_decode_workspace_bytes(B, H, d, T, r, ap.AP_F32))
    ap.ap_decode_attn(dq, dCk, dCv, dBk, dBv, out, ws, T=T, sm_scale=1.0 / math.sqrt(d), rank_k=dr, rank_v=dr)
    torch.cuda.synchronize()
    ref = oracle.decode_attn_batched(q, Ck, Cv, Bk, Bv, T, rank_k=rank, rank_v=rank, kv_heads=Hkv)
    assert_close(to_host64(out), ref, "f32", "grouped queries fp32")


@pytest.mark.parametrize("dtype,B,H,Hkv,d,r,T0", [("bf16", 2, 32, 8, 128, 256, 150), ("f16", 2, 16, 4, 64, 128, 65)])
def test_decode_step_grouped_queries(dtype, B, H, Hkv, d, r, T0):
    """Append + attend in one call; the rows appended equal those of ap_compact bit for bit
    (both take the whole-row pass), the output matches the oracle on the stored bits."""
    from paper_2603_23914_amd import binding as ap
    steps = 3
    case, qs = gqa_case(dtype, B, H, Hkv, d, r, T0, steps, 53, True)
    P = lambda x: oracle.promote(x, dtype)
    dCk, dCv, dBk, dBv = (to_dev(x, dtype) for x in (case.Ck, case.Cv, case.Bk, case.Bv))
    dCk2, dCv2 = dCk.clone(), dCv.clone()
    out = torch.empty((B, H, d), dtype=torch.float32, device="cuda")
    for step in range(steps):
        T = T0 + step + 1
        kn, vn = wl.step_new_token(case, step, P(case.Bk), P(case.Bv))
        dq, dkn, dvn = (to_dev(x, dtype) for x in (qs[step], kn, vn))
        ws = workspace(ap.ap_decode_workspace_bytes(B, H, d, T, r, ap._DT[TORCH_DT[dtype]]))
        ap.ap_decode_step(dq, dkn, dvn, dCk, dCv, dBk, dBv, out, ws, T=T, sm_scale=1.0 / math.sqrt(d))
        ap.ap_compact(dkn[:, None, :].contiguous(), dvn[:, None, :].contiguous(), dBk, dBv, dCk2, dCv2, n=1, row0=T - 1)
        torch.cuda.synchronize()
        assert torch.equal(dCk.view(torch.int16), dCk2.view(torch.int16))
        assert torch.equal(dCv.view(torch.int16), dCv2.view(torch.int16))
        Ck_h = dCk.view(torch.int16).cpu().numpy().view(np.uint16) if dtype == "bf16" else dCk.cpu().numpy()
        Cv_h = dCv.view(torch.int16).cpu().numpy().view(np.uint16) if dtype == "bf16" else dCv.cpu().numpy()
        ref = oracle.decode_attn_batched(P(qs[step]), P(Ck_h), P(Cv_h), P(case.Bk), P(case.Bv), T, absorbed=True,
                                         kv_heads=Hkv)
        assert_close(to_host64(out), ref, dtype, f"grouped-query step {step}")
        c_ref = oracle.compact(P(kn)[0][None], P(case.Bk)[0])[0]
        assert np.abs(P(Ck_h)[0, T - 1] - c_ref).max() <= 2.0 ** -7 * np.abs(c_ref).max()


def test_ragged_ranks_grouped_queries():
    from paper_2603_23914_amd import binding as ap
    dtype, B, H, Hkv, d, r, T = "f16", 2, 32, 8, 128, 256, 333
    case, qs = gqa_case(dtype, B, H, Hkv, d, r, T, 0, 54, False)
    q = qs[0]
    granks, cum, den = (256, 128, 64), (1, 2, 4), 4
    mass = torch.from_numpy(wl.rng_for(54, 1).random((B, T)).astype(np.float32)).cuda()
    rank = torch.empty((B, T), dtype=torch.int32, device="cuda")
    off = torch.empty((B, 4), dtype=torch.int32, device="cuda")
    idx = torch.empty((B, T), dtype=torch.int32, device="cuda")
    ap.ap_select_ranks(mass, granks, cum, den, rank, off, idx, workspace(ap.ap_select_workspace_bytes(B, T, 3)))
    dq, dCk, dCv, dBk, dBv = (to_dev(x, dtype) for x in (q, case.Ck, case.Cv, case.Bk, case.Bv))
    out = torch.empty((B, H, d), dtype=torch.float32, device="cuda")
    ws = workspace(ap.ap_decode_workspace_bytes(B, H, d, T, r, ap.AP_F16))
    ap.ap_decode_attn(dq, dCk, dCv, dBk, dBv, out, ws, T=T, sm_scale=1.0 / math.sqrt(d), rank_k=rank,
                      rank_v=rank, bucket_off=off, bucket_idx=idx, F=3)
    torch.cuda.synchronize()
    P = lambda x: oracle.promote(x, dtype)
    rank_np = rank.cpu().numpy()
    ref = oracle.decode_attn_batched(P(q), P(case.Ck), P(case.Cv), P(case.Bk), P(case.Bv), T, rank_k=rank_np,
                                     rank_v=rank_np, absorbed=True, kv_heads=Hkv)
    assert_close(to_host64(out), ref, dtype, "ragged grouped queries")


@pytest.mark.parametrize("dtype,B,H,Hkv,d,T_u", [("bf16", 2, 32, 8, 128, 130), ("f16", 1, 8, 1, 64, 300)])
def test_raw_segment_grouped_queries(dtype, B, H, Hkv, d, T_u):
    from paper_2603_23914_amd import binding as ap
    rng = wl.rng_for(55, B, H, T_u)
    q = wl.store(rng.standard_normal((B, H, d)), dtype)
    K = wl.store(rng.standard_normal((B, T_u, Hkv * d)), dtype)
    V = wl.store(rng.standard_normal((B, T_u, Hkv * d)), dtype)
    dq, dK, dV = (to_dev(x, dtype) for x in (q, K, V))
    out = torch.empty((B, H, d), dtype=torch.float32, device="cuda")
    lse = torch.empty((B, H), dtype=torch.float32, device="cuda")
    ap.ap_raw_attn(dq, dK, dV, out, workspace(ap.ap_raw_workspace_bytes(B, H, d, T_u)), T_u=T_u,
                   sm_scale=1.0 / math.sqrt(d), lse=lse)
    torch.cuda.synchronize()
    P = lambda x: oracle.promote(x, dtype)
    for b in range(B):
        ref, ref_lse = oracle.raw_attn(P(q)[b], P(K)[b], P(V)[b], return_lse=True, kv_heads=Hkv)
        assert_close(to_host64(out[b]), ref, dtype, f"raw grouped queries b={b}")
        assert np.abs(to_host64(lse[b]) - ref_lse).max() <= 2e-3 * max(1.0, np.abs(ref_lse).max())


def test_int8_coefficients_grouped_queries():
    """int8 coefficients with grouped queries: the dequantising kernel sees folded queries and
    coefficient sums per query head only, the head map lives in the fold and the expansion."""
    from paper_2603_23914_amd import binding as ap
    dtype, B, H, Hkv, d, r, T = "f16", 2, 32, 8, 128, 256, 300
    case, qs = gqa_case(dtype, B, H, Hkv, d, r, T, 0, 56, False)
    q = qs[0]
    Ck8 = np.zeros(case.Ck.shape, np.int8)
    Cv8 = np.zeros(case.Cv.shape, np.int8)
    sk = np.zeros(case.Ck.shape[:2] + (r // 64,), np.float16)
    sv = np.zeros_like(sk)
    ck = np.zeros(case.Ck.shape)
    cv = np.zeros(case.Cv.shape)
    for b in range(B):
        Ck8[b, :T], sk[b, :T] = oracle.quantize_i8(case.Ck[b, :T])
        Cv8[b, :T], sv[b, :T] = oracle.quantize_i8(case.Cv[b, :T])
        ck[b, :T] = oracle.dequantize_i8(Ck8[b, :T], sk[b, :T])
        cv[b, :T] = oracle.dequantize_i8(Cv8[b, :T], sv[b, :T])
    dq, dBk, dBv = (to_dev(x, dtype) for x in (q, case.Bk, case.Bv))
    out = torch.empty((B, H, d), dtype=torch.float32, device="cuda")
    ws = workspace(ap.ap_decode_workspace_bytes(B, H, d, T, r, ap.AP_F16))
    ap.ap_decode_attn(dq, torch.from_numpy(Ck8).cuda(), torch.from_numpy(Cv8).cuda(), dBk, dBv, out, ws, T=T,
                      sm_scale=1.0 / math.sqrt(d), scale_k=torch.from_numpy(sk).cuda(),
                      scale_v=torch.from_numpy(sv).cuda())
    torch.cuda.synchronize()
    P = lambda x: oracle.promote(x, dtype)
    ref = oracle.decode_attn_batched(P(q), ck, cv, P(case.Bk), P(case.Bv), T, absorbed=True, kv_heads=Hkv)
    assert_close(to_host64(out), ref, dtype, "int8 grouped queries")
