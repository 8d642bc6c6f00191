"""GPU parity over a seeded sweep of shapes: head counts on both sides of every 16-head tile
boundary, all head widths, every rank class of the kernels (token-split up to 128, then 256 /
512 / 640), token counts around tile and split boundaries, uniform ranks, per-token ranks and
int8 coefficients, attend-only and fused step.  Each case is small enough for the fp64 oracle."""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2603_23914_amd import workloads as wl
from gpu_util import TORCH_DT, assert_close, to_dev, to_host64, workspace

pytestmark = pytest.mark.gpu


def sweep_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    while len(cases) < n:
        d = int(rng.choice([32, 64, 128, 256]))
        H = int(rng.integers(1, min(64, 8192 // d) + 1))
        r = 64 * int(rng.integers(1, 11))
        if r > H * d:
            continue                                    # a rank above the hidden size means nothing
        T = int(rng.choice([1, 2, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 257, 400, 513, 700]))
        B = int(rng.integers(1, 4))
        dtype = str(rng.choice(["f16", "bf16"]))
        mode = str(rng.choice(["attend", "step", "ragged", "int8"]))
        if mode == "int8":
            dtype = "f16"
        if mode == "step" and T < 2:
            T = 2
        cases.append((dtype, B, H, d, r, T, mode))
    return cases


@pytest.mark.parametrize("dtype,B,H,d,r,T,mode", sweep_cases(80, 2024))
def test_shape_sweep(dtype, B, H, d, r, T, mode):
    from paper_2603_23914_amd import binding as ap
    print(f"sweep {mode} {dtype} B={B} H={H} d={d} r={r} T={T}", flush=True)
    steps = 1 if mode == "step" else 0
    T0 = T - steps
    case = wl.decode_case(dtype, B, H, d, r, T0, steps=steps, seed=H * 131 + T, append=steps > 0)
    P = lambda x: oracle.promote(x, dtype)
    q = wl.step_query(case, 0)
    dq, dCk, dCv, dBk, dBv = (to_dev(x, dtype) for x in (q, case.Ck, case.Cv, case.Bk, case.Bv))
    out = torch.full((B, H, d), float("nan"), dtype=torch.float32, device="cuda")
    ws = workspace(ap.ap_decode_workspace_bytes(B, H, d, T, r, ap._DT[TORCH_DT[dtype]]))
    scale = 1.0 / math.sqrt(d)
    if mode == "attend":
        ap.ap_decode_attn(dq, dCk, dCv, dBk, dBv, out, ws, T=T, sm_scale=scale)
        torch.cuda.synchronize()
        ref = oracle.decode_attn_batched(P(q), P(case.Ck), P(case.Cv), P(case.Bk), P(case.Bv), T, absorbed=True)
    elif mode == "step":
        kn, vn = wl.step_new_token(case, 0, P(case.Bk), P(case.Bv))
        # every other case forces the new value row into the expansion pass (small cases would
        # otherwise all append it next to the key row)
        ap.ap_set_fused_value_min_bytes(0 if (H + T + r // 64) % 2 else -1)
        try:
            ap.ap_decode_step(dq, to_dev(kn, dtype), to_dev(vn, dtype), dCk, dCv, dBk, dBv, out, ws, T=T, sm_scale=scale)
            torch.cuda.synchronize()
        finally:
            ap.ap_set_fused_value_min_bytes(-1)
        bits = (lambda t: t.view(torch.int16).cpu().numpy().view(np.uint16)) if dtype == "bf16" else (lambda t: t.cpu().numpy())
        ref = oracle.decode_attn_batched(P(q), P(bits(dCk)), P(bits(dCv)), P(case.Bk), P(case.Bv), T, absorbed=True)
        c_ref = oracle.compact(P(kn)[0][None], P(case.Bk)[0])[0]
        tol = 2.0 ** -7 if dtype == "bf16" else 2.0 ** -10
        assert np.abs(P(bits(dCk))[0, T - 1] - c_ref).max() <= tol * np.abs(c_ref).max() + 1e-6
    elif mode == "ragged":
        granks = tuple(sorted({r, max(64, (r // 128) * 64), 64}, reverse=True))
        F = len(granks)
        cum = tuple(range(1, F + 1))
        mass = torch.from_numpy(wl.rng_for(T, r, H).random((B, T)).astype(np.float32)).cuda()
        rank = torch.empty((B, T), dtype=torch.int32, device="cuda")
        off = torch.empty((B, F + 1), dtype=torch.int32, device="cuda")
        idx = torch.empty((B, T), dtype=torch.int32, device="cuda")
        ap.ap_select_ranks(mass, granks, cum, F, rank, off, idx, workspace(ap.ap_select_workspace_bytes(B, T, F)))
        ap.ap_decode_attn(dq, dCk, dCv, dBk, dBv, out, ws, T=T, sm_scale=scale, rank_k=rank, rank_v=rank,
                          bucket_off=off, bucket_idx=idx, F=F)
        torch.cuda.synchronize()
        rk = rank.cpu().numpy()
        for b in range(B):
            r_ref, _, _ = oracle.select_ranks(mass[b].cpu().numpy(), granks, cum, F)
            assert (rk[b] == r_ref).all()
        ref = oracle.decode_attn_batched(P(q), P(case.Ck), P(case.Cv), P(case.Bk), P(case.Bv), T, rank_k=rk,
                                         rank_v=rk, absorbed=True)
    else:   # int8 coefficients
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
        ap.ap_decode_attn(dq, torch.from_numpy(Ck8).cuda(), torch.from_numpy(Cv8).cuda(), dBk, dBv, out, ws, T=T,
                          sm_scale=scale, scale_k=torch.from_numpy(sk).cuda(), scale_v=torch.from_numpy(sv).cuda())
        torch.cuda.synchronize()
        ref = oracle.decode_attn_batched(P(q), ck, cv, P(case.Bk), P(case.Bv), T, absorbed=True)
    assert_close(to_host64(out), ref, dtype, f"{mode} H={H} d={d} r={r} T={T}")


def one_sided_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    while len(cases) < n:
        d = int(rng.choice([32, 64, 128, 256]))
        Hkv = int(rng.integers(1, min(16, 4096 // d) + 1))
        G = int(rng.choice([1, 1, 2, 3, 4, 5, 8, 12]))          # query heads per key/value head
        r = 8 * int(rng.integers(1, 81))
        mode = str(rng.choice(["raw", "key-only", "value-only"]))
        if r > Hkv * d or (mode == "value-only" and d == 32 and r > 320):
            continue
        T = int(rng.choice([1, 2, 15, 16, 17, 63, 64, 65, 127, 129, 255, 257, 400, 513, 700, 1100]))
        B = int(rng.integers(1, 4))
        dtype = str(rng.choice(["f16", "bf16"]))
        cases.append((mode, dtype, B, Hkv * G, Hkv, d, r, T))
    return cases


@pytest.mark.parametrize("mode,dtype,B,H,Hkv,d,r,T", one_sided_cases(60, 2025))
def test_one_sided_shape_sweep(mode, dtype, B, H, Hkv, d, r, T):
    """The flash-decode entry points (uncompressed segment, key-only and value-only compression)
    over head groupings of every workgroup shape (1, 2, 4 and 8 heads per workgroup, with and
    without a partial last block), ranks that are any multiple of 8, token counts around the
    round and split boundaries."""
    from paper_2603_23914_amd import binding as ap
    print(f"sweep {mode} {dtype} B={B} H={H} Hkv={Hkv} d={d} r={r} T={T}", flush=True)
    case = wl.decode_case(dtype, B, Hkv, d, r, T, steps=0, seed=Hkv * 17 + T, append=False)
    rng = wl.rng_for(2025, H, T, r)
    q = wl.store(rng.standard_normal((B, H, d)), dtype)
    K = wl.store(rng.standard_normal((B, T, Hkv * d)), dtype)
    V = wl.store(rng.standard_normal((B, T, Hkv * d)), dtype)
    P = lambda x: oracle.promote(x, dtype)
    dq, dK, dV = (to_dev(x, dtype) for x in (q, K, V))
    out = torch.full((B, H, d), float("nan"), dtype=torch.float32, device="cuda")
    lse = torch.full((B, H), float("nan"), dtype=torch.float32, device="cuda")
    scale = 1.0 / math.sqrt(d)
    if mode == "raw":
        ap.ap_raw_attn(dq, dK, dV, out, workspace(ap.ap_raw_workspace_bytes(B, H, d, T)), T_u=T, sm_scale=scale, lse=lse)
        seg = lambda b: dict(K=P(K)[b], V=P(V)[b])
    elif mode == "key-only":
        ap.ap_keyonly_attn(dq, to_dev(case.Ck, dtype), to_dev(case.Bk, dtype), dV, out,
                           workspace(ap.ap_keyonly_workspace_bytes(B, H, Hkv, d, T, r)), T=T, sm_scale=scale, lse=lse)
        seg = lambda b: dict(Ck=P(case.Ck)[b], Bk=P(case.Bk)[b], V=P(V)[b])
    else:
        ap.ap_valueonly_attn(dq, dK, to_dev(case.Cv, dtype), to_dev(case.Bv, dtype), out,
                             workspace(ap.ap_valueonly_workspace_bytes(B, H, Hkv, d, T, r)), T=T, sm_scale=scale, lse=lse)
        seg = lambda b: dict(K=P(K)[b], Cv=P(case.Cv)[b], Bv=P(case.Bv)[b])
    torch.cuda.synchronize()
    for b in range(B):
        ref, ref_lse = oracle.decode_attn_segments(P(q)[b], [seg(b)], return_lse=True, kv_heads=Hkv)
        assert_close(to_host64(out[b]), ref, dtype, f"{mode} b={b}")
        assert np.abs(to_host64(lse[b]) - ref_lse).max() <= 2e-3 * max(1.0, np.abs(ref_lse).max())
