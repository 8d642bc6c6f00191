"""GPU parity: the uncompressed segment of the cache and the merge of segments under one softmax
(Alg. 1: decompressed tokens and uncompressed tokens are concatenated before the softmax),
against the fp64 oracle's definition by concatenation."""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2603_23914_amd import workloads as wl
from gpu_util import TORCH_DT, assert_close, to_dev, to_host64, workspace

pytestmark = pytest.mark.gpu


def raw_case(dtype, B, H, d, T_cap, seed):
    rng = wl.rng_for(seed, B, H, d, T_cap)
    q = wl.store(rng.standard_normal((B, H, d)), dtype)
    K = wl.store(rng.standard_normal((B, T_cap, H * d)), dtype)
    V = wl.store(rng.standard_normal((B, T_cap, H * d)), dtype)
    return q, K, V


def gpu_raw(dtype, q, K, V, T_u):
    from paper_2603_23914_amd import binding as ap
    B, H, d = q.shape
    dq, dK, dV = (to_dev(x, dtype) for x in (q, K, V))
    out = torch.full((B, H, d), float("nan"), dtype=torch.float32, device="cuda")
    lse = torch.full((B, H), float("nan"), dtype=torch.float32, device="cuda")
    ap.ap_raw_attn(dq, dK, dV, out, workspace(ap.ap_raw_workspace_bytes(B, H, d, T_u)), T_u=T_u,
                   sm_scale=1.0 / math.sqrt(d), lse=lse)
    torch.cuda.synchronize()
    return out, lse


@pytest.mark.parametrize("dtype,B,H,d,T_u,T_cap", [
    ("bf16", 2, 40, 128, 301, 320),      # several rounds and a ragged tail
    ("f16", 3, 8, 64, 97, 97),
    ("f16", 2, 5, 256, 70, 80),
    ("bf16", 2, 6, 32, 300, 300),
    ("f16", 1, 8, 128, 3000, 3000),      # one sequence: the tokens are split over workgroups
    ("bf16", 1, 40, 128, 1, 16),         # a single token
    ("f16", 2, 4, 128, 17, 32),          # fewer tokens than lane groups
])
def test_raw_attn_small(dtype, B, H, d, T_u, T_cap):
    q, K, V = raw_case(dtype, B, H, d, T_cap, 41)
    print(f"raw {dtype} B={B} H={H} d={d} T_u={T_u}", flush=True)
    out, lse = gpu_raw(dtype, q, K, V, T_u)
    P = lambda x: oracle.promote(x, dtype)
    for b in range(B):
        ref, ref_lse = oracle.raw_attn(P(q)[b], P(K)[b, :T_u], P(V)[b, :T_u], return_lse=True)
        assert_close(to_host64(out[b]), ref, dtype, f"raw attention b={b}")
        assert np.abs(to_host64(lse[b]) - ref_lse).max() <= 2e-3 * max(1.0, np.abs(ref_lse).max())


def test_raw_attn_empty_segment():
    q, K, V = raw_case("f16", 2, 8, 128, 8, 42)
    out, lse = gpu_raw("f16", q, K, V, 0)
    assert (out == 0).all().item() and torch.isneginf(lse).all().item()


@pytest.mark.parametrize("dtype,B,H,d,r,T,T_u,ragged", [
    ("bf16", 2, 40, 128, 640, 301, 45, False),
    ("f16", 2, 32, 128, 512, 333, 130, True),
    ("f16", 1, 8, 64, 128, 97, 1, False),
    ("bf16", 2, 24, 64, 192, 129, 0, False),      # empty uncompressed segment
])
def test_compressed_plus_uncompressed_under_one_softmax(dtype, B, H, d, r, T, T_u, ragged):
    from paper_2603_23914_amd import binding as ap
    case = wl.decode_case(dtype, B, H, d, r, T, steps=0, seed=43, append=False)
    q = wl.step_query(case, 0)
    _, K, V = raw_case(dtype, B, H, d, max(T_u, 1), 44)
    print(f"segments {dtype} B={B} H={H} r={r} T={T} T_u={T_u} ragged={ragged}", flush=True)
    dq, dCk, dCv, dBk, dBv, dK, dV = (to_dev(x, dtype) for x in (q, case.Ck, case.Cv, case.Bk, case.Bv, K, V))
    kw, rank_np = {}, None
    if ragged:
        granks, cum, den = (r, r // 2, 64), (1, 3, 8), 8
        mass = torch.from_numpy(wl.rng_for(45).random((B, T)).astype(np.float32)).cuda()
        rank = torch.empty((B, T), dtype=torch.int32, device="cuda")
        off = torch.empty((B, 4), dtype=torch.int32, device="cuda")
        idx = torch.empty((B, T), dtype=torch.int32, device="cuda")
        ap.ap_select_ranks(mass, granks, cum, den, rank, off, idx, workspace(ap.ap_select_workspace_bytes(B, T, 3)))
        kw = dict(rank_k=rank, rank_v=rank, bucket_off=off, bucket_idx=idx, F=3)
        torch.cuda.synchronize()
        rank_np = rank.cpu().numpy()
    out_c = torch.empty((B, H, d), dtype=torch.float32, device="cuda")
    lse_c = torch.empty((B, H), dtype=torch.float32, device="cuda")
    ap.ap_decode_attn(dq, dCk, dCv, dBk, dBv, out_c, workspace(ap.ap_decode_workspace_bytes(B, H, d, T, r, ap._DT[TORCH_DT[dtype]])),
                      T=T, sm_scale=1.0 / math.sqrt(d), lse=lse_c, **kw)
    out_u = torch.empty_like(out_c)
    lse_u = torch.empty_like(lse_c)
    ap.ap_raw_attn(dq, dK, dV, out_u, workspace(ap.ap_raw_workspace_bytes(B, H, d, T_u)), T_u=T_u,
                   sm_scale=1.0 / math.sqrt(d), lse=lse_u)
    out = torch.empty((B, H, d), dtype=torch.float32, device="cuda")
    lse = torch.empty((B, H), dtype=torch.float32, device="cuda")
    ap.ap_merge_segments(out_c, lse_c, out_u, lse_u, out, lse=lse)
    out16 = torch.empty((B, H, d), dtype=TORCH_DT[dtype], device="cuda")
    ap.ap_merge_segments(out_c, lse_c, out_u, lse_u, out16)
    ap.ap_merge_segments(out_c, lse_c, out_u, lse_u, out_c)                      # in place
    torch.cuda.synchronize()
    assert torch.equal(out, out_c)
    # the 16-bit output is the fp32 result rounded once, to nearest even
    assert torch.equal(out16.view(torch.int16), out.to(TORCH_DT[dtype]).view(torch.int16))
    P = lambda x: oracle.promote(x, dtype)
    for b in range(B):
        segs = [dict(Ck=P(case.Ck)[b, :T], Cv=P(case.Cv)[b, :T], Bk=P(case.Bk)[b], Bv=P(case.Bv)[b],
                     rank_k=None if rank_np is None else rank_np[b], rank_v=None if rank_np is None else rank_np[b]),
                dict(K=P(K)[b, :T_u], V=P(V)[b, :T_u])]
        ref, ref_lse = oracle.decode_attn_segments(P(q)[b], segs, return_lse=True)
        assert_close(to_host64(out[b]), ref, dtype, f"two segments b={b}")
        assert np.abs(to_host64(lse[b]) - ref_lse).max() <= 2e-3 * max(1.0, np.abs(ref_lse).max())
        # the 16-bit output is the fp32 one rounded once
        assert np.abs(to_host64(out16[b]) - to_host64(out[b])).max() <= 2.0 ** -8 * np.abs(ref).max()


def test_decode_loop_with_uncompressed_tail():
    """Alg. 1's loop: the prompt's cache is compressed, every generated token's key and value
    go to the uncompressed segment as they are, and each step attends to both."""
    from paper_2603_23914_amd import binding as ap
    dtype, B, H, d, r, T, steps = "bf16", 2, 40, 128, 640, 200, 5
    case = wl.decode_case(dtype, B, H, d, r, T, steps=steps, seed=46, append=False)
    P = lambda x: oracle.promote(x, dtype)
    dCk, dCv, dBk, dBv = (to_dev(x, dtype) for x in (case.Ck, case.Cv, case.Bk, case.Bv))
    tail_cap = 8
    dK = torch.zeros((B, tail_cap, H * d), dtype=TORCH_DT[dtype], device="cuda")
    dV = torch.zeros_like(dK)
    K_h = np.zeros((B, 0, H * d))
    V_h = np.zeros((B, 0, H * d))
    ws_c = workspace(ap.ap_decode_workspace_bytes(B, H, d, T, r, ap._DT[TORCH_DT[dtype]]))
    out_c = torch.empty((B, H, d), dtype=torch.float32, device="cuda")
    lse_c = torch.empty((B, H), dtype=torch.float32, device="cuda")
    out_u, lse_u = torch.empty_like(out_c), torch.empty_like(lse_c)
    out = torch.empty_like(out_c)
    for step in range(steps):
        kn, vn = wl.step_new_token(case, step, P(case.Bk), P(case.Bv))
        q = wl.step_query(case, step)
        print(f"tail loop step {step}", flush=True)
        dq, dkn, dvn = (to_dev(x, dtype) for x in (q, kn, vn))
        ap.ap_raw_append(dkn, dvn, dK, dV, row=step)
        T_u = step + 1
        ap.ap_decode_attn(dq, dCk, dCv, dBk, dBv, out_c, ws_c, T=T, sm_scale=1.0 / math.sqrt(d), lse=lse_c)
        ap.ap_raw_attn(dq, dK, dV, out_u, workspace(ap.ap_raw_workspace_bytes(B, H, d, T_u)), T_u=T_u,
                       sm_scale=1.0 / math.sqrt(d), lse=lse_u)
        ap.ap_merge_segments(out_c, lse_c, out_u, lse_u, out)
        torch.cuda.synchronize()
        K_h = np.concatenate([K_h, P(kn)[:, None, :]], axis=1)
        V_h = np.concatenate([V_h, P(vn)[:, None, :]], axis=1)
        for b in range(B):
            ref = oracle.decode_attn_segments(P(q)[b], [
                dict(Ck=P(case.Ck)[b, :T], Cv=P(case.Cv)[b, :T], Bk=P(case.Bk)[b], Bv=P(case.Bv)[b]),
                dict(K=K_h[b], V=V_h[b])])
            assert_close(to_host64(out[b]), ref, dtype, f"step {step} b={b}")
    assert torch.equal(dK[:, :steps].cpu(), torch.stack([to_dev(wl.step_new_token(case, s, P(case.Bk), P(case.Bv))[0], dtype).cpu() for s in range(steps)], dim=1))


def test_tail_joins_the_compressed_cache_every_tp_steps():
    """Alg. 1's periodic step with the bases kept: generated tokens wait in the uncompressed
    segment; once T_p of them are there they are projected onto the sequence's bases in one
    ap_compact call (rows appended to the coefficient cache) and the segment starts over.  The
    oracle keeps the same three things: the coefficient rows the GPU holds (read back bit for bit
    after every compaction), the raw tail, and the definition of attention over their union."""
    from paper_2603_23914_amd import binding as ap
    dtype, B, H, d, r, T0, T_p, steps = "f16", 2, 16, 64, 128, 150, 3, 8
    case = wl.decode_case(dtype, B, H, d, r, T0, steps=steps, seed=47, append=True)
    P = lambda x: oracle.promote(x, dtype)
    dCk, dCv, dBk, dBv = (to_dev(x, dtype) for x in (case.Ck, case.Cv, case.Bk, case.Bv))
    dK = torch.zeros((B, T_p, H * d), dtype=TORCH_DT[dtype], device="cuda")
    dV = torch.zeros_like(dK)
    out_c = torch.empty((B, H, d), dtype=torch.float32, device="cuda")
    lse_c = torch.empty((B, H), dtype=torch.float32, device="cuda")
    out_u, lse_u, out = torch.empty_like(out_c), torch.empty_like(lse_c), torch.empty_like(out_c)
    scale = 1.0 / math.sqrt(d)
    T, T_u = T0, 0                      # rows in the compressed cache, rows in the tail
    tail_k, tail_v = [], []
    compactions = 0
    for step in range(steps):
        kn, vn = wl.step_new_token(case, step, P(case.Bk), P(case.Bv))
        q = wl.step_query(case, step)
        dq, dkn, dvn = (to_dev(x, dtype) for x in (q, kn, vn))
        ap.ap_raw_append(dkn, dvn, dK, dV, row=T_u)
        T_u += 1
        tail_k.append(P(kn))
        tail_v.append(P(vn))
        print(f"T_p loop step {step}: {T} compressed + {T_u} raw tokens", flush=True)
        ap.ap_decode_attn(dq, dCk, dCv, dBk, dBv, out_c, workspace(ap.ap_decode_workspace_bytes(B, H, d, T, r, ap.AP_F16)),
                          T=T, sm_scale=scale, lse=lse_c)
        ap.ap_raw_attn(dq, dK, dV, out_u, workspace(ap.ap_raw_workspace_bytes(B, H, d, T_u)), T_u=T_u, sm_scale=scale,
                       lse=lse_u)
        ap.ap_merge_segments(out_c, lse_c, out_u, lse_u, out)
        torch.cuda.synchronize()
        Ck_h, Cv_h = P(dCk.cpu().numpy()), P(dCv.cpu().numpy())
        for b in range(B):
            ref = oracle.decode_attn_segments(P(q)[b], [
                dict(Ck=Ck_h[b, :T], Cv=Cv_h[b, :T], Bk=P(case.Bk)[b], Bv=P(case.Bv)[b]),
                dict(K=np.stack([k[b] for k in tail_k]), V=np.stack([v[b] for v in tail_v]))])
            assert_close(to_host64(out[b]), ref, dtype, f"step {step} b={b}")
        if T_u == T_p:                  # the trigger: the tail joins the compressed cache
            ap.ap_compact(dK, dV, dBk, dBv, dCk, dCv, n=T_p, row0=T)
            torch.cuda.synchronize()
            c_ref = oracle.compact(np.stack([k[0] for k in tail_k]), P(case.Bk)[0])
            got = P(dCk.cpu().numpy())[0, T:T + T_p]
            assert np.abs(got - c_ref).max() <= 2.0 ** -10 * np.abs(c_ref).max() + 1e-6
            T += T_p
            T_u = 0
            tail_k, tail_v = [], []
            compactions += 1
    assert compactions == 2 and T == T0 + 6 and T_u == 2
