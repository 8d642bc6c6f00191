"""GPU parity: key-only compression (compressed keys, raw values: the text-domain experiment of the
appendix "Analysis of Textual Token Compression" compresses keys only, R_k = 64) against the fp64 oracle's definition (rebuild the keys,
attend), alone, joined with an uncompressed tail, and over a decode loop that appends."""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2603_23914_amd import workloads as wl
from gpu_util import TORCH_DT, assert_close, to_dev, to_host64, workspace

pytestmark = pytest.mark.gpu


def keyonly_case(dtype, B, H, Hkv, d, r, T, seed, T_cap=None):
    """Key coefficients and bases in the law of the compressed-cache workloads (Hkv*d hidden
    columns), raw values N(0,1), queries for H heads."""
    T_cap = T if T_cap is None else T_cap
    case = wl.decode_case(dtype, B, Hkv, d, r, T, steps=T_cap - T, seed=seed, append=True)
    rng = wl.rng_for(seed, 88, T)
    q = wl.store(rng.standard_normal((B, H, d)), dtype)
    V = wl.store(rng.standard_normal((B, T_cap, Hkv * d)), dtype)
    return case, q, V


@pytest.mark.parametrize("dtype,B,H,Hkv,d,r,T", [
    ("bf16", 1, 32, 8, 128, 64, 1500),      # LLaMA-3.1-8B-like heads, R_k = 64
    ("f16", 2, 8, 8, 64, 128, 333),         # every head its own keys and values
    ("bf16", 2, 12, 4, 256, 320, 257),
    ("f16", 1, 40, 20, 32, 640, 70),        # the widest per-lane share of a coefficient row
    ("f16", 3, 16, 2, 64, 72, 129),         # a rank that is no multiple of 64
    ("bf16", 1, 8, 1, 128, 128, 64),        # one key/value head
    ("f16", 2, 40, 40, 128, 640, 200),
    ("bf16", 1, 6, 3, 64, 192, 1),          # a single token
    ("f16", 1, 64, 8, 128, 384, 2100),      # many splits
    # head width 128 with ranks up to 128 and at most 16 heads per group: the matrix-core kernel
    ("f16", 2, 32, 8, 128, 64, 257),        # a tile with a single token at the end
    ("bf16", 3, 16, 1, 128, 72, 95),        # 16 heads on one key/value head; rank no multiple of 32
    ("f16", 2, 10, 2, 128, 8, 33),          # five heads per group, one coefficient chunk
    ("bf16", 1, 24, 8, 128, 128, 5000),     # several splits, four rank steps
    ("f16", 4, 4, 4, 128, 96, 31),          # every head its own keys; less than one tile
    ("bf16", 2, 34, 2, 128, 64, 300),       # 17 heads per group: back on the vector kernel
])
def test_keyonly_attn(dtype, B, H, Hkv, d, r, T):
    from paper_2603_23914_amd import binding as ap
    print(f"key-only {dtype} B={B} H={H} Hkv={Hkv} d={d} r={r} T={T}", flush=True)
    case, q, V = keyonly_case(dtype, B, H, Hkv, d, r, T, 81)
    dq, dCk, dBk, dV = (to_dev(x, dtype) for x in (q, case.Ck, case.Bk, V))
    out = torch.full((B, H, d), float("nan"), dtype=torch.float32, device="cuda")
    lse = torch.full((B, H), float("nan"), dtype=torch.float32, device="cuda")
    ws = workspace(ap.ap_keyonly_workspace_bytes(B, H, Hkv, d, T, r))
    ap.ap_keyonly_attn(dq, dCk, dBk, dV, out, ws, T=T, sm_scale=1.0 / math.sqrt(d), lse=lse)
    torch.cuda.synchronize()
    P = lambda x: oracle.promote(x, dtype)
    for b in range(B):
        ref, ref_lse = oracle.decode_attn_segments(P(q)[b], [dict(Ck=P(case.Ck)[b, :T], Bk=P(case.Bk)[b], V=P(V)[b, :T])],
                                                   return_lse=True, kv_heads=Hkv)
        assert_close(to_host64(out[b]), ref, dtype, f"key-only b={b}")
        assert np.abs(to_host64(lse[b]) - ref_lse).max() <= 2e-3 * max(1.0, np.abs(ref_lse).max())


def test_keyonly_shared_basis_and_no_lse():
    from paper_2603_23914_amd import binding as ap
    dtype, B, H, Hkv, d, r, T = "f16", 3, 16, 4, 128, 64, 500
    case = wl.decode_case(dtype, B, Hkv, d, r, T, steps=0, seed=82, shared_basis=True, append=False)
    rng = wl.rng_for(82, 1)
    q = wl.store(rng.standard_normal((B, H, d)), dtype)
    V = wl.store(rng.standard_normal((B, T, Hkv * d)), dtype)
    dq, dCk, dBk, dV = (to_dev(x, dtype) for x in (q, case.Ck, case.Bk, V))
    out = torch.empty((B, H, d), dtype=torch.float32, device="cuda")
    ws = workspace(ap.ap_keyonly_workspace_bytes(B, H, Hkv, d, T, r))
    ap.ap_keyonly_attn(dq, dCk, dBk, dV, out, ws, T=T, sm_scale=0.07)
    torch.cuda.synchronize()
    P = lambda x: oracle.promote(x, dtype)
    for b in range(B):
        ref = oracle.decode_attn_segments(P(q)[b], [dict(Ck=P(case.Ck)[b], Bk=P(case.Bk), V=P(V)[b])],
                                          sm_scale=0.07, kv_heads=Hkv)
        assert_close(to_host64(out[b]), ref, dtype, f"shared basis b={b}")


def test_keyonly_empty_cache():
    from paper_2603_23914_amd import binding as ap
    dtype, B, H, Hkv, d, r = "bf16", 2, 8, 2, 64, 64
    case, q, V = keyonly_case(dtype, B, H, Hkv, d, r, 4, 83)
    dq, dCk, dBk, dV = (to_dev(x, dtype) for x in (q, case.Ck, case.Bk, V))
    out = torch.full((B, H, d), float("nan"), dtype=torch.float32, device="cuda")
    lse = torch.full((B, H), float("nan"), dtype=torch.float32, device="cuda")
    ap.ap_keyonly_attn(dq, dCk, dBk, dV, out, workspace(ap.ap_keyonly_workspace_bytes(B, H, Hkv, d, 0, r)), T=0,
                       sm_scale=0.125, lse=lse)
    torch.cuda.synchronize()
    assert (out == 0).all() and torch.isneginf(lse).all()


def test_keyonly_decode_loop_with_raw_tail():
    """Alg. 1's loop for a key-only cache: each step appends the new token (key coefficients by
    projection, value row as is), attends the compressed-key part and an uncompressed tail, and
    joins the two under one softmax."""
    from paper_2603_23914_amd import binding as ap
    dtype, B, H, Hkv, d, r, T0, T_u, steps = "bf16", 2, 16, 4, 128, 64, 300, 37, 3
    HD = Hkv * d
    case, q0, V = keyonly_case(dtype, B, H, Hkv, d, r, T0, 84, T_cap=T0 + steps)
    rng = wl.rng_for(84, 2)
    Ku = wl.store(rng.standard_normal((B, T_u, HD)), dtype)
    Vu = wl.store(rng.standard_normal((B, T_u, HD)), dtype)
    P = lambda x: oracle.promote(x, dtype)
    bits = lambda t: t.view(torch.int16).cpu().numpy().view(np.uint16)
    dCk, dBk, dV, dKu, dVu = (to_dev(x, dtype) for x in (case.Ck, case.Bk, V, Ku, Vu))
    out_c = torch.empty((B, H, d), dtype=torch.float32, device="cuda")
    lse_c = torch.empty((B, H), dtype=torch.float32, device="cuda")
    out_u, lse_u, out = torch.empty_like(out_c), torch.empty_like(lse_c), torch.empty_like(out_c)
    scale = 1.0 / math.sqrt(d)
    for step in range(steps):
        T = T0 + step + 1
        kn, vn = wl.step_new_token(case, step, P(case.Bk), P(case.Bk))
        q = wl.store(wl.rng_for(84, 3, step).standard_normal((B, H, d)), dtype)
        dq, dkn, dvn = (to_dev(x, dtype) for x in (q, kn, vn))
        ap.ap_compact(dkn[:, None, :].contiguous(), None, dBk, None, dCk, None, n=1, row0=T - 1)
        ap.ap_raw_append(None, dvn, None, dV, row=T - 1)
        ap.ap_keyonly_attn(dq, dCk, dBk, dV, out_c, workspace(ap.ap_keyonly_workspace_bytes(B, H, Hkv, d, T, r)), T=T,
                           sm_scale=scale, lse=lse_c)
        ap.ap_raw_attn(dq, dKu, dVu, out_u, workspace(ap.ap_raw_workspace_bytes(B, H, d, T_u)), T_u=T_u,
                       sm_scale=scale, lse=lse_u)
        ap.ap_merge_segments(out_c, lse_c, out_u, lse_u, out)
        torch.cuda.synchronize()
        Ck_h, V_h = P(bits(dCk)), P(bits(dV))
        assert (V_h[:, T - 1] == P(vn)).all()
        for b in range(B):
            ref = oracle.decode_attn_segments(P(q)[b], [dict(Ck=Ck_h[b, :T], Bk=P(case.Bk)[b], V=V_h[b, :T]),
                                                        dict(K=P(Ku)[b], V=P(Vu)[b])], kv_heads=Hkv)
            assert_close(to_host64(out[b]), ref, dtype, f"step {step} b={b}")
        c_ref = oracle.compact(P(kn)[0][None], P(case.Bk)[0])[0]
        assert np.abs(Ck_h[0, T - 1] - c_ref).max() <= 2.0 ** -7 * np.abs(c_ref).max()


def test_keyonly_rejects_bad_arguments():
    from paper_2603_23914_amd import binding as ap
    q = torch.zeros((1, 8, 64), dtype=torch.float16, device="cuda")
    Ck = torch.zeros((1, 16, 64), dtype=torch.float16, device="cuda")
    Bk = torch.zeros((64, 128), dtype=torch.float16, device="cuda")
    V = torch.zeros((1, 16, 128), dtype=torch.float16, device="cuda")
    out = torch.zeros((1, 8, 64), dtype=torch.float32, device="cuda")
    with pytest.raises(RuntimeError):                      # workspace too small
        ap.ap_keyonly_attn(q, Ck, Bk, V, out, torch.empty(256, dtype=torch.uint8, device="cuda"), T=16, sm_scale=1.0)
    with pytest.raises(RuntimeError):                      # more tokens than the cache holds
        ap.ap_keyonly_attn(q, Ck, Bk, V, out, workspace(1 << 20), T=17, sm_scale=1.0)
    assert ap.ap_keyonly_workspace_bytes(1, 8, 2, 64, 16, 644) == 0      # rank not a multiple of 8
    assert ap.ap_keyonly_workspace_bytes(1, 8, 2, 48, 16, 64) == 0    # head width not supported
    assert ap.ap_keyonly_workspace_bytes(1, 8, 3, 64, 16, 64) == 0    # key/value heads must divide the heads
