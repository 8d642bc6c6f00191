"""GPU parity: value-only compression (raw keys, compressed values) against the fp64 oracle's
definition (rebuild the values, attend), alone and joined with an uncompressed tail."""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2603_23914_amd import workloads as wl
from gpu_util import assert_close, to_dev, to_host64, workspace

pytestmark = pytest.mark.gpu


def valueonly_case(dtype, B, H, Hkv, d, r, T, seed, shared=False):
    """Value coefficients and bases in the law of the compressed-cache workloads (Hkv*d hidden
    columns), raw keys N(0,1), queries for H heads."""
    case = wl.decode_case(dtype, B, Hkv, d, r, T, steps=0, seed=seed, append=False, shared_basis=shared)
    rng = wl.rng_for(seed, 89, T)
    q = wl.store(rng.standard_normal((B, H, d)), dtype)
    K = wl.store(rng.standard_normal((B, T, Hkv * d)), dtype)
    return case, q, K


@pytest.mark.parametrize("dtype,B,H,Hkv,d,r,T", [
    ("bf16", 1, 32, 8, 128, 256, 1500),     # 32 query heads on 8 key/value heads
    ("f16", 2, 8, 8, 64, 128, 333),         # every head its own keys and values
    ("bf16", 2, 12, 4, 256, 320, 257),
    ("f16", 1, 20, 10, 32, 320, 70),        # the widest per-lane share of a coefficient row
    ("f16", 3, 16, 2, 64, 72, 129),         # a rank that is no multiple of 64
    ("bf16", 1, 8, 1, 128, 64, 64),         # one key/value head, eight query heads in a workgroup
    ("f16", 2, 40, 40, 128, 640, 200),
    ("bf16", 1, 6, 3, 64, 192, 1),          # a single token
    ("f16", 1, 64, 8, 128, 384, 2100),      # more than eight splits: merged by their own kernel
    ("bf16", 2, 20, 10, 64, 640, 99),      # ten coefficient chunks per lane
])
def test_valueonly_attn(dtype, B, H, Hkv, d, r, T):
    from paper_2603_23914_amd import binding as ap
    print(f"value-only {dtype} B={B} H={H} Hkv={Hkv} d={d} r={r} T={T}", flush=True)
    case, q, K = valueonly_case(dtype, B, H, Hkv, d, r, T, 91)
    dq, dK, dCv, dBv = (to_dev(x, dtype) for x in (q, K, case.Cv, case.Bv))
    out = torch.full((B, H, d), float("nan"), dtype=torch.float32, device="cuda")
    lse = torch.full((B, H), float("nan"), dtype=torch.float32, device="cuda")
    ws = workspace(ap.ap_valueonly_workspace_bytes(B, H, Hkv, d, T, r))
    ap.ap_valueonly_attn(dq, dK, dCv, dBv, out, ws, T=T, sm_scale=1.0 / math.sqrt(d), lse=lse)
    torch.cuda.synchronize()
    P = lambda x: oracle.promote(x, dtype)
    for b in range(B):
        ref, ref_lse = oracle.decode_attn_segments(P(q)[b], [dict(K=P(K)[b, :T], Cv=P(case.Cv)[b, :T], Bv=P(case.Bv)[b])],
                                                   return_lse=True, kv_heads=Hkv)
        assert_close(to_host64(out[b]), ref, dtype, f"value-only b={b}")
        assert np.abs(to_host64(lse[b]) - ref_lse).max() <= 2e-3 * max(1.0, np.abs(ref_lse).max())


def test_valueonly_shared_basis_joined_with_raw_tail():
    from paper_2603_23914_amd import binding as ap
    dtype, B, H, Hkv, d, r, T, T_u = "f16", 3, 16, 4, 128, 128, 500, 41
    case, q, K = valueonly_case(dtype, B, H, Hkv, d, r, T, 92, shared=True)
    rng = wl.rng_for(92, 1)
    Ku = wl.store(rng.standard_normal((B, T_u, Hkv * d)), dtype)
    Vu = wl.store(rng.standard_normal((B, T_u, Hkv * d)), dtype)
    dq, dK, dCv, dBv, dKu, dVu = (to_dev(x, dtype) for x in (q, K, case.Cv, case.Bv, Ku, Vu))
    out_c = torch.empty((B, H, d), dtype=torch.float32, device="cuda")
    lse_c = torch.empty((B, H), dtype=torch.float32, device="cuda")
    out_u, lse_u, out = torch.empty_like(out_c), torch.empty_like(lse_c), torch.empty_like(out_c)
    ap.ap_valueonly_attn(dq, dK, dCv, dBv, out_c, workspace(ap.ap_valueonly_workspace_bytes(B, H, Hkv, d, T, r)), T=T,
                         sm_scale=0.07, lse=lse_c)
    ap.ap_raw_attn(dq, dKu, dVu, out_u, workspace(ap.ap_raw_workspace_bytes(B, H, d, T_u)), T_u=T_u, sm_scale=0.07,
                   lse=lse_u)
    ap.ap_merge_segments(out_c, lse_c, out_u, lse_u, out)
    torch.cuda.synchronize()
    P = lambda x: oracle.promote(x, dtype)
    for b in range(B):
        ref = oracle.decode_attn_segments(P(q)[b], [dict(K=P(K)[b], Cv=P(case.Cv)[b], Bv=P(case.Bv)),
                                                    dict(K=P(Ku)[b], V=P(Vu)[b])], sm_scale=0.07, kv_heads=Hkv)
        assert_close(to_host64(out[b]), ref, dtype, f"value-only + raw tail b={b}")


def test_valueonly_rejects_bad_arguments():
    from paper_2603_23914_amd import binding as ap
    q = torch.zeros((1, 8, 64), dtype=torch.float16, device="cuda")
    K = torch.zeros((1, 16, 128), dtype=torch.float16, device="cuda")
    Cv = torch.zeros((1, 16, 64), dtype=torch.float16, device="cuda")
    Bv = torch.zeros((64, 128), dtype=torch.float16, device="cuda")
    out = torch.zeros((1, 8, 64), dtype=torch.float32, device="cuda")
    with pytest.raises(RuntimeError):                      # workspace too small
        ap.ap_valueonly_attn(q, K, Cv, Bv, out, torch.empty(256, dtype=torch.uint8, device="cuda"), T=16, sm_scale=1.0)
    with pytest.raises(RuntimeError):                      # an empty cache has no softmax
        ap.ap_valueonly_attn(q, K, Cv, Bv, out, workspace(1 << 20), T=0, sm_scale=1.0)
    assert ap.ap_valueonly_workspace_bytes(1, 8, 2, 32, 16, 640) == 0     # rank limit at d = 32
    assert ap.ap_valueonly_workspace_bytes(1, 8, 3, 64, 16, 64) == 0      # key/value heads must divide the heads
