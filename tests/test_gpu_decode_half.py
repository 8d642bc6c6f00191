"""GPU parity: fp16 / bf16 decode attention (uniform rank) against the fp64 oracle."""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2603_23914_amd import workloads as wl
from gpu_util import TORCH_DT, assert_close, to_dev, to_host64, workspace

pytestmark = pytest.mark.gpu


def run_half(case_dtype, q, Ck, Cv, Bk, Bv, T, want_lse=False, **kw):
    """All array arguments are stored host arrays (bf16 as uint16 bit patterns)."""
    from paper_2603_23914_amd import binding as ap
    B, H, d = q.shape
    r = Ck.shape[2]
    dq, dCk, dCv, dBk, dBv = (to_dev(x, case_dtype) for x in (q, Ck, Cv, Bk, Bv))
    # bf16 keeps 8 significant bits (unit roundoff 3.9e-3 > the 2e-3 bound): take fp32 output there
    out_dt = torch.float32 if case_dtype == "bf16" and not kw.pop("bf16_out", False) else TORCH_DT[case_dtype]
    out = torch.empty((B, H, d), dtype=out_dt, device="cuda")
    lse = torch.empty((B, H), dtype=torch.float32, device="cuda") if want_lse else None
    ws = workspace(ap.ap_decode_workspace_bytes(B, H, d, T, r, ap._DT[TORCH_DT[case_dtype]]))
    ap.ap_decode_attn(dq, dCk, dCv, dBk, dBv, out, ws, T=T, sm_scale=1.0 / math.sqrt(d), lse=lse, **kw)
    torch.cuda.synchronize()
    return (to_host64(out), to_host64(lse)) if want_lse else to_host64(out)


def oracle_out(case_dtype, q, Ck, Cv, Bk, Bv, T, absorbed=True):
    P = lambda x: oracle.promote(x, case_dtype)
    return oracle.decode_attn_batched(P(q), P(Ck), P(Cv), P(Bk), P(Bv), T, absorbed=absorbed)


SHAPES = [
    # dtype, B, H,  d,   r,   T   (T spans several 32-token tiles and a ragged tail)
    ("f16", 2, 32, 128, 512, 333),
    ("bf16", 2, 40, 128, 640, 301),
    ("f16", 3, 8, 64, 128, 97),
    ("bf16", 1, 64, 32, 320, 257),
    ("f16", 2, 16, 128, 64, 70),
    ("bf16", 2, 24, 64, 192, 129),
    ("f16", 1, 40, 128, 640, 31),      # fewer tokens than one tile
    ("bf16", 1, 40, 128, 576, 1),      # a single cached token
    ("f16", 1, 5, 256, 256, 64),       # H < 16, d = 256
]


@pytest.mark.parametrize("dtype,B,H,d,r,T", SHAPES)
def test_decode_uniform_small(dtype, B, H, d, r, T):
    case = wl.decode_case(dtype, B, H, d, r, T, steps=3, seed=7, append=True)
    q = wl.step_query(case, 0)
    print(f"case {dtype} B={B} H={H} d={d} r={r} T={T}", flush=True)
    ref = oracle_out(dtype, q, case.Ck, case.Cv, case.Bk, case.Bv, T)
    # the reconstruct-then-attend definition agrees with the absorbed form on this input
    ref_def = oracle_out(dtype, q[:1], case.Ck[:1], case.Cv[:1], case.Bk[:1], case.Bv[:1], T, absorbed=False)
    assert np.abs(ref_def - ref[:1]).max() < 1e-9
    got, lse = run_half(dtype, q, case.Ck, case.Cv, case.Bk, case.Bv, T, want_lse=True)
    rel = assert_close(got, ref, dtype, f"{dtype} H={H} r={r} T={T}")
    print(f"  max|err|/||out||inf = {rel:.2e}", flush=True)
    P = lambda x: oracle.promote(x, dtype)
    _, ref_lse = oracle.decode_attn_absorbed(P(q)[0], P(case.Ck)[0, :T], P(case.Cv)[0, :T], P(case.Bk)[0],
                                             P(case.Bv)[0], return_lse=True)
    assert np.abs(lse[0] - ref_lse).max() < 2e-3 * max(1.0, np.abs(ref_lse).max())


def test_decode_shared_basis_and_determinism():
    case = wl.decode_case("f16", 4, 32, 128, 512, 200, steps=0, seed=3, shared_basis=True, append=False)
    q = wl.step_query(case, 1)
    ref = oracle_out("f16", q, case.Ck, case.Cv, case.Bk, case.Bv, 200)
    a = run_half("f16", q, case.Ck, case.Cv, case.Bk, case.Bv, 200)
    b = run_half("f16", q, case.Ck, case.Cv, case.Bk, case.Bv, 200)
    assert_close(a, ref, "f16", "shared basis")
    assert (a == b).all(), "same inputs twice must give identical bits"


def test_decode_peaked_softmax_large_logits():
    """Scores far from zero and one dominant token: the online softmax must not overflow."""
    dtype = "bf16"
    case = wl.decode_case(dtype, 1, 40, 128, 640, 200, steps=0, seed=5, append=False)
    q = wl.store(8.0 * wl.rng_for(5, 99).standard_normal((1, 40, 128)), dtype)   # logits ~ N(0, 64)
    ref = oracle_out(dtype, q, case.Ck, case.Cv, case.Bk, case.Bv, 200)
    got = run_half(dtype, q, case.Ck, case.Cv, case.Bk, case.Bv, 200)
    assert_close(got, ref, dtype, "peaked softmax")


@pytest.mark.parametrize("dtype,B,H,d,r,T0", [("bf16", 2, 40, 128, 640, 150), ("f16", 3, 32, 128, 512, 65),
                                              ("f16", 2, 8, 64, 192, 31)])
def test_decode_step_equals_compact_then_attend(dtype, B, H, d, r, T0, value_path):
    """ap_decode_step (key append fused with the fold, value append fused with the expansion)
    against ap_compact + ap_decode_attn: the appended key row has the same bits, the value row
    and the outputs agree to fp32 summation order, and both match the oracle."""
    from paper_2603_23914_amd import binding as ap
    case = wl.decode_case(dtype, B, H, d, r, T0, steps=2, seed=21, append=True)
    P = lambda x: oracle.promote(x, dtype)
    kn, vn = wl.step_new_token(case, 0, P(case.Bk), P(case.Bv))
    q = wl.step_query(case, 0)
    T = T0 + 1
    res = []
    for fused in (False, True):
        dq, dCk, dCv, dBk, dBv, dkn, dvn = (to_dev(x, dtype) for x in (q, case.Ck, case.Cv, case.Bk, case.Bv, kn, vn))
        out = torch.empty((B, H, d), dtype=torch.float32, device="cuda")
        ws = workspace(ap.ap_decode_workspace_bytes(B, H, d, T, r, ap._DT[TORCH_DT[dtype]]))
        if fused:
            ap.ap_decode_step(dq, dkn, dvn, dCk, dCv, dBk, dBv, out, ws, T=T, sm_scale=1.0 / math.sqrt(d))
        else:
            ap.ap_compact(dkn[:, None, :].contiguous(), dvn[:, None, :].contiguous(), dBk, dBv, dCk, dCv, n=1, row0=T0)
            ap.ap_decode_attn(dq, dCk, dCv, dBk, dBv, out, ws, T=T, sm_scale=1.0 / math.sqrt(d))
        torch.cuda.synchronize()
        res.append((out.cpu().numpy(), dCk.view(torch.int16).cpu().numpy(), dCv.view(torch.int16).cpu().numpy()))
    assert (res[0][1] == res[1][1]).all(), "appended key rows differ"
    va = Cv_a = res[0][2][:, T0].view(np.uint16).astype(np.int32)
    vb = res[1][2][:, T0].view(np.uint16).astype(np.int32)
    assert np.abs(va - vb).max() <= 1, "appended value rows differ by more than one unit in the last place"
    assert (res[0][2][:, :T0] == res[1][2][:, :T0]).all()
    assert np.abs(res[0][0] - res[1][0]).max() <= 2e-4 * np.abs(res[0][0]).max()
    # and the step is right: oracle on the stored bits
    Ck_h = res[1][1].view(np.uint16) if dtype == "bf16" else res[1][1].view(np.float16)
    Cv_h = res[1][2].view(np.uint16) if dtype == "bf16" else res[1][2].view(np.float16)
    ref = oracle.decode_attn_batched(P(q), P(Ck_h), P(Cv_h), P(case.Bk), P(case.Bv), T, absorbed=True)
    assert_close(res[1][0].astype(np.float64), ref, dtype, "fused step")
    c_ref = oracle.compact(P(kn)[0][None], P(case.Bk)[0])[0]
    assert np.abs(P(Ck_h)[0, T0] - c_ref).max() <= 2.0 ** -7 * np.abs(c_ref).max()


@pytest.mark.parametrize("dtype,B,H,d,r,T", [
    ("bf16", 2, 40, 128, 128, 1000),    # many rounds of four tiles and a ragged tail
    ("f16", 2, 32, 128, 64, 333),
    ("bf16", 1, 64, 32, 128, 129),      # four head tiles
    ("f16", 3, 5, 256, 64, 97),         # fewer tiles than one round
    ("bf16", 2, 40, 128, 64, 31),       # a single partial tile
    ("f16", 1, 16, 64, 128, 1),
    ("bf16", 64, 40, 128, 128, 520),    # every split has tiles in some slots only
    ("f16", 2, 64, 64, 64, 200),        # four head tiles at rank 64
    ("bf16", 2, 32, 128, 128, 32),      # the appended token opens a new tile
    ("f16", 8, 32, 128, 64, 4000),      # whole groups of 8 sequences, long
])
def test_decode_small_rank(dtype, B, H, d, r, T, value_path):
    """Ranks 64 and 128 run attn_small (waves work alone on whole tiles), except 64 heads at rank
    128, which stay on the token-split variant of the two-role kernel; checked against the
    oracle on the plain call and on the fused step (whose newest token's value row does not
    exist while the kernel runs), with and without the logits output."""
    from paper_2603_23914_amd import binding as ap
    case = wl.decode_case(dtype, B, H, d, r, T, steps=1, seed=27, append=True,
                          batch_subset=range(min(B, 3)), shared_basis=B > 3)
    q = wl.step_query(case, 0)
    nb = min(B, 3)
    print(f"small rank {dtype} B={B} H={H} d={d} r={r} T={T}", flush=True)
    got, lse = run_half(dtype, q, case.Ck, case.Cv, case.Bk, case.Bv, T, want_lse=True)
    Bks = case.Bk if case.Bk.ndim == 2 else case.Bk[:nb]
    Bvs = case.Bv if case.Bv.ndim == 2 else case.Bv[:nb]
    ref = oracle_out(dtype, q[:nb], case.Ck[:nb], case.Cv[:nb], Bks, Bvs, T)
    assert_close(got[:nb], ref, dtype, f"small rank r={r} T={T}")
    assert np.isfinite(got).all()
    # fused step with logits out: one more token, all through the same variant
    P = lambda x: oracle.promote(x, dtype)
    kn, vn = wl.step_new_token(case, 0, P(case.Bk), P(case.Bv))
    dq, dCk, dCv, dBk, dBv, dkn, dvn = (to_dev(x, dtype) for x in (q, case.Ck, case.Cv, case.Bk, case.Bv, kn, vn))
    dCk2, dCv2 = dCk.clone(), dCv.clone()
    out = torch.empty((B, H, d), dtype=torch.float32, device="cuda")
    lse_t = torch.empty((B, H), dtype=torch.float32, device="cuda")
    scores = torch.full((B, case.T_cap, H), float("nan"), dtype=torch.float32, device="cuda")
    ws = workspace(ap.ap_decode_workspace_bytes(B, H, d, T + 1, r, ap._DT[TORCH_DT[dtype]]))
    ap.ap_decode_step(dq, dkn, dvn, dCk, dCv, dBk, dBv, out, ws, T=T + 1, sm_scale=1.0 / math.sqrt(d),
                      lse=lse_t, scores=scores)
    torch.cuda.synchronize()
    Ck_h = dCk.view(torch.int16).cpu().numpy().view(np.uint16) if dtype == "bf16" else dCk.cpu().numpy()
    Cv_h = dCv.view(torch.int16).cpu().numpy().view(np.uint16) if dtype == "bf16" else dCv.cpu().numpy()
    ref2 = oracle_out(dtype, q[:nb], Ck_h[:nb], Cv_h[:nb], Bks, Bvs, T + 1)
    assert_close(to_host64(out[:nb]), ref2, dtype, "small rank fused step")
    # the same fused step without the logits: same appended rows, same result
    out2 = torch.full((B, H, d), float("nan"), dtype=torch.float32, device="cuda")
    lse2 = torch.empty((B, H), dtype=torch.float32, device="cuda")
    ap.ap_decode_step(dq, dkn, dvn, dCk2, dCv2, dBk, dBv, out2, ws, T=T + 1, sm_scale=1.0 / math.sqrt(d), lse=lse2)
    torch.cuda.synchronize()
    assert torch.equal(dCk2.view(torch.int16), dCk.view(torch.int16))
    assert torch.equal(dCv2.view(torch.int16), dCv.view(torch.int16))
    assert_close(to_host64(out2[:nb]), ref2, dtype, "small rank fused step, no logits")
    assert np.abs(to_host64(lse2) - to_host64(lse_t)).max() <= 2e-3 * max(1.0, float(lse_t.abs().max()))
    A = np.exp(to_host64(scores[0, :T + 1, :]).T - to_host64(lse_t[0])[:, None])
    Bk0 = P(case.Bk) if case.Bk.ndim == 2 else P(case.Bk)[0]
    A_ref = oracle.attention_probs(P(q)[0], P(Ck_h)[0, :T + 1], Bk0)
    assert np.abs(A - A_ref).max() <= 2e-3 * A_ref.max()


@pytest.mark.parametrize("B,H,d,r,T,fused", [(2, 40, 128, 640, 301, False), (3, 16, 64, 128, 97, False),
                                             (2, 40, 128, 640, 150, True)])
def test_bf16_output_is_the_fp32_result_rounded_once(B, H, d, r, T, fused, value_path):
    """dt_out = AP_BF16: the kernels round their fp32 result to bfloat16 (nearest even) on the way
    out.  bfloat16 keeps 8 significant bits, so the bound against the oracle is one rounding,
    2^-8 |out|, on top of the fp32 path's 2e-3 ||out||_inf."""
    from paper_2603_23914_amd import binding as ap
    dtype = "bf16"
    case = wl.decode_case(dtype, B, H, d, r, T - 1 if fused else T, steps=1 if fused else 0, seed=44, append=fused)
    q = wl.step_query(case, 0)
    P = lambda x: oracle.promote(x, dtype)
    dq, dBk, dBv = (to_dev(x, dtype) for x in (q, case.Bk, case.Bv))
    outs = []
    for odt in (torch.float32, torch.bfloat16):
        dCk, dCv = to_dev(case.Ck, dtype), to_dev(case.Cv, dtype)
        out = torch.empty((B, H, d), dtype=odt, device="cuda")
        ws = workspace(ap.ap_decode_workspace_bytes(B, H, d, T, r, ap.AP_BF16))
        print(f"bf16 out={odt} B={B} H={H} r={r} T={T} fused={fused}", flush=True)
        if fused:
            kn, vn = wl.step_new_token(case, 0, P(case.Bk), P(case.Bv))
            ap.ap_decode_step(dq, to_dev(kn, dtype), to_dev(vn, dtype), dCk, dCv, dBk, dBv, out, ws, T=T,
                              sm_scale=1.0 / math.sqrt(d))
        else:
            ap.ap_decode_attn(dq, dCk, dCv, dBk, dBv, out, ws, T=T, sm_scale=1.0 / math.sqrt(d))
        torch.cuda.synchronize()
        outs.append(out)
        Ck_h = dCk.view(torch.int16).cpu().numpy().view(np.uint16)
        Cv_h = dCv.view(torch.int16).cpu().numpy().view(np.uint16)
    assert torch.equal(outs[1].view(torch.int16), outs[0].to(torch.bfloat16).view(torch.int16))
    ref = oracle.decode_attn_batched(P(q), P(Ck_h), P(Cv_h), P(case.Bk), P(case.Bv), T, absorbed=True)
    err = np.abs(to_host64(outs[1]) - ref)
    assert (err <= 2.0 ** -8 * np.abs(ref) + 2e-3 * np.abs(ref).max()).all(), err.max()
