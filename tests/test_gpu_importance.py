"""GPU parity: importance tracking in the decode loop (Eq. 1, Sec. 3.2).

The decode call returns the scaled logits next to the log-sum-exp; ap_update_importance turns
them into head-averaged attention weights and folds them into the running mass; ap_select_ranks
cuts the mass into rank groups for the next step.  Each link is checked against the fp64 oracle:
weights against oracle.attention_probs, the moving average against oracle.importance_update,
the groups bit for bit against oracle.select_ranks of the mass the GPU holds.
"""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2603_23914_amd import workloads as wl
from gpu_util import TORCH_DT, assert_close, to_dev, to_host64, workspace

pytestmark = pytest.mark.gpu

PROB_TOL = 2e-3          # max|A_gpu - A_ref| <= PROB_TOL * max A_ref  (same bound as the outputs)


def stored(t: torch.Tensor, dtype: str) -> np.ndarray:
    """GPU tensor of the case's storage type -> host array in the stored form."""
    if dtype == "bf16":
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def oracle_probs(dtype, q, Ck, Bk, T, rank=None):
    P = lambda x: oracle.promote(x, dtype)
    B = q.shape[0]
    return np.stack([oracle.attention_probs(P(q)[b], P(Ck)[b, :T], P(Bk)[b if Bk.ndim == 3 else ...],
                                            rank_k=None if rank is None else rank[b])
                     for b in range(B)])


@pytest.mark.parametrize("dtype,B,H,d,r,T", [("bf16", 2, 40, 128, 640, 301), ("f16", 2, 32, 128, 512, 333),
                                             ("f16", 1, 5, 256, 256, 64), ("f32", 2, 4, 32, 48, 150)])
def test_scores_give_the_attention_weights(dtype, B, H, d, r, T):
    from paper_2603_23914_amd import binding as ap
    case = wl.decode_case(dtype, B, H, d, r, T, steps=0, seed=31, append=False)
    q = wl.step_query(case, 0)
    print(f"scores {dtype} B={B} H={H} d={d} r={r} T={T}", flush=True)
    dq, dCk, dCv, dBk, dBv = (to_dev(x, dtype) for x in (q, case.Ck, case.Cv, case.Bk, case.Bv))
    T_cap = case.Ck.shape[1]
    out = torch.empty((B, H, d), dtype=torch.float32, device="cuda")
    lse = torch.empty((B, H), dtype=torch.float32, device="cuda")
    scores = torch.full((B, T_cap, H), float("nan"), dtype=torch.float32, device="cuda")
    ws = workspace(ap.ap_decode_workspace_bytes(B, H, d, T, r, ap._DT[TORCH_DT[dtype]]))
    ap.ap_decode_attn(dq, dCk, dCv, dBk, dBv, out, ws, T=T, sm_scale=1.0 / math.sqrt(d), lse=lse,
                      scores=scores)
    torch.cuda.synchronize()
    s = to_host64(scores)[:, :T, :].transpose(0, 2, 1)
    assert np.isfinite(s).all(), "a logit of an attended token was not written"
    A = np.exp(s - to_host64(lse)[:, :, None])
    ref = oracle_probs(dtype, q, case.Ck, case.Bk, T)
    tol = 1e-5 if dtype == "f32" else PROB_TOL
    assert np.abs(A - ref).max() <= tol * ref.max()
    assert np.abs(A.sum(axis=2) - 1.0).max() <= (1e-5 if dtype == "f32" else 2e-3)
    # the same call without the extra output gives the same bits
    out2 = torch.empty_like(out)
    ap.ap_decode_attn(dq, dCk, dCv, dBk, dBv, out2, ws, T=T, sm_scale=1.0 / math.sqrt(d))
    torch.cuda.synchronize()
    assert torch.equal(out, out2)


@pytest.mark.parametrize("B,H,T,T_cap,stride,alpha", [(3, 40, 1000, 1024, 1100, 0.9), (1, 7, 5, 5, 5, 0.0),
                                                      (2, 32, 257, 300, 257, 1.0), (2, 8, 4224, 4224, 4224, 0.5),
                                                      (1, 256, 200, 200, 200, 0.3), (1, 260, 130, 131, 130, 0.3)])
def test_update_importance_kernel(B, H, T, T_cap, stride, alpha):
    """The moving average alone, on logits and log-sum-exp made on the host."""
    from paper_2603_23914_amd import binding as ap
    rng = wl.rng_for(32, B, H, T)
    s = (3.0 * rng.standard_normal((B, H, T_cap))).astype(np.float32)
    m = s[:, :, :T].astype(np.float64)
    lse = (np.log(np.exp(m - m.max(axis=2, keepdims=True)).sum(axis=2)) + m.max(axis=2)).astype(np.float32)
    mass0 = rng.random((B, stride)).astype(np.float32)
    ds, dl, dm = (torch.from_numpy(x).cuda() for x in (np.ascontiguousarray(s.transpose(0, 2, 1)), lse, mass0))
    ap.ap_update_importance(ds, dl, dm, T=T, alpha=alpha)
    torch.cuda.synchronize()
    got = dm.cpu().numpy()
    A = np.exp(m - lse.astype(np.float64)[:, :, None])                     # [B, H, T]
    for b in range(B):
        ref = oracle.importance_update(mass0[b, :T], A[b][None], alpha)
        assert np.abs(got[b, :T] - ref).max() <= 2e-6 * max(ref.max(), 1e-30)
        assert (got[b, T:] == mass0[b, T:]).all(), "mass beyond T must not change"


def test_importance_loop_feeds_rank_selection():
    """Decode steps with append; after each step the mass is updated from that step's weights
    and the next step runs at the ranks selected from it."""
    from paper_2603_23914_amd import binding as ap
    dtype, B, H, d, r, T0, steps, alpha = "bf16", 2, 40, 128, 640, 150, 4, 0.8
    granks, cum, den = (640, 320, 64), (1, 3, 8), 8
    F = len(granks)
    case = wl.decode_case(dtype, B, H, d, r, T0, steps=steps, seed=33, append=True)
    P = lambda x: oracle.promote(x, dtype)
    T_cap = case.T_cap
    dCk, dCv, dBk, dBv = (to_dev(x, dtype) for x in (case.Ck, case.Cv, case.Bk, case.Bv))
    mass0 = np.zeros((B, T_cap), np.float32)
    mass0[:, :T0] = wl.rng_for(33, 7).random((B, T0)).astype(np.float32) / T0
    dmass = torch.from_numpy(mass0).cuda()
    ref_mass = mass0.astype(np.float64)
    out = torch.empty((B, H, d), dtype=torch.float32, device="cuda")
    lse = torch.empty((B, H), dtype=torch.float32, device="cuda")
    scores = torch.empty((B, T_cap, H), dtype=torch.float32, device="cuda")
    rank_np = None
    rank = off = idx = None
    for step in range(steps):
        T = T0 + step + 1
        print(f"importance loop step {step}: T={T}", flush=True)
        kn, vn = wl.step_new_token(case, step, P(case.Bk), P(case.Bv))
        q = wl.step_query(case, step)
        dq, dkn, dvn = (to_dev(x, dtype) for x in (q, kn, vn))
        ws = workspace(ap.ap_decode_workspace_bytes(B, H, d, T, r, ap._DT[TORCH_DT[dtype]]))
        if rank is None:
            ap.ap_decode_step(dq, dkn, dvn, dCk, dCv, dBk, dBv, out, ws, T=T, sm_scale=1.0 / math.sqrt(d),
                              lse=lse, scores=scores)
        else:
            ap.ap_decode_step(dq, dkn, dvn, dCk, dCv, dBk, dBv, out, ws, T=T, sm_scale=1.0 / math.sqrt(d),
                              rank_k=rank, rank_v=rank, bucket_off=off, bucket_idx=idx, F=F, lse=lse,
                              scores=scores)
        ap.ap_update_importance(scores, lse, dmass, T=T, alpha=alpha)
        torch.cuda.synchronize()
        # oracle on the coefficient bits the GPU holds after the append
        Ck_h, Cv_h = stored(dCk, dtype), stored(dCv, dtype)
        ref_out = oracle.decode_attn_batched(P(q), P(Ck_h), P(Cv_h), P(case.Bk), P(case.Bv), T,
                                             rank_k=rank_np, rank_v=rank_np, absorbed=True)
        assert_close(to_host64(out), ref_out, dtype, f"step {step} output")
        A = oracle_probs(dtype, q, Ck_h, case.Bk, T, rank_np)
        for b in range(B):
            ref_mass[b, :T] = oracle.importance_update(ref_mass[b, :T], A[b][None], alpha)
        got_mass = dmass.cpu().numpy()
        assert np.abs(got_mass[:, :T] - ref_mass[:, :T]).max() <= PROB_TOL * ref_mass[:, :T].max()
        assert (got_mass[:, T:] == 0).all()
        # groups for the next step: the newest token is listed at rank r first (it has no history),
        # so select over T+1 entries with the coming token's mass set above every other
        Tn = T + 1
        if Tn > T_cap:
            break
        sel = dmass[:, :Tn].clone()
        sel[:, T] = 2.0
        rank = torch.empty((B, Tn), dtype=torch.int32, device="cuda")
        off = torch.empty((B, F + 1), dtype=torch.int32, device="cuda")
        idx = torch.empty((B, Tn), dtype=torch.int32, device="cuda")
        ap.ap_select_ranks(sel, granks, cum, den, rank, off, idx,
                           workspace(ap.ap_select_workspace_bytes(B, Tn, F)))
        torch.cuda.synchronize()
        sel_h = sel.cpu().numpy()
        rank_np = rank.cpu().numpy()
        for b in range(B):
            r_ref, o_ref, i_ref = oracle.select_ranks(sel_h[b], granks, cum, den)
            assert (rank_np[b] == r_ref).all() and (off[b].cpu().numpy() == o_ref).all()
            assert (idx[b].cpu().numpy() == i_ref).all()
            assert rank_np[b, T] == granks[0]
