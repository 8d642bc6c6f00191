"""GPU parity: decode attention over int8 coefficients (in-kernel dequantisation) against the
fp64 oracle run on code*scale; configuration 5's decode step at full size."""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2603_23914_amd import workloads as wl
from gpu_util import assert_close, to_dev, to_host64, workspace

pytestmark = pytest.mark.gpu


def quantize_case(case, T):
    """int8 codes and fp16 scales of the case's fp16 coefficients, by the oracle's recipe."""
    out = []
    for C in (case.Ck, case.Cv):
        codes = np.zeros(C.shape, np.int8)
        scales = np.zeros(C.shape[:2] + (C.shape[2] // 64,), np.float16)
        for b in range(C.shape[0]):
            codes[b, :T], scales[b, :T] = oracle.quantize_i8(C[b, :T])
        out += [codes, scales]
    return out


def run_i8(q, Ck8, sk, Cv8, sv, Bk, Bv, T):
    from paper_2603_23914_amd import binding as ap
    B, H, d = q.shape
    r = Ck8.shape[2]
    dq, dBk, dBv = (to_dev(x, "f16") for x in (q, Bk, Bv))
    dCk, dCv = torch.from_numpy(Ck8).cuda(), torch.from_numpy(Cv8).cuda()
    dsk, dsv = torch.from_numpy(sk).cuda(), torch.from_numpy(sv).cuda()
    out = torch.empty((B, H, d), dtype=torch.float32, device="cuda")
    ws = workspace(ap.ap_decode_workspace_bytes(B, H, d, T, r, ap.AP_F16))
    ap.ap_decode_attn(dq, dCk, dCv, dBk, dBv, out, ws, T=T, sm_scale=1.0 / math.sqrt(d),
                      scale_k=dsk, scale_v=dsv)
    torch.cuda.synchronize()
    return to_host64(out)


def oracle_i8(q, Ck8, sk, Cv8, sv, Bk, Bv, T, batch=None):
    P = lambda x: x.astype(np.float64)
    bs = range(q.shape[0]) if batch is None else batch
    out = {}
    for b in bs:
        ck = oracle.dequantize_i8(Ck8[b, :T], sk[b, :T])
        cv = oracle.dequantize_i8(Cv8[b, :T], sv[b, :T])
        bk = Bk[b] if Bk.ndim == 3 else Bk
        bv = Bv[b] if Bv.ndim == 3 else Bv
        out[b] = oracle.decode_attn_absorbed(P(q[b]), ck, cv, P(bk), P(bv))
    return out


@pytest.mark.parametrize("B,H,d,r,T", [
    (2, 32, 128, 512, 333),
    (1, 40, 128, 640, 150),
    (3, 8, 64, 128, 97),
    (2, 16, 128, 64, 70),
    (1, 64, 32, 320, 31),
    (1, 24, 64, 192, 1),
])
def test_decode_i8_small(B, H, d, r, T):
    case = wl.decode_case("f16", B, H, d, r, T, steps=0, seed=17, append=False)
    q = wl.step_query(case, 0)
    Ck8, sk, Cv8, sv = quantize_case(case, T)
    print(f"int8 decode B={B} H={H} d={d} r={r} T={T}", flush=True)
    ref = oracle_i8(q, Ck8, sk, Cv8, sv, case.Bk, case.Bv, T)
    got = run_i8(q, Ck8, sk, Cv8, sv, case.Bk, case.Bv, T)
    ref = np.stack([ref[b] for b in range(B)])
    rel = assert_close(got, ref, "f16", "int8 decode")
    print(f"  max|err|/||out||inf = {rel:.2e}", flush=True)
    # the quantised cache differs measurably from the fp16 one, so a path that ignored the
    # scales or read the wrong block could not pass
    P = lambda x: oracle.promote(x, "f16")
    ref16 = oracle.decode_attn_batched(P(q), P(case.Ck), P(case.Cv), P(case.Bk), P(case.Bv), T, absorbed=True)
    assert np.abs(ref16 - ref).max() > 1e-4 * np.abs(ref).max()


def test_config5_decode_full_size():
    """Configuration 5's decode step: B=16, H=32, d=128 (HD=4096), T=4224, r=512, int8
    coefficients produced on the GPU by ap_quantize_i8 from fp16 coefficients (codes checked
    against the oracle on a sample), one decode step, every sequence checked; the error bound
    is relative to the largest magnitude of the step's whole [B, H, d] output."""
    from paper_2603_23914_amd import binding as ap
    B, H, d, r, T = 16, 32, 128, 512, 4224
    case = wl.decode_case("f16", B, H, d, r, T, steps=0, seed=5, append=False)
    q = wl.step_query(case, 0)
    print("config 5 decode: inputs generated", flush=True)
    codes, scales = [], []
    for C in (case.Ck, case.Cv):
        dC = to_dev(C, "f16")
        c8 = torch.empty((B, T, r), dtype=torch.int8, device="cuda")
        sc = torch.empty((B, T, r // 64), dtype=torch.float16, device="cuda")
        ap.ap_quantize_i8(dC, c8, sc, T=T)
        torch.cuda.synchronize()
        codes.append(c8.cpu().numpy())
        scales.append(sc.cpu().numpy())
        rc, rs = oracle.quantize_i8(C[3])
        assert (codes[-1][3] == rc).all() and (scales[-1][3].view(np.uint16) == rs.view(np.uint16)).all()
    got = run_i8(q, codes[0], scales[0], codes[1], scales[1], case.Bk, case.Bv, T)
    ref = oracle_i8(q, codes[0], scales[0], codes[1], scales[1], case.Bk, case.Bv, T)
    ref = np.stack([ref[b] for b in range(B)])
    rel = assert_close(got, ref, "f16", "config 5 decode")
    per_seq = max(np.abs(got[b] - ref[b]).max() / np.abs(ref[b]).max() for b in range(B))
    print(f"  max|err|/||out||inf = {rel:.2e} over the step's output, {per_seq:.2e} per sequence", flush=True)
    assert per_seq <= 2e-3          # the stricter norm holds too (scales are applied in fp32)


@pytest.mark.parametrize("B,H,d,r,T,granks,cum,den,use_k,use_v", [
    (2, 32, 128, 512, 333, (512, 256, 128, 64), (1, 2, 3, 4), 4, True, True),
    (1, 40, 128, 640, 301, (640, 320, 64), (1, 3, 8), 8, True, True),
    (2, 16, 64, 192, 200, (192, 128, 64), (0, 1, 2), 2, False, True),     # values only, empty first group
    (1, 8, 128, 256, 20, (256, 64), (1, 2), 2, True, False),              # keys only, fewer tokens than a tile
])
def test_decode_i8_with_per_token_ranks(B, H, d, r, T, granks, cum, den, use_k, use_v):
    """int8 coefficients read at attention-chosen ranks (multiples of the 64-column scale block)."""
    from paper_2603_23914_amd import binding as ap
    case = wl.decode_case("f16", B, H, d, r, T, steps=0, seed=18, append=False)
    q = wl.step_query(case, 0)
    Ck8, sk, Cv8, sv = quantize_case(case, T)
    mass = wl.rng_for(18, T, r).random((B, T)).astype(np.float32)
    F = len(granks)
    dm = torch.from_numpy(mass).cuda()
    rank = torch.empty((B, T), dtype=torch.int32, device="cuda")
    off = torch.empty((B, F + 1), dtype=torch.int32, device="cuda")
    idx = torch.empty((B, T), dtype=torch.int32, device="cuda")
    ap.ap_select_ranks(dm, granks, cum, den, rank, off, idx, workspace(ap.ap_select_workspace_bytes(B, T, F)))
    dq, dBk, dBv = (to_dev(x, "f16") for x in (q, case.Bk, case.Bv))
    dCk, dCv = torch.from_numpy(Ck8).cuda(), torch.from_numpy(Cv8).cuda()
    dsk, dsv = torch.from_numpy(sk).cuda(), torch.from_numpy(sv).cuda()
    out = torch.empty((B, H, d), dtype=torch.float32, device="cuda")
    ws = workspace(ap.ap_decode_workspace_bytes(B, H, d, T, r, ap.AP_F16))
    print(f"int8 ragged B={B} H={H} d={d} r={r} T={T} F={F}", flush=True)
    ap.ap_decode_attn(dq, dCk, dCv, dBk, dBv, out, ws, T=T, sm_scale=1.0 / math.sqrt(d), scale_k=dsk,
                      scale_v=dsv, rank_k=rank if use_k else None, rank_v=rank if use_v else None,
                      bucket_off=off, bucket_idx=idx, F=F)
    torch.cuda.synchronize()
    rank_np = rank.cpu().numpy()
    ref = np.empty((B, H, d))
    for b in range(B):
        r_ref, _, _ = oracle.select_ranks(mass[b], granks, cum, den)
        assert (rank_np[b] == r_ref).all()
        ck = oracle.dequantize_i8(Ck8[b, :T], sk[b, :T])
        cv = oracle.dequantize_i8(Cv8[b, :T], sv[b, :T])
        ref[b] = oracle.decode_attn_absorbed(q[b].astype(np.float64), ck, cv, case.Bk[b].astype(np.float64),
                                             case.Bv[b].astype(np.float64),
                                             rank_k=rank_np[b] if use_k else None,
                                             rank_v=rank_np[b] if use_v else None)
    assert_close(to_host64(out), ref, "f16", "int8 with per-token ranks")
