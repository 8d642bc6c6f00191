"""GPU parity: 4-bit coefficients (paper Sec. 4.5 / Table 4 combine the method with 4-bit
quantisation; the uniform per-block format is this build's reading).  Codes and scales from the
GPU quantiser bit for bit against the oracle's, decode attention over them against the fp64
oracle run on code * scale."""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2603_23914_amd import workloads as wl
from gpu_util import assert_close, to_dev, to_host64, workspace

pytestmark = pytest.mark.gpu


def gpu_quantize(C, T):
    from paper_2603_23914_amd import binding as ap
    B, cap, r = C.shape
    codes = torch.zeros((B, cap, r // 2), dtype=torch.uint8, device="cuda")
    scales = torch.zeros((B, cap, r // 64), dtype=torch.float16, device="cuda")
    ap.ap_quantize_i4(to_dev(C, "f16"), codes, scales, T=T)
    torch.cuda.synchronize()
    return codes, scales


def check_codes(C, codes, scales, T, seqs):
    for b in seqs:
        rc, rs = oracle.quantize_i4(C[b, :T])
        assert (codes[b, :T].cpu().numpy() == rc).all(), f"4-bit codes differ (b={b})"
        assert (scales[b, :T].cpu().numpy().view(np.uint16) == rs.view(np.uint16)).all(), f"scales differ (b={b})"


def oracle_i4(q, ck4, sk, cv4, sv, Bk, Bv, T, rank_k=None, rank_v=None):
    out = np.empty(q.shape)
    for b in range(q.shape[0]):
        ck = oracle.dequantize_i4(ck4[b, :T], sk[b, :T])
        cv = oracle.dequantize_i4(cv4[b, :T], sv[b, :T])
        out[b] = oracle.decode_attn_absorbed(q[b].astype(np.float64), ck, cv, Bk[b].astype(np.float64),
                                             Bv[b].astype(np.float64),
                                             rank_k=None if rank_k is None else rank_k[b],
                                             rank_v=None if rank_v is None else rank_v[b])
    return out


@pytest.mark.parametrize("B,H,d,r,T", [
    (2, 32, 128, 512, 333),
    (1, 40, 128, 640, 150),
    (3, 8, 64, 128, 97),
    (2, 16, 128, 64, 70),
    (1, 64, 32, 320, 31),
    (1, 24, 64, 192, 1),
    (8, 32, 128, 256, 1200),     # whole groups of 8 sequences, many tiles
])
def test_decode_i4_small(B, H, d, r, T):
    from paper_2603_23914_amd import binding as ap
    case = wl.decode_case("f16", B, H, d, r, T, steps=0, seed=19, append=False)
    q = wl.step_query(case, 0)
    print(f"4-bit decode B={B} H={H} d={d} r={r} T={T}", flush=True)
    ck, sk = gpu_quantize(case.Ck, T)
    cv, sv = gpu_quantize(case.Cv, T)
    check_codes(case.Ck, ck, sk, T, range(B))
    check_codes(case.Cv, cv, sv, T, range(B))
    out = torch.empty((B, H, d), dtype=torch.float32, device="cuda")
    ws = workspace(ap.ap_decode_workspace_bytes(B, H, d, T, r, ap.AP_F16))
    ap.ap_decode_attn(to_dev(q, "f16"), ck, cv, to_dev(case.Bk, "f16"), to_dev(case.Bv, "f16"), out, ws, T=T,
                      sm_scale=1.0 / math.sqrt(d), scale_k=sk, scale_v=sv)
    torch.cuda.synchronize()
    ref = oracle_i4(q, ck.cpu().numpy(), sk.cpu().numpy(), cv.cpu().numpy(), sv.cpu().numpy(), case.Bk, case.Bv, T)
    rel = assert_close(to_host64(out), ref, "f16", "4-bit decode")
    print(f"  max|err|/||out||inf = {rel:.2e}", flush=True)
    # 4 bits are coarse: the quantised cache differs clearly from the fp16 one, so a path that
    # ignored the scales, the nibble order or the block layout could not pass
    P = lambda x: x.astype(np.float64)
    ref16 = oracle.decode_attn_batched(P(q), P(case.Ck), P(case.Cv), P(case.Bk), P(case.Bv), T, absorbed=True)
    assert np.abs(ref16 - ref).max() > 5e-3 * np.abs(ref).max()


@pytest.mark.parametrize("B,H,d,r,T,granks,cum,den,use_k,use_v", [
    (2, 32, 128, 512, 333, (512, 256, 128, 64), (1, 2, 3, 4), 4, True, True),
    (1, 40, 128, 640, 301, (640, 320, 64), (1, 3, 8), 8, True, True),
    (2, 16, 64, 192, 200, (192, 128, 64), (0, 1, 2), 2, False, True),
    (1, 8, 128, 256, 20, (256, 64), (1, 2), 2, True, False),
])
def test_decode_i4_with_per_token_ranks(B, H, d, r, T, granks, cum, den, use_k, use_v):
    from paper_2603_23914_amd import binding as ap
    case = wl.decode_case("f16", B, H, d, r, T, steps=0, seed=20, append=False)
    q = wl.step_query(case, 0)
    ck, sk = gpu_quantize(case.Ck, T)
    cv, sv = gpu_quantize(case.Cv, T)
    mass = wl.rng_for(20, T, r).random((B, T)).astype(np.float32)
    F = len(granks)
    rank = torch.empty((B, T), dtype=torch.int32, device="cuda")
    off = torch.empty((B, F + 1), dtype=torch.int32, device="cuda")
    idx = torch.empty((B, T), dtype=torch.int32, device="cuda")
    ap.ap_select_ranks(torch.from_numpy(mass).cuda(), granks, cum, den, rank, off, idx,
                       workspace(ap.ap_select_workspace_bytes(B, T, F)))
    out = torch.empty((B, H, d), dtype=torch.float32, device="cuda")
    ws = workspace(ap.ap_decode_workspace_bytes(B, H, d, T, r, ap.AP_F16))
    print(f"4-bit ragged B={B} H={H} d={d} r={r} T={T} F={F}", flush=True)
    ap.ap_decode_attn(to_dev(q, "f16"), ck, cv, to_dev(case.Bk, "f16"), to_dev(case.Bv, "f16"), out, ws, T=T,
                      sm_scale=1.0 / math.sqrt(d), scale_k=sk, scale_v=sv, rank_k=rank if use_k else None,
                      rank_v=rank if use_v else None, bucket_off=off, bucket_idx=idx, F=F)
    torch.cuda.synchronize()
    rank_np = rank.cpu().numpy()
    ref = oracle_i4(q, ck.cpu().numpy(), sk.cpu().numpy(), cv.cpu().numpy(), sv.cpu().numpy(), case.Bk, case.Bv, T,
                    rank_np if use_k else None, rank_np if use_v else None)
    assert_close(to_host64(out), ref, "f16", "4-bit with per-token ranks")


def test_decode_i4_full_size():
    """Configuration 5's decode shape with 4-bit coefficients: B=16, H=32, d=128, T=4224, r=512."""
    from paper_2603_23914_amd import binding as ap
    B, H, d, r, T = 16, 32, 128, 512, 4224
    case = wl.decode_case("f16", B, H, d, r, T, steps=0, seed=6, append=False)
    q = wl.step_query(case, 0)
    print("4-bit full size: inputs generated", flush=True)
    ck, sk = gpu_quantize(case.Ck, T)
    cv, sv = gpu_quantize(case.Cv, T)
    check_codes(case.Ck, ck, sk, T, (0, 9))
    check_codes(case.Cv, cv, sv, T, (3, 15))
    out = torch.empty((B, H, d), dtype=torch.float32, device="cuda")
    ws = workspace(ap.ap_decode_workspace_bytes(B, H, d, T, r, ap.AP_F16))
    ap.ap_decode_attn(to_dev(q, "f16"), ck, cv, to_dev(case.Bk, "f16"), to_dev(case.Bv, "f16"), out, ws, T=T,
                      sm_scale=1.0 / math.sqrt(d), scale_k=sk, scale_v=sv)
    torch.cuda.synchronize()
    ref = oracle_i4(q, ck.cpu().numpy(), sk.cpu().numpy(), cv.cpu().numpy(), sv.cpu().numpy(), case.Bk, case.Bv, T)
    got = to_host64(out)
    rel = assert_close(got, ref, "f16", "4-bit full size")
    per_seq = max(np.abs(got[b] - ref[b]).max() / np.abs(ref[b]).max() for b in range(B))
    print(f"  max|err|/||out||inf = {rel:.2e} over the step's output, {per_seq:.2e} per sequence", flush=True)
    assert per_seq <= 2e-3
