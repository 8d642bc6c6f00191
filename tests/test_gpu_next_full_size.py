"""GPU parity at full batch size for the rows built after the hot path: importance tracking,
the uncompressed segment, grouped queries, key-only compression and the loop of Alg. 1 at the
paper's operating point, in the launch shapes a 64-sequence decode uses.
Inputs are drawn on the GPU with torch (seeded, the law of the benchmark's coefficients); the
sampled sequences are read back bit for bit and the fp64 oracle computes their results alone."""
import math

import numpy as np
import pytest
import torch

import oracle
from gpu_util import assert_close, to_host64, workspace

pytestmark = pytest.mark.gpu

SAMPLE = (0, 37)


def bits(t: torch.Tensor) -> np.ndarray:
    """bf16 GPU tensor -> uint16 bit patterns on the host (what oracle.promote(.., "bf16") takes)."""
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def P(t: torch.Tensor) -> np.ndarray:
    return oracle.promote(bits(t), "bf16")


def draw_cache(B, T_cap, r, HD, seed):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    sig = torch.arange(1, r + 1, device="cuda", dtype=torch.float32) ** -0.7
    ks = sig * math.sqrt(HD / float((sig ** 2).sum()))
    out = []
    for _ in range(2):                                   # C_k, C_v
        c = torch.empty((B, T_cap, r), dtype=torch.bfloat16, device="cuda")
        for b0 in range(0, B, 8):
            x = torch.randn((8, T_cap, r), generator=g, device="cuda") * ks
            x += 0.01 * torch.randn((8, T_cap, r), generator=g, device="cuda")
            c[b0:b0 + 8] = x.to(torch.bfloat16)
        out.append(c)
    for _ in range(2):                                   # B_k, B_v: rows of unit norm on average
        out.append((torch.randn((B, r, HD), generator=g, device="cuda") / math.sqrt(HD)).to(torch.bfloat16))
    return out, g


def test_importance_tracking_full_size():
    from paper_2603_23914_amd import binding as ap
    B, H, d, r, T0 = 64, 40, 128, 640, 4223
    T, HD = T0 + 1, H * d
    (Ck, Cv, Bk, Bv), g = draw_cache(B, T, r, HD, 61)
    q = torch.randn((B, H, d), generator=g, device="cuda").to(torch.bfloat16)
    kn = torch.randn((B, HD), generator=g, device="cuda").to(torch.bfloat16)
    vn = torch.randn((B, HD), generator=g, device="cuda").to(torch.bfloat16)
    mass = torch.rand((B, T), generator=g, device="cuda") / T
    mass[:, T - 1] = 0.0                                  # the token being appended has no history
    mass0 = mass.clone()
    out = torch.empty((B, H, d), dtype=torch.float32, device="cuda")
    lse = torch.empty((B, H), dtype=torch.float32, device="cuda")
    scores = torch.empty((B, T, H), dtype=torch.float32, device="cuda")
    ws = workspace(ap.ap_decode_workspace_bytes(B, H, d, T, r, ap.AP_BF16))
    print("importance, 64 sequences at T=4224", flush=True)
    ap.ap_decode_step(q, kn, vn, Ck, Cv, Bk, Bv, out, ws, T=T, sm_scale=1.0 / math.sqrt(d), lse=lse, scores=scores)
    ap.ap_update_importance(scores, lse, mass, T=T, alpha=0.9)
    granks, cum, den = (640, 320, 128, 64), (1, 2, 3, 4), 4
    rank = torch.empty((B, T), dtype=torch.int32, device="cuda")
    off = torch.empty((B, 5), dtype=torch.int32, device="cuda")
    idx = torch.empty((B, T), dtype=torch.int32, device="cuda")
    ap.ap_select_ranks(mass, granks, cum, den, rank, off, idx, workspace(ap.ap_select_workspace_bytes(B, T, 4)))
    torch.cuda.synchronize()
    for b in SAMPLE:
        A = oracle.attention_probs(P(q[b]), P(Ck[b, :T]), P(Bk[b]))
        ref = oracle.importance_update(mass0[b].cpu().numpy(), A[None], 0.9)
        got = mass[b].cpu().numpy()
        assert np.abs(got - ref).max() <= 2e-3 * ref.max(), f"b={b}"
        r_ref, o_ref, i_ref = oracle.select_ranks(got, granks, cum, den)      # same fp32 mass on both sides
        assert (rank[b].cpu().numpy() == r_ref).all() and (off[b].cpu().numpy() == o_ref).all()
        assert (idx[b].cpu().numpy() == i_ref).all()
        ref_out = oracle.decode_attn_absorbed(P(q[b]), P(Ck[b, :T]), P(Cv[b, :T]), P(Bk[b]), P(Bv[b]))
        assert_close(to_host64(out[b]), ref_out, "bf16", f"output with logits stored, b={b}")


def test_uncompressed_segment_full_size():
    from paper_2603_23914_amd import binding as ap
    B, H, d, r, T, T_u = 64, 40, 128, 640, 4224, 256
    HD = H * d
    (Ck, Cv, Bk, Bv), g = draw_cache(B, T, r, HD, 62)
    q = torch.randn((B, H, d), generator=g, device="cuda").to(torch.bfloat16)
    K = torch.randn((B, T_u, HD), generator=g, device="cuda").to(torch.bfloat16)
    V = torch.randn((B, T_u, HD), generator=g, device="cuda").to(torch.bfloat16)
    out_c = torch.empty((B, H, d), dtype=torch.float32, device="cuda")
    lse_c = torch.empty((B, H), dtype=torch.float32, device="cuda")
    out_u, lse_u = torch.empty_like(out_c), torch.empty_like(lse_c)
    out = torch.empty_like(out_c)
    print("compressed 4224 + uncompressed 256 tokens, 64 sequences", flush=True)
    ap.ap_decode_attn(q, Ck, Cv, Bk, Bv, out_c, workspace(ap.ap_decode_workspace_bytes(B, H, d, T, r, ap.AP_BF16)),
                      T=T, sm_scale=1.0 / math.sqrt(d), lse=lse_c)
    ap.ap_raw_attn(q, K, V, out_u, workspace(ap.ap_raw_workspace_bytes(B, H, d, T_u)), T_u=T_u,
                   sm_scale=1.0 / math.sqrt(d), lse=lse_u)
    ap.ap_merge_segments(out_c, lse_c, out_u, lse_u, out)
    torch.cuda.synchronize()
    for b in SAMPLE:
        ref = oracle.decode_attn_segments(P(q[b]), [dict(Ck=P(Ck[b]), Cv=P(Cv[b]), Bk=P(Bk[b]), Bv=P(Bv[b])),
                                                    dict(K=P(K[b]), V=P(V[b]))])
        assert_close(to_host64(out[b]), ref, "bf16", f"two segments, b={b}")
        ref_u = oracle.raw_attn(P(q[b]), P(K[b]), P(V[b]))
        assert_close(to_host64(out_u[b]), ref_u, "bf16", f"uncompressed segment alone, b={b}")


def test_grouped_queries_full_size():
    from paper_2603_23914_amd import binding as ap
    B, H, Hkv, d, r, T0 = 64, 32, 8, 128, 256, 4223
    T, HD = T0 + 1, Hkv * d
    (Ck, Cv, Bk, Bv), g = draw_cache(B, T, r, HD, 63)
    q = torch.randn((B, H, d), generator=g, device="cuda").to(torch.bfloat16)
    kn = torch.randn((B, HD), generator=g, device="cuda").to(torch.bfloat16)
    vn = torch.randn((B, HD), generator=g, device="cuda").to(torch.bfloat16)
    out = torch.empty((B, H, d), dtype=torch.float32, device="cuda")
    ws = workspace(ap.ap_decode_workspace_bytes(B, H, d, T, r, ap.AP_BF16))
    print("grouped queries 32/8 heads, 64 sequences at T=4224", flush=True)
    ap.ap_decode_step(q, kn, vn, Ck, Cv, Bk, Bv, out, ws, T=T, sm_scale=1.0 / math.sqrt(d))
    torch.cuda.synchronize()
    for b in SAMPLE:
        ref = oracle.decode_attn_absorbed(P(q[b]), P(Ck[b, :T]), P(Cv[b, :T]), P(Bk[b]), P(Bv[b]), kv_heads=Hkv)
        assert_close(to_host64(out[b]), ref, "bf16", f"grouped queries, b={b}")
        c_ref = oracle.compact(P(kn[b])[None, :], P(Bk[b]))[0]
        err = np.abs(P(Ck[b, T - 1]) - c_ref)
        assert (err <= 2.0 ** -7 * np.abs(c_ref) + 1e-5 * np.abs(c_ref).max()).all()


def test_key_only_compression_full_size():
    """Head layout and key rank of the text-domain experiment (32 query heads on 8 key/value heads,
    R_k = 64), 8 sequences of 8192 tokens: the launch shape profiles/next_rows_kernel_trace.md times."""
    from paper_2603_23914_amd import binding as ap
    B, H, Hkv, d, r, T = 8, 32, 8, 128, 64, 8192
    HD = Hkv * d
    g = torch.Generator(device="cuda")
    g.manual_seed(64)
    sig = torch.arange(1, r + 1, device="cuda", dtype=torch.float32) ** -0.7
    Ck = (torch.randn((B, T, r), generator=g, device="cuda") * (sig * math.sqrt(HD / float((sig ** 2).sum())))).to(torch.bfloat16)
    Bk = (torch.randn((B, r, HD), generator=g, device="cuda") / math.sqrt(HD)).to(torch.bfloat16)
    V = torch.randn((B, T, HD), generator=g, device="cuda").to(torch.bfloat16)
    q = torch.randn((B, H, d), generator=g, device="cuda").to(torch.bfloat16)
    out = torch.empty((B, H, d), dtype=torch.float32, device="cuda")
    lse = torch.empty((B, H), dtype=torch.float32, device="cuda")
    print("key-only compression, 8 sequences at T=8192", flush=True)
    ap.ap_keyonly_attn(q, Ck, Bk, V, out, workspace(ap.ap_keyonly_workspace_bytes(B, H, Hkv, d, T, r)), T=T,
                       sm_scale=1.0 / math.sqrt(d), lse=lse)
    torch.cuda.synchronize()
    for b in (0, 5):
        ref, ref_lse = oracle.decode_attn_segments(P(q[b]), [dict(Ck=P(Ck[b]), Bk=P(Bk[b]), V=P(V[b]))],
                                                   return_lse=True, kv_heads=Hkv)
        assert_close(to_host64(out[b]), ref, "bf16", f"key-only, b={b}")
        assert np.abs(to_host64(lse[b]) - ref_lse).max() <= 2e-3 * max(1.0, np.abs(ref_lse).max())


def test_attention_aware_loop_full_size():
    """The paper's loop at its own operating point, in the shapes bench.py times as
    `attention_aware_loop`: 64 sequences of 4224 tokens, 32 heads, R = 64, a quarter of the tokens
    at the full value rank and the rest at 16 (Sec. 3.2), two rounds of group selection, fused
    step with per-token value ranks and the logits written, importance update (Eq. 1).  Sampled
    sequences: groups bit for bit, appended rows, outputs and masses against the oracle."""
    from paper_2603_23914_amd import binding as ap
    B, H, d, r, T, alpha = 64, 32, 128, 64, 4224, 0.9
    HD = H * d
    (Ck, Cv, Bk, Bv), g = draw_cache(B, T, r, HD, 67)
    mass = torch.rand((B, T), generator=g, device="cuda") / T
    out = torch.empty((B, H, d), dtype=torch.float32, device="cuda")
    lse = torch.empty((B, H), dtype=torch.float32, device="cuda")
    scores = torch.empty((B, T, H), dtype=torch.float32, device="cuda")
    rank = torch.empty((B, T), dtype=torch.int32, device="cuda")
    idx = torch.empty((B, T), dtype=torch.int32, device="cuda")
    off = torch.empty((B, 3), dtype=torch.int32, device="cuda")
    ws = workspace(ap.ap_decode_workspace_bytes(B, H, d, T, r, ap.AP_BF16))
    wsel = workspace(ap.ap_select_workspace_bytes(B, T, 2))
    granks, cum, den = (r, 16), (1, 4), 4
    for rnd in range(2):
        print(f"attention-aware loop, round {rnd}: 64 sequences at T={T}", flush=True)
        q = torch.randn((B, H, d), generator=g, device="cuda").to(torch.bfloat16)
        kn = torch.randn((B, HD), generator=g, device="cuda").to(torch.bfloat16)
        vn = torch.randn((B, HD), generator=g, device="cuda").to(torch.bfloat16)
        mass[:, T - 1] = 2.0                               # the token being appended: full rank
        sel = mass.clone()
        ap.ap_select_ranks(sel, granks, cum, den, rank, off, idx, wsel)
        mass[:, T - 1] = 0.0                               # and no history yet (reading of Eq. 1's start)
        mass0 = mass.clone()
        ap.ap_decode_step(q, kn, vn, Ck, Cv, Bk, Bv, out, ws, T=T, sm_scale=1.0 / math.sqrt(d),
                          rank_v=rank, bucket_off=off, bucket_idx=idx, F=2, lse=lse, scores=scores)
        ap.ap_update_importance(scores, lse, mass, T=T, alpha=alpha)
        torch.cuda.synchronize()
        for b in SAMPLE:
            r_ref, o_ref, i_ref = oracle.select_ranks(sel[b].cpu().numpy(), granks, cum, den)
            rank_b = rank[b].cpu().numpy()
            assert (rank_b == r_ref).all() and (off[b].cpu().numpy() == o_ref).all()
            assert (idx[b].cpu().numpy() == i_ref).all()
            for C, Bm, x, name in ((Ck, Bk, kn, "key"), (Cv, Bv, vn, "value")):
                c_ref = oracle.compact(P(x[b])[None], P(Bm[b]))[0]
                assert np.abs(P(C[b, T - 1]) - c_ref).max() <= 2.0 ** -7 * np.abs(c_ref).max(), f"{name} row, b={b}"
            ref_out = oracle.decode_attn_absorbed(P(q[b]), P(Ck[b, :T]), P(Cv[b, :T]), P(Bk[b]), P(Bv[b]),
                                                  rank_v=rank_b)
            assert_close(to_host64(out[b]), ref_out, "bf16", f"round {rnd} output, b={b}")
            A = oracle.attention_probs(P(q[b]), P(Ck[b, :T]), P(Bk[b]))
            ref_mass = oracle.importance_update(mass0[b].cpu().numpy(), A[None], alpha)
            assert np.abs(mass[b].cpu().numpy() - ref_mass).max() <= 2e-3 * ref_mass.max(), f"mass, b={b}"


def test_shared_basis_step_full_size():
    """bench.py's `shared_basis` step at full size: one basis pair for all 64 sequences
    (basis_batch_stride = 0).  With 6.5 MB of value basis the step appends the value row next to
    the key row and expands with the plain expansion kernel, a different set of launches than
    the per-sequence headline; forcing the one-pass expansion must give the same result."""
    from paper_2603_23914_amd import binding as ap
    B, H, d, r, T = 64, 40, 128, 640, 4224
    HD = H * d
    (Ck, Cv, Bk, Bv), g = draw_cache(B, T, r, HD, 71)
    Bk1, Bv1 = Bk[0].contiguous(), Bv[0].contiguous()
    del Bk, Bv
    q = torch.randn((B, H, d), generator=g, device="cuda").to(torch.bfloat16)
    kn = torch.randn((B, HD), generator=g, device="cuda").to(torch.bfloat16)
    vn = torch.randn((B, HD), generator=g, device="cuda").to(torch.bfloat16)
    ws = workspace(ap.ap_decode_workspace_bytes(B, H, d, T, r, ap.AP_BF16))
    outs = []
    for force in (False, True):
        print(f"shared bases, 64 sequences at T={T}, value row {'in the expansion pass' if force else 'by the rule'}", flush=True)
        Ck2, Cv2 = Ck.clone(), Cv.clone()
        out = torch.empty((B, H, d), dtype=torch.float32, device="cuda")
        ap.ap_set_fused_value_min_bytes(0 if force else -1)
        try:
            ap.ap_decode_step(q, kn, vn, Ck2, Cv2, Bk1, Bv1, out, ws, T=T, sm_scale=1.0 / math.sqrt(d))
            torch.cuda.synchronize()
        finally:
            ap.ap_set_fused_value_min_bytes(-1)
        outs.append(out)
        for b in SAMPLE:
            for C, Bm, x, name in ((Ck2, Bk1, kn, "key"), (Cv2, Bv1, vn, "value")):
                c_ref = oracle.compact(P(x[b])[None], P(Bm))[0]
                assert np.abs(P(C[b, T - 1]) - c_ref).max() <= 2.0 ** -7 * np.abs(c_ref).max(), f"{name} row, b={b}"
            ref = oracle.decode_attn_absorbed(P(q[b]), P(Ck2[b, :T]), P(Cv2[b, :T]), P(Bk1), P(Bv1))
            assert_close(to_host64(out[b]), ref, "bf16", f"shared-basis step, b={b}")
        del Ck2, Cv2
    assert (outs[0] - outs[1]).abs().max() <= 2e-3 * outs[0].abs().max()


def test_fused_step_with_per_token_ranks_full_size():
    """The fused step under attention-aware ranks at the headline shape (64 sequences, r=640,
    quartile groups 640/320/128/64) in the launch the library picks there: the gathered kernel
    leaves the new token's value row to the expansion pass.  The new token sits in the first
    group in the sampled sequence 0 and in the last group in sequence 37; both value paths must
    agree with each other and with the oracle on the stored bits."""
    from paper_2603_23914_amd import binding as ap
    B, H, d, r, T0 = 64, 40, 128, 640, 4223
    T, HD = T0 + 1, H * d
    (Ck, Cv, Bk, Bv), g = draw_cache(B, T, r, HD, 67)
    q = torch.randn((B, H, d), generator=g, device="cuda").to(torch.bfloat16)
    kn = torch.randn((B, HD), generator=g, device="cuda").to(torch.bfloat16)
    vn = torch.randn((B, HD), generator=g, device="cuda").to(torch.bfloat16)
    mass = torch.rand((B, T), generator=g, device="cuda")
    mass[:, T - 1] = 2.0
    mass[37, T - 1] = 0.0
    granks, cum, den = (640, 320, 128, 64), (1, 2, 3, 4), 4
    rank = torch.empty((B, T), dtype=torch.int32, device="cuda")
    off = torch.empty((B, 5), dtype=torch.int32, device="cuda")
    idx = torch.empty((B, T), dtype=torch.int32, device="cuda")
    ap.ap_select_ranks(mass, granks, cum, den, rank, off, idx, workspace(ap.ap_select_workspace_bytes(B, T, 4)))
    torch.cuda.synchronize()
    assert int(rank[0, T - 1]) == 640 and int(rank[37, T - 1]) == 64
    ws = workspace(ap.ap_decode_workspace_bytes(B, H, d, T, r, ap.AP_BF16))
    outs = []
    for force in (-1, 1 << 50):
        print(f"per-token ranks, 64 sequences at T={T}, value row "
              f"{'by the rule (in the expansion pass)' if force < 0 else 'next to the key row'}", flush=True)
        Ck2, Cv2 = Ck.clone(), Cv.clone()
        out = torch.empty((B, H, d), dtype=torch.float32, device="cuda")
        ap.ap_set_fused_value_min_bytes(force)
        try:
            ap.ap_decode_step(q, kn, vn, Ck2, Cv2, Bk, Bv, out, ws, T=T, sm_scale=1.0 / math.sqrt(d),
                              rank_k=rank, rank_v=rank, bucket_off=off, bucket_idx=idx, F=4)
            torch.cuda.synchronize()
        finally:
            ap.ap_set_fused_value_min_bytes(-1)
        outs.append(out)
        for b in SAMPLE:
            rk = rank[b].cpu().numpy()
            for C, Bm, x, name in ((Ck2, Bk, kn, "key"), (Cv2, Bv, vn, "value")):
                c_ref = oracle.compact(P(x[b])[None], P(Bm[b]))[0]
                assert np.abs(P(C[b, T - 1]) - c_ref).max() <= 2.0 ** -7 * np.abs(c_ref).max(), f"{name} row, b={b}"
            ref = oracle.decode_attn_absorbed(P(q[b]), P(Ck2[b, :T]), P(Cv2[b, :T]), P(Bk[b]), P(Bv[b]),
                                              rank_k=rk, rank_v=rk)
            assert_close(to_host64(out[b]), ref, "bf16", f"step with per-token ranks, b={b}")
        del Ck2, Cv2
    assert (outs[0] - outs[1]).abs().max() <= 2e-3 * outs[0].abs().max()
