"""The decode calls enqueue kernels only (no allocation, no memset, no synchronisation), so a
caller may capture them in a HIP graph.  Capture a fused step and an attend-only call with
logits out, replay them several times with eager work in between, and compare every replay
with the eager result bit for bit."""
import math

import numpy as np
import pytest
import torch

from paper_2603_23914_amd import workloads as wl
from gpu_util import TORCH_DT, to_dev, workspace

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype,B,H,d,r,T", [("bf16", 2, 40, 128, 640, 301), ("f16", 3, 32, 128, 128, 200)])
def test_decode_calls_in_a_captured_graph(dtype, B, H, d, r, T, value_path):
    from paper_2603_23914_amd import binding as ap
    case = wl.decode_case(dtype, B, H, d, r, T - 1, steps=1, seed=71, append=True)
    P = lambda x: __import__("oracle").promote(x, dtype)
    kn, vn = wl.step_new_token(case, 0, P(case.Bk), P(case.Bv))
    q = wl.step_query(case, 0)
    dq, dCk0, dCv0, dBk, dBv, dkn, dvn = (to_dev(x, dtype) for x in (q, case.Ck, case.Cv, case.Bk, case.Bv, kn, vn))
    ws = workspace(ap.ap_decode_workspace_bytes(B, H, d, T, r, ap._DT[TORCH_DT[dtype]]))
    scale = 1.0 / math.sqrt(d)

    def run(Ck, Cv, out, lse, scores):
        ap.ap_decode_step(dq, dkn, dvn, Ck, Cv, dBk, dBv, out, ws, T=T, sm_scale=scale)
        ap.ap_decode_attn(dq, Ck, Cv, dBk, dBv, out, ws, T=T, sm_scale=scale, lse=lse, scores=scores)

    def fresh():
        return (dCk0.clone(), dCv0.clone(), torch.zeros((B, H, d), dtype=torch.float32, device="cuda"),
                torch.zeros((B, H), dtype=torch.float32, device="cuda"),
                torch.zeros((B, case.T_cap, H), dtype=torch.float32, device="cuda"))

    eager = fresh()
    run(*eager)
    torch.cuda.synchronize()

    cap = fresh()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run(*cap)                                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        run(*cap)
    for rep in range(3):
        for t in cap[2:]:
            t.fill_(float("nan"))                    # eager work between the replays
        cap[0].copy_(dCk0)
        cap[1].copy_(dCv0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(eager, cap):
            assert torch.equal(a.view(torch.int16) if a.dtype != torch.float32 else a,
                               b.view(torch.int16) if b.dtype != torch.float32 else b), f"replay {rep}"


@pytest.mark.parametrize("B,T,r,H", [(2, 700, 256, 16), (1, 25000, 128, 8)])
def test_attention_aware_step_in_a_captured_graph(B, T, r, H):
    """The whole attention-aware step as one graph: group selection (the second case is long
    enough for the row to be split over workgroups, whose kernels clear their own counters),
    fused step under per-token ranks with logits out, importance update.  Every replay must
    reproduce the eager run bit for bit, with the importance restored in between."""
    from paper_2603_23914_amd import binding as ap
    dtype, d = "f16", 64
    HD = H * d
    g = torch.Generator(device="cuda")
    g.manual_seed(73)
    T_cap = T + 8
    Ck0 = torch.randn((B, T_cap, r), generator=g, device="cuda").to(torch.float16)
    Cv0 = torch.randn((B, T_cap, r), generator=g, device="cuda").to(torch.float16)
    Bk = (torch.randn((B, r, HD), generator=g, device="cuda") / math.sqrt(HD)).to(torch.float16)
    Bv = (torch.randn((B, r, HD), generator=g, device="cuda") / math.sqrt(HD)).to(torch.float16)
    q = torch.randn((B, H, d), generator=g, device="cuda").to(torch.float16)
    kn = torch.randn((B, HD), generator=g, device="cuda").to(torch.float16)
    vn = torch.randn((B, HD), generator=g, device="cuda").to(torch.float16)
    mass0 = torch.exp(2.0 * torch.randn((B, T), generator=g, device="cuda")) * 1e-3
    mass0[:, T - 1] = 10.0                                # the token being appended: first group
    granks, cum, den, F = (r, r // 2, 32), (1, 2, 4), 4, 3
    ws = workspace(ap.ap_decode_workspace_bytes(B, H, d, T, r, ap.AP_F16))
    wsel = workspace(ap.ap_select_workspace_bytes(B, T, F))
    scale = 1.0 / math.sqrt(d)

    def fresh():
        return dict(Ck=Ck0.clone(), Cv=Cv0.clone(), mass=mass0.clone(),
                    rank=torch.zeros((B, T), dtype=torch.int32, device="cuda"),
                    off=torch.zeros((B, F + 1), dtype=torch.int32, device="cuda"),
                    idx=torch.zeros((B, T), dtype=torch.int32, device="cuda"),
                    out=torch.zeros((B, H, d), dtype=torch.float32, device="cuda"),
                    lse=torch.zeros((B, H), dtype=torch.float32, device="cuda"),
                    scores=torch.zeros((B, T_cap, H), dtype=torch.float32, device="cuda"))

    def run(s):
        ap.ap_select_ranks(s["mass"], granks, cum, den, s["rank"], s["off"], s["idx"], wsel)
        ap.ap_decode_step(q, kn, vn, s["Ck"], s["Cv"], Bk, Bv, s["out"], ws, T=T, sm_scale=scale,
                          rank_k=s["rank"], rank_v=s["rank"], bucket_off=s["off"], bucket_idx=s["idx"], F=F,
                          lse=s["lse"], scores=s["scores"])
        ap.ap_update_importance(s["scores"], s["lse"], s["mass"], T=T, alpha=0.9)

    print(f"attention-aware step in a graph: B={B} T={T} r={r}", flush=True)
    eager = fresh()
    run(eager)
    torch.cuda.synchronize()
    cap = fresh()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run(cap)                                    # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    cap["mass"].copy_(mass0)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        run(cap)
    for rep in range(3):
        for k in ("out", "lse", "scores"):
            cap[k].fill_(float("nan"))               # eager work between the replays
        for k in ("rank", "off", "idx"):
            cap[k].fill_(-1)
        cap["Ck"].copy_(Ck0)
        cap["Cv"].copy_(Cv0)
        cap["mass"].copy_(mass0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k in eager:
            a, b = eager[k], cap[k]
            if k == "scores":                        # rows beyond T are not written
                a, b = a[:, :T], b[:, :T]
            if a.dtype == torch.float16:
                a, b = a.view(torch.int16), b.view(torch.int16)
            assert torch.equal(a, b), f"replay {rep}: {k}"
