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
