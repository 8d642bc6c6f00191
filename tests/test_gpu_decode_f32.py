"""GPU parity: fp32 decode path (configuration 1 and small ragged cases)."""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2603_23914_amd import workloads as wl
from gpu_util import assert_close, to_dev, to_host64, workspace

pytestmark = pytest.mark.gpu


def run_f32(q, Ck, Cv, Bk, Bv, T, rank_k=None, rank_v=None, sm_scale=None, want_lse=False):
    from paper_2603_23914_amd import binding as ap
    B, H, d = q.shape
    r = Ck.shape[2]
    dq, dCk, dCv, dBk, dBv = (to_dev(np.asarray(x, np.float32), "f32") for x in (q, Ck, Cv, Bk, Bv))
    out = torch.empty((B, H, d), dtype=torch.float32, device="cuda")
    lse = torch.empty((B, H), dtype=torch.float32, device="cuda") if want_lse else None
    ws = workspace(ap.ap_decode_workspace_bytes(B, H, d, T, r, ap.AP_F32))
    rk = None if rank_k is None else torch.from_numpy(np.asarray(rank_k, np.int32)).cuda()
    rv = None if rank_v is None else torch.from_numpy(np.asarray(rank_v, np.int32)).cuda()
    ap.ap_decode_attn(dq, dCk, dCv, dBk, dBv, out, ws, T=T,
                      sm_scale=(1.0 / math.sqrt(d) if sm_scale is None else sm_scale),
                      rank_k=rk, rank_v=rv, lse=lse)
    torch.cuda.synchronize()
    return (to_host64(out), to_host64(lse)) if want_lse else to_host64(out)


def test_config1_tiny_fp32():
    c = wl.config1(0)
    K, V, q = c["K"], c["V"], c["q"]
    r = c["r"]
    Bk = oracle.bases(K, r).astype(np.float32)
    Bv = oracle.bases(V, r).astype(np.float32)
    # stored fp32 coefficients come from the oracle's projection: both sides read the same bits
    Ck = oracle.compact(K, Bk).astype(np.float32)
    Cv = oracle.compact(V, Bv).astype(np.float32)
    q32 = q.astype(np.float32)
    ref, ref_lse = oracle.decode_attn(q32, Ck, Cv, Bk, Bv, return_lse=True)
    got, lse = run_f32(q32[None], Ck[None], Cv[None], Bk, Bv, c["T"], want_lse=True)
    assert_close(got[0], ref, "f32", "config 1")
    assert np.abs(lse[0] - ref_lse).max() < 1e-5 * max(1.0, np.abs(ref_lse).max())


@pytest.mark.parametrize("seed", [0, 1])
def test_fp32_ragged_batched(seed):
    rng = np.random.default_rng(seed)
    B, H, d, T, r, cap = 3, 5, 24, 301, 40, 310
    q = rng.standard_normal((B, H, d)).astype(np.float32)
    Ck = rng.standard_normal((B, cap, r)).astype(np.float32)
    Cv = rng.standard_normal((B, cap, r)).astype(np.float32)
    Bk = (rng.standard_normal((B, r, H * d)) / math.sqrt(r)).astype(np.float32)
    Bv = rng.standard_normal((B, r, H * d)).astype(np.float32)
    rk = rng.integers(0, r + 1, size=(B, T)).astype(np.int32)
    rv = rng.integers(0, r + 1, size=(B, T)).astype(np.int32)
    ref = oracle.decode_attn_batched(q, Ck, Cv, Bk, Bv, T, rk, rv)
    got = run_f32(q, Ck, Cv, Bk, Bv, T, rk, rv)
    assert_close(got, ref, "f32", "fp32 ragged")
    # shared basis (batch stride 0) and uniform rank
    ref2 = oracle.decode_attn_batched(q, Ck, Cv, Bk[0], Bv[0], T)
    got2 = run_f32(q, Ck, Cv, Bk[0], Bv[0], T)
    assert_close(got2, ref2, "f32", "fp32 shared basis")
