"""GPU parity: compaction with given bases (projection) and int8 coefficients."""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_23914_amd import workloads as wl
from gpu_util import TORCH_DT, assert_close, to_dev, to_host64, workspace

pytestmark = pytest.mark.gpu

# |c_gpu - c_exact| <= rel * |c| + abs_: one rounding to the storage type of an fp32-accumulated
# dot product (unit roundoff 2^-11 fp16, 2^-8 bf16, 2^-24 fp32) plus accumulation error
ROUND = {"f16": 2.0 ** -10, "bf16": 2.0 ** -7, "f32": 2.0 ** -20}


def run_compact(dtype, K, V, Bk, Bv, T_cap, row0, out_dtype=None):
    from paper_2603_23914_amd import binding as ap
    B, n, HD = K.shape
    r = Bk.shape[-2]
    dK, dV, dBk, dBv = (to_dev(x, dtype) for x in (K, V, Bk, Bv))
    odt = TORCH_DT[dtype] if out_dtype is None else out_dtype
    Ck = torch.zeros((B, T_cap, r), dtype=odt, device="cuda")
    Cv = torch.zeros((B, T_cap, r), dtype=odt, device="cuda")
    sk = sv = None
    if odt == torch.int8:
        sk = torch.zeros((B, T_cap, r // 64), dtype=torch.float16, device="cuda")
        sv = torch.zeros((B, T_cap, r // 64), dtype=torch.float16, device="cuda")
    ap.ap_compact(dK, dV, dBk, dBv, Ck, Cv, sk, sv, n=n, row0=row0)
    torch.cuda.synchronize()
    return Ck, Cv, sk, sv


@pytest.mark.parametrize("dtype,B,n,HD,r,shared", [
    ("f16", 2, 1, 4096, 512, False),      # append of one token (per-step case)
    ("bf16", 3, 1, 5120, 640, False),
    ("bf16", 2, 7, 1024, 192, True),      # ragged row block, shared basis
    ("f32", 1, 64, 128, 16, True),        # configuration 1 shape
    ("f16", 1, 37, 520, 80, False),       # hidden axis not a multiple of 512, r not of 64
    # 32 and more rows with the hidden axis a multiple of 64: matrix-core GEMM tiles
    ("f16", 2, 300, 1024, 192, False),    # ragged token tile, ragged column tile
    ("bf16", 1, 129, 512, 640, True),
    ("f16", 3, 128, 4096, 512, False),    # whole tiles, configuration 5's hidden axis and rank
    ("bf16", 2, 32, 5120, 80, False),     # r not a multiple of 64
])
def test_compact_projection(dtype, B, n, HD, r, shared):
    rng = wl.rng_for(11, n, HD)
    X = [wl.store(rng.standard_normal((B, n, HD)), dtype) for _ in range(2)]
    shape = (r, HD) if shared else (B, r, HD)
    Bm = [wl.store(rng.standard_normal(shape) / np.sqrt(HD), dtype) for _ in range(2)]
    T_cap, row0 = n + 5, 3
    print(f"compact {dtype} B={B} n={n} HD={HD} r={r}", flush=True)
    Ck, Cv, _, _ = run_compact(dtype, X[0], X[1], Bm[0], Bm[1], T_cap, row0)
    P = lambda a: oracle.promote(a, dtype)
    for C, Xi, Bi in ((Ck, X[0], Bm[0]), (Cv, X[1], Bm[1])):
        got = to_host64(C)
        assert (got[:, :row0] == 0).all() and (got[:, row0 + n:] == 0).all(), "rows outside the range touched"
        for b in range(B):
            ref = oracle.compact(P(Xi)[b], P(Bi) if shared else P(Bi)[b])
            err = np.abs(got[b, row0:row0 + n] - ref)
            assert (err <= ROUND[dtype] * np.abs(ref) + 1e-5 * np.abs(ref).max()).all(), err.max()


def test_quantize_i8_bit_exact():
    from paper_2603_23914_amd import binding as ap
    rng = wl.rng_for(12)
    B, T, cap, r = 2, 77, 80, 512
    C = (rng.standard_normal((B, cap, r)) * rng.uniform(1e-3, 60, size=(B, cap, 1))).astype(np.float16)
    C[0, 3, :64] = 0
    C[1, 5, 64:128] = np.float16(6e-8)            # scale underflows to 0 in fp16
    dC = to_dev(C, "f16")
    codes = torch.zeros((B, cap, r), dtype=torch.int8, device="cuda")
    scales = torch.zeros((B, cap, r // 64), dtype=torch.float16, device="cuda")
    ap.ap_quantize_i8(dC, codes, scales, T=T)
    torch.cuda.synchronize()
    for b in range(B):
        rc, rs = oracle.quantize_i8(C[b, :T])
        assert (codes[b, :T].cpu().numpy() == rc).all(), "int8 codes differ from the oracle"
        assert (scales[b, :T].cpu().numpy().view(np.uint16) == rs.view(np.uint16)).all(), "scales differ"
    assert (codes[:, T:] == 0).all()


def test_compact_to_int8_matches_quantized_projection():
    """ap_compact with int8 output == quantising its own fp16 projection (codes bit-exact)."""
    _int8_vs_quantized_projection(2, 9, 1024, 128)


def test_compact_gemm_to_int8_matches_quantized_projection():
    """The same identity on the matrix-core path (n >= 32), ragged tiles included."""
    _int8_vs_quantized_projection(2, 200, 1024, 192)


def _int8_vs_quantized_projection(B, n, HD, r):
    from paper_2603_23914_amd import binding as ap
    rng = wl.rng_for(13, n)
    K = wl.store(rng.standard_normal((B, n, HD)), "f16")
    V = wl.store(rng.standard_normal((B, n, HD)), "f16")
    Bk = wl.store(rng.standard_normal((B, r, HD)) / 32, "f16")
    Bv = wl.store(rng.standard_normal((B, r, HD)) / 32, "f16")
    Ck16, Cv16, _, _ = run_compact("f16", K, V, Bk, Bv, n, 0)
    Ck8, Cv8, sk, sv = run_compact("f16", K, V, Bk, Bv, n, 0, out_dtype=torch.int8)
    for C16, C8, s in ((Ck16, Ck8, sk), (Cv16, Cv8, sv)):
        h = C16.cpu().numpy()
        for b in range(B):
            rc, rs = oracle.quantize_i8(h[b])
            assert (C8[b].cpu().numpy() == rc).all()
            assert (s[b].cpu().numpy().view(np.uint16) == rs.view(np.uint16)).all()


def test_config5_full_size_sampled():
    """Configuration 5 at full size (T=4224, HD=4096, r=512, fp16 -> int8) in the launch shape
    of the benchmark (B=16: two generated sequences, repeated): sampled token rows against the
    fp64 projection, and the int8 codes / scales of those rows bit-exact against the oracle's
    quantiser applied to the GPU's own fp16 projection."""
    from paper_2603_23914_amd import binding as ap
    T, HD, r, B = 4224, 4096, 512, 16
    seqs = [wl.config5_sequence(b, seed=0, T=T, HD=HD, r=r) for b in range(2)]
    print("config 5: inputs generated", flush=True)
    K = np.stack([seqs[b % 2][0] for b in range(B)])
    V = np.stack([seqs[b % 2][1] for b in range(B)])
    Bk = np.stack([seqs[b % 2][2] for b in range(B)])
    Bv = np.stack([seqs[b % 2][3] for b in range(B)])
    C16k, C16v, _, _ = run_compact("f16", K, V, Bk, Bv, T, 0)
    C8k, C8v, sk, sv = run_compact("f16", K, V, Bk, Bv, T, 0, out_dtype=torch.int8)
    rows = np.unique(np.concatenate([[0, 1, 127, 128, 4095, 4096, T - 1], wl.rng_for(14).integers(0, T, 40)]))
    for b in (0, 1, 7, 15):
        for C16, C8, s, X, Bm in ((C16k, C8k, sk, K, Bk), (C16v, C8v, sv, V, Bv)):
            ref = oracle.compact(X[b][rows].astype(np.float64), Bm[b].astype(np.float64))
            got16 = C16[b].cpu().numpy()[rows]
            err = np.abs(got16.astype(np.float64) - ref)
            assert (err <= ROUND["f16"] * np.abs(ref) + 1e-5 * np.abs(ref).max()).all(), (b, err.max())
            rc, rs = oracle.quantize_i8(got16)
            assert (C8[b].cpu().numpy()[rows] == rc).all(), f"codes differ (b={b})"
            assert (s[b].cpu().numpy()[rows].view(np.uint16) == rs.view(np.uint16)).all(), f"scales differ (b={b})"


def test_config5_chain_with_true_svd_bases():
    """Configuration 5 as one chain on one sequence whose bases are the true leading right singular
    vectors (oracle.bases of the fp16 cache): prefill compaction to fp16 and to int8 on the GPU,
    then one decode step over the int8 coefficients.  Projection against the fp64 product, codes
    and scales bit for bit against the oracle's quantiser on the GPU's fp16 coefficients, decode
    output against the oracle on code * scale."""
    from paper_2603_23914_amd import binding as ap
    import math
    T, H, d, r = 1100, 8, 128, 128
    HD = H * d
    K, V, _, _ = wl.config5_sequence(0, seed=3, T=T, HD=HD, r=r)
    P = lambda x: x.astype(np.float64)
    Bk = oracle.bases(P(K), r).astype(np.float16)
    Bv = oracle.bases(P(V), r).astype(np.float16)
    print("config 5 chain: singular bases computed", flush=True)
    C16k, C16v, _, _ = run_compact("f16", K[None], V[None], Bk[None], Bv[None], T, 0)
    C8k, C8v, sk, sv = run_compact("f16", K[None], V[None], Bk[None], Bv[None], T, 0, out_dtype=torch.int8)
    for C16, C8, s, X, Bm in ((C16k, C8k, sk, K, Bk), (C16v, C8v, sv, V, Bv)):
        ref = oracle.compact(P(X), P(Bm))
        got16 = C16[0].cpu().numpy()
        err = np.abs(P(got16) - ref)
        assert (err <= ROUND["f16"] * np.abs(ref) + 1e-5 * np.abs(ref).max()).all(), err.max()
        rc, rs = oracle.quantize_i8(got16)
        assert (C8[0].cpu().numpy() == rc).all()
        assert (s[0].cpu().numpy().view(np.uint16) == rs.view(np.uint16)).all()
    # the coefficients of a singular basis carry the spectrum: column energies do not increase
    en = (P(C16k[0].cpu().numpy()) ** 2).sum(axis=0)
    assert (en[1:] <= en[:-1] * 1.02).all()
    q = wl.store(wl.rng_for(3, 77).standard_normal((1, H, d)), "f16")
    out = torch.empty((1, H, d), dtype=torch.float32, device="cuda")
    ws = workspace(ap.ap_decode_workspace_bytes(1, H, d, T, r, ap.AP_F16))
    ap.ap_decode_attn(to_dev(q, "f16"), C8k, C8v, to_dev(Bk[None], "f16"), to_dev(Bv[None], "f16"), out, ws, T=T,
                      sm_scale=1.0 / math.sqrt(d), scale_k=sk, scale_v=sv)
    torch.cuda.synchronize()
    ck = oracle.dequantize_i8(C8k[0].cpu().numpy(), sk[0].cpu().numpy())
    cv = oracle.dequantize_i8(C8v[0].cpu().numpy(), sv[0].cpu().numpy())
    ref = oracle.decode_attn_absorbed(P(q[0]), ck, cv, P(Bk), P(Bv))
    assert_close(to_host64(out[0]), ref, "f16", "config 5 chain decode")
    # and the int8 cache stands in for the uncompressed one (sanity, not equality: half of the
    # planted directions lie beyond the rank kept)
    plain = oracle.raw_attn(P(q[0]), P(K), P(V))
    assert np.abs(ref - plain).max() < 0.5 * np.abs(plain).max()
