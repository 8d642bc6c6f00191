"""GPU: the compression step (ap_compute_bases: randomized SVD of the head-merged cache, paper
Sec. 3.1 / Alg. 1 compress step) and the retrieve step as a matrix (ap_decompress).  A basis is
unique only up to signs, so the result is judged by the oracle's quality checker against the exact
truncated SVD, and against the oracle's own fp64 run of the same scheme from the same start block."""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2603_23914_amd import workloads as wl
from gpu_util import TORCH_DT, to_dev, to_host64, workspace

pytestmark = pytest.mark.gpu

ORTH_TOL = {"f16": 2e-3, "bf16": 1.6e-2}       # rows rounded to storage: |d.d - 1| <= 2 * unit roundoff-ish


def cache_matrix(seed, b, n, HD, r, dtype):
    """Keys of one sequence in configuration 5's law: 2r planted directions with spectrum i^-0.7
    plus 1 % noise, rounded to storage."""
    K, _, _, _ = wl.config5_sequence(b, seed=seed, T=n, HD=HD, r=r, dtype=dtype)
    return K


def host_bits(t, dtype):
    return t.view(torch.int16).cpu().numpy().view(np.uint16) if dtype == "bf16" else t.cpu().numpy()


def gpu_bases(X, Omega, r, q, dtype, want_sigma=True):
    from paper_2603_23914_amd import binding as ap
    B, n, HD = X.shape
    l = Omega.shape[-2]
    dX, dOm = to_dev(X, dtype), to_dev(Omega, dtype)
    Bm = torch.zeros((B, r, HD), dtype=TORCH_DT[dtype], device="cuda")
    sig = torch.zeros((B, r), dtype=torch.float32, device="cuda") if want_sigma else None
    ws = workspace(ap.ap_bases_workspace_bytes(B, n, HD, r, l - r))
    ap.ap_compute_bases(dX, dOm, Bm, ws, power_iters=q, sigma=sig)
    torch.cuda.synchronize()
    return host_bits(Bm, dtype), (sig.cpu().numpy() if want_sigma else None)


@pytest.mark.parametrize("dtype,B,n,HD,r,over,q", [
    ("f16", 2, 520, 512, 64, 32, 2),        # token count not a multiple of 64 (padded contraction)
    ("bf16", 1, 768, 1024, 128, 32, 2),
    ("f16", 1, 264, 256, 32, 16, 1),        # the paper's image rank with a light sketch
    ("bf16", 3, 512, 512, 64, 64, 0),       # no power iteration, shared start block
])
def test_bases_against_the_truncated_svd(dtype, B, n, HD, r, over, q):
    l = r + over
    X = np.stack([cache_matrix(11, b, n, HD, r, dtype) for b in range(B)])
    shared = q == 0
    om = wl.rng_for(11, 900).standard_normal((l, HD) if shared else (B, l, HD))
    Omega = wl.store(om, dtype)
    print(f"bases {dtype} B={B} n={n} HD={HD} r={r} l={l} q={q}", flush=True)
    D, sig = gpu_bases(X, Omega, r, q, dtype)
    P = lambda a: oracle.promote(a, dtype)
    for b in range(B):
        Xb, Db = P(X[b]), P(D[b])
        got = oracle.basis_quality(Xb, Db)
        Dref, sref = oracle.randomized_bases(Xb, P(Omega if shared else Omega[b]), r, q)
        ref = oracle.basis_quality(Xb, Dref)
        print(f"  b={b}: orth {got['orth_err']:.1e}  residual/optimal {got['ratio']:.4f} (fp64 scheme {ref['ratio']:.4f})"
              f"  lead capture {got['lead_capture']:.4f} ({ref['lead_capture']:.4f})", flush=True)
        assert got["orth_err"] <= ORTH_TOL[dtype]
        # as good as the same scheme in fp64 from the same start block, and near the optimum
        assert got["ratio"] <= ref["ratio"] * 1.01 + 1e-3
        assert got["lead_capture"] >= ref["lead_capture"] - 5e-3
        assert got["order_violation"] <= 1e-2
        if q >= 1:
            assert got["ratio"] <= 1.10
        # the singular values that come with the rows are the rows' own: sigma_i = ||X d_i||
        assert np.abs(sig[b] - np.sqrt(got["energy"])).max() <= 1e-2 * np.sqrt(got["energy"][0])
        # the leading rows are the fp64 scheme's rows up to sign (where the spectrum separates them)
        lead = max(4, r // 8)
        dots = np.abs(np.sum(Db[:lead] * Dref[:lead], axis=1))
        assert dots.min() >= 0.97, dots


def test_bases_degenerate_inputs():
    """A cache of exact rank 8 (fewer directions than the sketch holds): the leading rows span it,
    the rest come out as zero rows or carry no energy, nothing is NaN."""
    dtype, n, HD, r, l = "f16", 256, 256, 32, 48
    rng = wl.rng_for(12, 1)
    X = wl.store(rng.standard_normal((n, 8)) @ (np.linalg.qr(rng.standard_normal((HD, 8)))[0].T * np.arange(8, 0, -1)[:, None]), dtype)
    Omega = wl.store(rng.standard_normal((l, HD)), dtype)
    D, sig = gpu_bases(X[None], Omega, r, 1, dtype)
    Dd = oracle.promote(D[0], dtype)
    Xd = oracle.promote(X, dtype)
    assert np.isfinite(Dd).all() and np.isfinite(sig).all()
    lead = Dd[:8]
    assert np.abs(lead @ lead.T - np.eye(8)).max() <= 5e-3
    res = np.linalg.norm(Xd - (Xd @ lead.T) @ lead) ** 2 / np.linalg.norm(Xd) ** 2
    assert res <= 1e-4                                    # fp16 storage of the cache itself
    assert (np.linalg.norm(Xd @ Dd[8:].T, axis=0) <= 2e-2 * np.linalg.norm(Xd @ Dd[0])).all()


@pytest.mark.parametrize("dtype,B,T,cap,HD,r,ranked,shared", [
    ("f16", 2, 300, 320, 512, 128, False, False),
    ("bf16", 1, 333, 333, 1024, 192, True, False),
    ("f16", 3, 64, 70, 256, 64, True, True),
])
def test_decompress_is_the_retrieve_step(dtype, B, T, cap, HD, r, ranked, shared):
    from paper_2603_23914_amd import binding as ap
    rng = wl.rng_for(13, T)
    C = wl.store(rng.standard_normal((B, cap, r)), dtype)
    Bm = wl.store(rng.standard_normal((r, HD) if shared else (B, r, HD)) / math.sqrt(HD), dtype)
    rank = rng.choice([r, r // 2, 64, 16, 0], size=(B, T)).astype(np.int32) if ranked else None
    dX = torch.zeros((B, T, HD), dtype=TORCH_DT[dtype], device="cuda")
    ws = workspace(ap.ap_decompress_workspace_bytes(B, T, HD, r, ranked))
    print(f"decompress {dtype} B={B} T={T} HD={HD} r={r} ranked={ranked}", flush=True)
    ap.ap_decompress(to_dev(C, dtype), to_dev(Bm, dtype), dX, ws, T=T,
                     rank=None if rank is None else torch.from_numpy(rank).cuda())
    torch.cuda.synchronize()
    got = to_host64(dX)
    P = lambda a: oracle.promote(a, dtype)
    eps = 2.0 ** -10 if dtype == "f16" else 2.0 ** -7
    for b in range(B):
        ref = oracle.decompress(P(C)[b, :T], P(Bm) if shared else P(Bm)[b], None if rank is None else rank[b])
        assert (np.abs(got[b] - ref) <= eps * np.abs(ref) + 1e-5 * np.abs(ref).max()).all()


def test_recompression_of_a_compressed_cache_with_a_raw_tail():
    """Alg. 1's compress step when the uncompressed tail has grown: the retrieved cache
    (decompressed coefficients, then the raw rows) is decomposed again.  The new basis must serve
    the retrieved cache as well as its exact truncated SVD does, and the new coefficients must be
    its projection."""
    from paper_2603_23914_amd import binding as ap
    dtype, n0, tail, HD, r, over = "f16", 448, 64, 512, 64, 32
    P = lambda a: oracle.promote(a, dtype)
    X0 = cache_matrix(21, 0, n0, HD, r, dtype)
    Xtail = cache_matrix(21, 1, tail, HD, r, dtype)
    D0 = wl.store(oracle.bases(P(X0), r), dtype)
    C0 = wl.store(oracle.compact(P(X0), P(D0)), dtype)
    T = n0 + tail
    dXt = torch.zeros((1, T, HD), dtype=TORCH_DT[dtype], device="cuda")
    ws = workspace(ap.ap_decompress_workspace_bytes(1, n0, HD, r, False))
    head = torch.zeros((1, n0, HD), dtype=TORCH_DT[dtype], device="cuda")
    ap.ap_decompress(to_dev(C0[None], dtype), to_dev(D0[None], dtype), head, ws, T=n0)
    dXt[:, :n0] = head
    dXt[:, n0:] = to_dev(Xtail[None], dtype)
    Omega = wl.store(wl.rng_for(21, 5).standard_normal((r + over, HD)), dtype)
    D1 = torch.zeros((1, r, HD), dtype=TORCH_DT[dtype], device="cuda")
    ap.ap_compute_bases(dXt, to_dev(Omega, dtype), D1, workspace(ap.ap_bases_workspace_bytes(1, T, HD, r, over)),
                        power_iters=2)
    C1 = torch.zeros((1, T, r), dtype=TORCH_DT[dtype], device="cuda")
    ap.ap_compact(dXt, None, D1, None, C1, None, None, None, n=T, row0=0)
    torch.cuda.synchronize()
    Xt = to_host64(dXt[0])
    ref_head = oracle.decompress(P(C0), P(D0))
    assert np.abs(Xt[:n0] - ref_head).max() <= 2.0 ** -10 * np.abs(ref_head).max() * 1.01 + 1e-5
    assert (Xt[n0:] == P(Xtail)).all()
    qv = oracle.basis_quality(Xt, to_host64(D1[0]))
    print(f"  recompress: orth {qv['orth_err']:.1e} residual/optimal {qv['ratio']:.4f}", flush=True)
    assert qv["orth_err"] <= ORTH_TOL[dtype] and qv["ratio"] <= 1.10 and qv["order_violation"] <= 1e-2
    cref = oracle.compact(Xt, to_host64(D1[0]))
    assert (np.abs(to_host64(C1[0]) - cref) <= 2.0 ** -10 * np.abs(cref) + 1e-5 * np.abs(cref).max()).all()


def test_bases_full_size_one_sequence():
    """Configuration 5's shape: n = 4224 tokens, HD = 4096, r = 512 (l = 544), fp16, one sequence
    checked against the exact singular values."""
    dtype, n, HD, r, over = "f16", 4224, 4096, 512, 32
    X = cache_matrix(5, 0, n, HD, r, dtype)
    Omega = wl.store(wl.rng_for(5, 901).standard_normal((r + over, HD)), dtype)
    print("bases full size: inputs generated", flush=True)
    D, sig = gpu_bases(X[None], Omega, r, 2, dtype)
    Xd, Dd = oracle.promote(X, dtype), oracle.promote(D[0], dtype)
    print("bases full size: GPU done, exact singular values next", flush=True)
    S = np.linalg.svd(Xd, compute_uv=False)
    C = Xd @ Dd.T
    residual = np.linalg.norm(Xd - C @ Dd) ** 2
    optimal = np.sum(S[r:] ** 2)
    energy = (C ** 2).sum(axis=0)
    lead = (np.cumsum(energy) / np.cumsum(S[:r] ** 2)).min()
    orth = np.abs(Dd @ Dd.T - np.eye(r)).max()
    print(f"  orth {orth:.1e} residual/optimal {residual / optimal:.4f} lead capture {lead:.4f}", flush=True)
    assert orth <= ORTH_TOL[dtype] and residual / optimal <= 1.10 and lead >= 0.97
    assert np.max(np.diff(energy)) <= 1e-2 * energy[0]
    assert np.abs(sig[0] - np.sqrt(energy)).max() <= 1e-2 * np.sqrt(energy[0])


def test_algorithm1_loop_with_new_bases_at_every_trigger():
    """Alg. 1 end to end on the GPU entry points: the prompt's keys and values are decomposed
    (ap_compute_bases) and projected (ap_compact); generated tokens wait in the uncompressed
    segment and every step attends to both under one softmax; once T_p tokens wait, the retrieved
    cache (ap_decompress) and the tail are decomposed AGAIN, with new bases, and the tail starts
    over.  Bases are unique only up to signs, so the oracle takes what the GPU stored (bases and
    coefficients, bit for bit) and checks (a) every step's output against attention over the
    union by its definition, (b) at every compression that the new bases serve the retrieved
    cache as well as its exact truncated SVD and that the coefficients are its projection."""
    from paper_2603_23914_amd import binding as ap
    dtype, H, d, r, over, n0, T_p, steps = "f16", 8, 64, 64, 32, 320, 8, 17     # token counts stay multiples of 8
    HD, T_cap = H * d, n0 + steps + 8
    P = lambda a: oracle.promote(a, dtype)
    tdt = TORCH_DT[dtype]
    Kp, Vp, _, _ = wl.config5_sequence(0, seed=31, T=n0 + steps, HD=HD, r=r, dtype=dtype)
    K_all, V_all = Kp, Vp
    Omega = to_dev(wl.store(wl.rng_for(31, 5).standard_normal((r + over, HD)), dtype), dtype)
    dBk = torch.zeros((1, r, HD), dtype=tdt, device="cuda")
    dBv = torch.zeros_like(dBk)
    dCk = torch.zeros((1, T_cap, r), dtype=tdt, device="cuda")
    dCv = torch.zeros_like(dCk)
    dK = torch.zeros((1, T_p, HD), dtype=tdt, device="cuda")
    dV = torch.zeros_like(dK)
    scale = 1.0 / math.sqrt(d)
    out_c = torch.empty((1, H, d), dtype=torch.float32, device="cuda")
    lse_c = torch.empty((1, H), dtype=torch.float32, device="cuda")
    out_u, lse_u, out = torch.empty_like(out_c), torch.empty_like(lse_c), torch.empty_like(out_c)

    def compress(dXk, dXv, n):
        """bases of the n rows of dXk / dXv, then their coefficients: rows 0..n-1 of the cache"""
        wsb = workspace(ap.ap_bases_workspace_bytes(1, n, HD, r, over))
        ap.ap_compute_bases(dXk, Omega, dBk, wsb, power_iters=2)
        ap.ap_compute_bases(dXv, Omega, dBv, wsb, power_iters=2)
        ap.ap_compact(dXk, dXv, dBk, dBv, dCk, dCv, n=n, row0=0)
        torch.cuda.synchronize()
        for X, Bm, C, name in ((dXk, dBk, dCk, "keys"), (dXv, dBv, dCv, "values")):
            Xh, Dh = to_host64(X[0, :n]), to_host64(Bm[0])
            qv = oracle.basis_quality(Xh, Dh)
            print(f"  compress {name} n={n}: orth {qv['orth_err']:.1e} residual/optimal {qv['ratio']:.4f}", flush=True)
            assert qv["orth_err"] <= ORTH_TOL[dtype] and qv["ratio"] <= 1.10, name
            cref = oracle.compact(Xh, Dh)
            assert (np.abs(to_host64(C[0, :n]) - cref) <= 2.0 ** -10 * np.abs(cref) + 1e-5 * np.abs(cref).max()).all()

    compress(to_dev(K_all[None, :n0], dtype), to_dev(V_all[None, :n0], dtype), n0)
    T, T_u, compressions = n0, 0, 1
    rng = wl.rng_for(31, 77)
    for step in range(steps):
        row = n0 + step
        ap.ap_raw_append(to_dev(K_all[None, row], dtype), to_dev(V_all[None, row], dtype), dK, dV, row=T_u)
        T_u += 1
        q = wl.store(rng.standard_normal((1, H, d)), dtype)
        print(f"Alg. 1 loop step {step}: {T} compressed + {T_u} raw tokens", flush=True)
        ap.ap_decode_attn(to_dev(q, dtype), dCk, dCv, dBk, dBv, out_c,
                          workspace(ap.ap_decode_workspace_bytes(1, H, d, T, r, ap.AP_F16)), T=T, sm_scale=scale, lse=lse_c)
        ap.ap_raw_attn(to_dev(q, dtype), dK, dV, out_u, workspace(ap.ap_raw_workspace_bytes(1, H, d, T_u)), T_u=T_u,
                       sm_scale=scale, lse=lse_u)
        ap.ap_merge_segments(out_c, lse_c, out_u, lse_u, out)
        torch.cuda.synchronize()
        ref = oracle.decode_attn_segments(P(q)[0], [
            dict(Ck=to_host64(dCk[0, :T]), Cv=to_host64(dCv[0, :T]), Bk=to_host64(dBk[0]), Bv=to_host64(dBv[0])),
            dict(K=to_host64(dK[0, :T_u]), V=to_host64(dV[0, :T_u]))])
        err = np.abs(to_host64(out[0]) - ref).max()
        assert err <= 2e-3 * np.abs(ref).max(), f"step {step}: {err:.2e}"
        if T_u == T_p:                  # the trigger: retrieve, join the tail, decompose again
            n = T + T_u
            dXk = torch.zeros((1, n, HD), dtype=tdt, device="cuda")
            dXv = torch.zeros_like(dXk)
            wsd = workspace(ap.ap_decompress_workspace_bytes(1, T, HD, r, False))
            headk = torch.zeros((1, T, HD), dtype=tdt, device="cuda")
            headv = torch.zeros_like(headk)
            ap.ap_decompress(dCk, dBk, headk, wsd, T=T)
            ap.ap_decompress(dCv, dBv, headv, wsd, T=T)
            dXk[:, :T], dXk[:, T:] = headk, dK[:, :T_u]
            dXv[:, :T], dXv[:, T:] = headv, dV[:, :T_u]
            compress(dXk, dXv, n)
            T, T_u = n, 0
            compressions += 1
    assert compressions == 3 and T == n0 + 16 and T_u == 1
