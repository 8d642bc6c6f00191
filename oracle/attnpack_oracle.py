"""Plain fp64 CPU oracle for decode attention over a multi-head-compacted,
low-rank KV cache (AttentionPack).

TEST INFRASTRUCTURE ONLY: slow, obviously-correct NumPy.  The product (the HIP
library and its Python binding) never imports this file and this file imports
nothing from the product.

Notation follows the paper: a layer's cache K, V in R^{T x HD} (heads merged
along the hidden axis, Sec. 3.1) is stored as coefficients  Kbar, Vbar in
R^{T x R}  ("C_k", "C_v" here) and decompression matrices  D_k, D_v in
R^{R x HD}  ("B_k", "B_v", the bases).  Head h owns hidden columns
[h*d, (h+1)*d).

Grouped-query attention (Sec. 4.5: models whose H query heads share H_kv < H
key/value heads): the cache and the bases then have H_kv*d hidden columns and
query head h reads the slice of key/value head h // (H / H_kv).  Functions
that take `kv_heads` implement this; None means H_kv = H.

Every function works on ONE sequence of ONE layer unless it says "batched".
All arithmetic is float64 except `quantize_i8`, whose recipe fixes fp32/fp16.
"""
from __future__ import annotations

import math
from typing import Optional, Sequence, Tuple

import numpy as np

# --------------------------------------------------------------------------
# exact promotion of stored bits to float64
# --------------------------------------------------------------------------

def promote(x: np.ndarray, dtype: str) -> np.ndarray:
    """Stored array -> float64, exactly.

    dtype: "f32" (np.float32 array), "f16" (np.float16 array) or "bf16"
    (np.uint16 array holding bfloat16 bit patterns: a bfloat16 is the upper
    half of an IEEE binary32, so shifting left by 16 bits gives its value).
    """
    if dtype == "f32":
        assert x.dtype == np.float32
        return x.astype(np.float64)
    if dtype == "f16":
        assert x.dtype == np.float16
        return x.astype(np.float64)
    if dtype == "bf16":
        assert x.dtype == np.uint16
        return (x.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    raise ValueError(f"unknown dtype tag {dtype!r}")


# --------------------------------------------------------------------------
# compression (Sec. 3.1): K ~= Kbar D_k
# --------------------------------------------------------------------------

def bases(X: np.ndarray, r: int) -> np.ndarray:
    """Decompression matrix D in R^{r x HD} of the head-merged cache X [T, HD].

    Sec. 3.1: low-rank SVD of the matrix with all heads concatenated along the
    hidden axis.  Rows of D are the r leading right singular vectors (plain
    SVD, no centring), ordered by decreasing singular value.
    """
    X = np.asarray(X, dtype=np.float64)
    _, _, vt = np.linalg.svd(X, full_matrices=False)
    return vt[:r].copy()


def compact(X: np.ndarray, D: np.ndarray) -> np.ndarray:
    """Coefficients Kbar = X D^T  [T, r]  for a given decompression matrix.

    Sec. 3.1: the first factor of the decomposition has its columns scaled by
    the singular values, i.e. Kbar = U_r Sigma_r; for D with orthonormal rows
    (right singular vectors) that equals X D^T.  The same projection is used
    when a token is appended to a cache whose basis is already fixed.
    """
    return np.asarray(X, dtype=np.float64) @ np.asarray(D, dtype=np.float64).T


def randomized_bases(X: np.ndarray, Omega: np.ndarray, r: int, power_iters: int) -> Tuple[np.ndarray, np.ndarray]:
    """Randomized low-rank SVD of the head-merged cache X [T, HD] (the appendix's
    implementation details name randomized SVD for the compression step of
    Sec. 3.1 / Alg. 1), written out from the published range-finder scheme on the
    ROW space, the start block passed in:

      P <- Omega                      [l, HD], l = r + oversampling, any full-rank start
      repeat power_iters + 1 times:   P <- orthonormal rows spanning rows of (P X^T) X
      Z <- X P^T                      [T, l]   (Rayleigh-Ritz in the span of P)
      Z = U S W^T  (plain SVD)        D <- (W^T P)[:r],  sigma <- S[:r]

    Returns (D [r, HD] with orthonormal rows ordered by decreasing sigma, sigma [r]).
    With Omega spanning the leading l right singular vectors, or as power_iters
    grows, D tends to `bases(X, r)` up to the sign of each row.
    """
    X = np.asarray(X, np.float64)
    P = np.asarray(Omega, np.float64)
    for _ in range(int(power_iters) + 1):
        M = (P @ X.T) @ X                                  # [l, HD]
        Q, _ = np.linalg.qr(M.T)                           # orthonormal columns spanning rows of M
        P = Q.T
    Z = X @ P.T
    _, S, Wt = np.linalg.svd(Z, full_matrices=False)
    return (Wt @ P)[:r].copy(), S[:r].copy()


def basis_quality(X: np.ndarray, D: np.ndarray) -> dict:
    """How good a rank-r decompression matrix D [r, HD] is for the cache X [T, HD],
    against what the definition (truncated SVD, Sec. 3.1) achieves.  A basis is
    only determined up to signs (and rotations inside repeated singular values),
    so it is judged by what is unique:

      orth_err        max |D D^T - I|                      rows orthonormal
      residual        ||X - (X D^T) D||_F^2                 what the cache loses
      optimal         sum_{i>r} sigma_i^2                   Eckart-Young minimum
      ratio           residual / optimal                    >= 1 for orthonormal rows
      energy          e_i = ||X d_i||^2                     per row of D
      lead_capture    min_k sum_{i<=k} e_i / sum_{i<=k} sigma_i^2   (<= 1, Ky Fan): every
                      leading-k truncation of the basis (attention-aware decompression
                      reads leading columns) is as good as the best rank-k one
      order_violation max_i (e_{i+1} - e_i) / e_1, positive part   rows ordered by energy
      sin_angle       sine of the largest principal angle between the row space of D
                      and the span of the r leading right singular vectors
    """
    X = np.asarray(X, np.float64)
    D = np.asarray(D, np.float64)
    r = D.shape[0]
    _, S, Vt = np.linalg.svd(X, full_matrices=False)
    C = X @ D.T
    residual = float(np.linalg.norm(X - C @ D) ** 2)
    optimal = float(np.sum(S[r:] ** 2))
    energy = (C ** 2).sum(axis=0)
    lead = np.cumsum(energy) / np.cumsum(S[:r] ** 2)
    Q, _ = np.linalg.qr(D.T)                               # orthonormal basis of the row space of D
    out_of_span = Q - Vt[:r].T @ (Vt[:r] @ Q)
    return {
        "orth_err": float(np.abs(D @ D.T - np.eye(r)).max()),
        "residual": residual,
        "optimal": optimal,
        "ratio": residual / optimal if optimal > 0 else (1.0 if residual == 0 else np.inf),
        "energy": energy,
        "lead_capture": float(lead.min()),
        "order_violation": float(max(0.0, np.max(np.diff(energy), initial=0.0)) / energy[0]),
        "sin_angle": float(np.linalg.norm(out_of_span, 2)),
        "sigma": S,
    }


def decompress(C: np.ndarray, D: np.ndarray, rank: Optional[np.ndarray] = None) -> np.ndarray:
    """Alg. 1 "retrieve cache" for a compressed segment on its own: row t is
    C[t, :rank[t]] D[:rank[t]] (rank None = all r columns).  [T, HD]."""
    C = np.asarray(C, np.float64)
    return _partial_decompress(C, np.asarray(D, np.float64), _ranks(rank, C.shape[0], C.shape[1]))


# --------------------------------------------------------------------------
# decode attention (Alg. 1, retrieve / scores / output steps)
# --------------------------------------------------------------------------

def _ranks(rank: Optional[np.ndarray], T: int, r: int) -> np.ndarray:
    if rank is None:
        return np.full(T, r, dtype=np.int64)
    rank = np.asarray(rank).astype(np.int64)
    assert rank.shape == (T,)
    assert rank.min() >= 0 and rank.max() <= r
    return rank


def _partial_decompress(C: np.ndarray, D: np.ndarray, rank: np.ndarray) -> np.ndarray:
    """Alg. 1 "retrieve cache": token t is rebuilt from its leading rank[t]
    coefficient columns and the leading rank[t] rows of D."""
    T = C.shape[0]
    X = np.zeros((T, D.shape[1]), dtype=np.float64)
    for t in range(T):
        rt = int(rank[t])
        X[t] = C[t, :rt] @ D[:rt, :]
    return X


def _kv_slice(h: int, H: int, d: int, kv_heads: Optional[int]) -> slice:
    """Hidden columns that query head h reads (grouped-query attention: consecutive
    groups of H / H_kv query heads share one key/value head)."""
    Hkv = H if kv_heads is None else int(kv_heads)
    assert Hkv >= 1 and H % Hkv == 0
    g = h // (H // Hkv)
    return slice(g * d, (g + 1) * d)


def _softmax_rows(s: np.ndarray) -> np.ndarray:
    m = s.max(axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / e.sum(axis=-1, keepdims=True)


def attention_probs(q, Ck, Bk, rank_k=None, sm_scale=None, kv_heads=None) -> np.ndarray:
    """Attention weights A [H, T] of one decode query (Alg. 1 score step):
    softmax over all cached tokens of q_h . Ktilde_h[t] / sqrt(d)."""
    q = np.asarray(q, np.float64)
    Ck = np.asarray(Ck, np.float64)
    Bk = np.asarray(Bk, np.float64)
    H, d = q.shape
    T, r = Ck.shape
    if sm_scale is None:
        sm_scale = 1.0 / math.sqrt(d)
    Kt = _partial_decompress(Ck, Bk, _ranks(rank_k, T, r))
    s = np.empty((H, T))
    for h in range(H):
        s[h] = Kt[:, _kv_slice(h, H, d, kv_heads)] @ q[h] * sm_scale
    return _softmax_rows(s)


def decode_attn(q, Ck, Cv, Bk, Bv, rank_k=None, rank_v=None, sm_scale=None,
                return_lse: bool = False, kv_heads=None):
    """DEFINITION FORM: reconstruct, then textbook softmax attention.

    q [H, d]; Ck, Cv [T, r]; Bk, Bv [r, H*d]; rank_k, rank_v [T] ints or None
    (None = every token at full rank r).  Returns out [H, d] float64 (the
    product A Vtilde of Alg. 1, before the output projection W_o) and, if asked,
    lse [H] = log sum_t exp(scaled score).
    """
    q = np.asarray(q, np.float64)
    Ck = np.asarray(Ck, np.float64)
    Cv = np.asarray(Cv, np.float64)
    Bk = np.asarray(Bk, np.float64)
    Bv = np.asarray(Bv, np.float64)
    H, d = q.shape
    T, r = Ck.shape
    HDkv = (H if kv_heads is None else int(kv_heads)) * d
    assert Cv.shape == (T, r) and Bk.shape == (r, HDkv) and Bv.shape == (r, HDkv)
    if sm_scale is None:
        sm_scale = 1.0 / math.sqrt(d)
    Kt = _partial_decompress(Ck, Bk, _ranks(rank_k, T, r))
    Vt = _partial_decompress(Cv, Bv, _ranks(rank_v, T, r))
    out = np.empty((H, d))
    lse = np.empty(H)
    for h in range(H):
        sl = _kv_slice(h, H, d, kv_heads)
        s = Kt[:, sl] @ q[h] * sm_scale                          # [T]
        m = s.max()
        e = np.exp(s - m)
        z = e.sum()
        p = e / z
        out[h] = p @ Vt[:, sl]
        lse[h] = m + math.log(z)
    return (out, lse) if return_lse else out


def decode_attn_absorbed(q, Ck, Cv, Bk, Bv, rank_k=None, rank_v=None, sm_scale=None,
                         return_lse: bool = False, kv_heads=None):
    """ABSORBED FORM: the same result by associativity, never forming K, V.

    q'_h = D_k[:, head h] q_h;  score[h,t] = Kbar[t,:rk_t] . q'_h[:rk_t];
    u_h[j] = sum_{t: rv_t > j} p[h,t] Vbar[t,j];  out_h = u_h D_v[:, head h].
    """
    q = np.asarray(q, np.float64)
    Ck = np.asarray(Ck, np.float64)
    Cv = np.asarray(Cv, np.float64)
    Bk = np.asarray(Bk, np.float64)
    Bv = np.asarray(Bv, np.float64)
    H, d = q.shape
    T, r = Ck.shape
    if sm_scale is None:
        sm_scale = 1.0 / math.sqrt(d)
    rk = _ranks(rank_k, T, r)
    rv = _ranks(rank_v, T, r)
    cols = np.arange(r)
    Mk = (cols[None, :] < rk[:, None])          # [T, r] column kept for K
    Mv = (cols[None, :] < rv[:, None])
    Ckm = np.where(Mk, Ck, 0.0)
    Cvm = np.where(Mv, Cv, 0.0)
    out = np.empty((H, d))
    lse = np.empty(H)
    for h in range(H):
        sl = _kv_slice(h, H, d, kv_heads)
        qp = Bk[:, sl] @ q[h]                    # [r]
        s = Ckm @ qp * sm_scale
        m = s.max()
        e = np.exp(s - m)
        z = e.sum()
        u = (e / z) @ Cvm                        # [r]
        out[h] = u @ Bv[:, sl]
        lse[h] = m + math.log(z)
    return (out, lse) if return_lse else out


def decode_attn_batched(q, Ck, Cv, Bk, Bv, T: int, rank_k=None, rank_v=None,
                        sm_scale=None, absorbed: bool = False, kv_heads=None) -> np.ndarray:
    """Batched wrapper.  q [B,H,d]; Ck, Cv [B,T_cap,r] (rows >= T ignored);
    Bk, Bv [B,r,HD] or [r,HD] (shared); ranks [B,T] or None.  -> [B,H,d]."""
    fn = decode_attn_absorbed if absorbed else decode_attn
    B = q.shape[0]
    out = np.empty(q.shape, dtype=np.float64)
    for b in range(B):
        bk = Bk[b] if Bk.ndim == 3 else Bk
        bv = Bv[b] if Bv.ndim == 3 else Bv
        rk = None if rank_k is None else rank_k[b][:T]
        rv = None if rank_v is None else rank_v[b][:T]
        out[b] = fn(q[b], Ck[b, :T], Cv[b, :T], bk, bv, rk, rv, sm_scale, kv_heads=kv_heads)
    return out


# --------------------------------------------------------------------------
# the cache the paper's Alg. 1 keeps: compressed segments next to an
# uncompressed one (text tokens, and new tokens until the next compression)
# --------------------------------------------------------------------------

def raw_attn(q, K, V, sm_scale=None, return_lse: bool = False, kv_heads=None):
    """Textbook softmax attention of one decode query over an uncompressed
    cache K, V [T, H*d] (the C_u of Alg. 1).  T = 0 gives out = 0, lse = -inf."""
    q = np.asarray(q, np.float64)
    K = np.asarray(K, np.float64)
    V = np.asarray(V, np.float64)
    H, d = q.shape
    if sm_scale is None:
        sm_scale = 1.0 / math.sqrt(d)
    out = np.zeros((H, d))
    lse = np.full(H, -np.inf)
    if K.shape[0] > 0:
        for h in range(H):
            sl = _kv_slice(h, H, d, kv_heads)
            s = K[:, sl] @ q[h] * sm_scale
            m = s.max()
            e = np.exp(s - m)
            out[h] = (e / e.sum()) @ V[:, sl]
            lse[h] = m + math.log(e.sum())
    return (out, lse) if return_lse else out


def decode_attn_segments(q, segments, sm_scale=None, return_lse: bool = False, kv_heads=None):
    """Alg. 1's attention over a cache made of several segments, by its
    definition: every compressed segment is (partially) decompressed, all keys
    and all values are concatenated along the token axis (Ktilde = (+)_f
    Kbar[m_f, :R_f] D_k[:R_f] (+) K), and one softmax runs over the lot.

    segments: sequence of dicts; the key side and the value side of a segment
    are given independently, each either compressed or uncompressed:
      keys    {"Ck", "Bk"[, "rank_k"]}  coefficients and own basis   or  {"K"} [T, H_kv*d]
      values  {"Cv", "Bv"[, "rank_v"]}                                or  {"V"} [T, H_kv*d]
    A segment with compressed keys and raw values is the key-only compression
    of the text-domain experiment (appendix "Analysis of Textual Token
    Compression": R_k = 64, values kept).
    """
    q = np.asarray(q, np.float64)
    H, d = q.shape
    HDkv = (H if kv_heads is None else int(kv_heads)) * d

    def side(seg, raw, coef, basis, rank):
        if raw in seg:
            return np.asarray(seg[raw], np.float64).reshape(-1, HDkv)
        C = np.asarray(seg[coef], np.float64)
        T, r = C.shape
        return _partial_decompress(C, np.asarray(seg[basis], np.float64), _ranks(seg.get(rank), T, r))

    Ks, Vs = [], []
    for seg in segments:
        Ks.append(side(seg, "K", "Ck", "Bk", "rank_k"))
        Vs.append(side(seg, "V", "Cv", "Bv", "rank_v"))
        if Ks[-1].shape[0] != Vs[-1].shape[0]:
            raise ValueError("a segment's keys and values must cover the same tokens")
    return raw_attn(q, np.concatenate(Ks, axis=0), np.concatenate(Vs, axis=0), sm_scale, return_lse,
                    kv_heads=kv_heads)


def merge_segments(outs, lses):
    """Outputs and log-sum-exps of attention over disjoint token sets ->
    those of attention over their union: softmax weights of the union are the
    per-set weights scaled by exp(lse_i - lse), lse = log sum_i exp(lse_i).
    outs [N, H, d], lses [N, H]; a set may be empty (lse = -inf)."""
    outs = np.asarray(outs, np.float64)
    lses = np.asarray(lses, np.float64)
    m = lses.max(axis=0)                                  # [H]
    w = np.exp(lses - m[None, :])                         # [N, H]
    z = w.sum(axis=0)
    out = (w[:, :, None] * outs).sum(axis=0) / z[:, None]
    return out, m + np.log(z)


# --------------------------------------------------------------------------
# attention-aware rank groups (Sec. 3.2; Alg. 1, group-selection step)
# --------------------------------------------------------------------------

def select_ranks(mass: np.ndarray, group_rank: Sequence[int], cum_num: Sequence[int],
                 den: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Tokens ordered by importance, cut into F groups; group f decodes at
    rank group_rank[f] (group 0 = most important = the compression rank).

    Reading fixed for what the paper leaves open: order = (mass descending,
    token index ascending); group f holds sorted positions
    [floor(T*cum_num[f-1]/den), floor(T*cum_num[f]/den)) with cum_num[F-1]==den;
    inside a group token indices are listed ascending.

    Returns (rank [T] int32, bucket_off [F+1] int32, bucket_idx [T] int32).
    """
    mass = np.asarray(mass)
    assert mass.ndim == 1
    T = mass.shape[0]
    F = len(group_rank)
    assert len(cum_num) == F and int(cum_num[-1]) == int(den)
    order = np.lexsort((np.arange(T), -mass.astype(np.float64)))  # last key primary
    bounds = [0] + [(T * int(c)) // int(den) for c in cum_num]
    rank = np.empty(T, dtype=np.int32)
    bucket_idx = np.empty(T, dtype=np.int32)
    for f in range(F):
        members = np.sort(order[bounds[f]:bounds[f + 1]])
        rank[members] = int(group_rank[f])
        bucket_idx[bounds[f]:bounds[f + 1]] = members
    return rank, np.asarray(bounds, dtype=np.int32), bucket_idx


def importance_update(I: np.ndarray, A_new: np.ndarray, alpha: float) -> np.ndarray:
    """Eq. 1: exponential moving average of head-averaged attention weights.

    I [T] running importance, A_new [T_q, H, T] attention weights of the T_q
    newest query positions.  I <- alpha^{T_q} I + (1 - alpha^{T_q}) * mean over
    the T_q new queries of (mean over heads of A).
    """
    A_new = np.asarray(A_new, np.float64)
    Tq = A_new.shape[0]
    a = float(alpha) ** Tq
    return a * np.asarray(I, np.float64) + (1.0 - a) * A_new.mean(axis=1).sum(axis=0) / Tq


# --------------------------------------------------------------------------
# int8 coefficients (workload definition; the paper only names 4-bit KVQuant)
# --------------------------------------------------------------------------

def quantize_i8(C: np.ndarray, block: int = 64) -> Tuple[np.ndarray, np.ndarray]:
    """Per-token, per-`block`-column symmetric int8 codes with an fp16 scale.

    The recipe is fixed in binary32/binary16 so that integer results are
    unique:  amax = max|c| over the block;  scale = fp16(fp32(amax) / 127f);
    scale == 0 -> all codes 0;  code = clamp(rint(fp32(c) / fp32(scale)),
    -127, 127) with IEEE division and round-half-to-even.

    C [T, r] float16 (or float32), r % block == 0.
    Returns (codes [T, r] int8, scales [T, r/block] float16).
    """
    C = np.asarray(C)
    T, r = C.shape
    assert r % block == 0
    c32 = C.astype(np.float32).reshape(T, r // block, block)
    amax = np.abs(c32).max(axis=2)                                   # exact
    scale16 = (amax / np.float32(127.0)).astype(np.float16)          # fp32 divide, RNE to fp16
    s32 = scale16.astype(np.float32)
    safe = np.where(s32 == 0, np.float32(1.0), s32)
    quo = c32 / safe[:, :, None]                                     # fp32 divide
    code = np.clip(np.rint(quo), -127.0, 127.0)
    code = np.where((s32 == 0)[:, :, None], 0.0, code)
    return code.astype(np.int8).reshape(T, r), scale16


def dequantize_i8(codes: np.ndarray, scales: np.ndarray, block: int = 64) -> np.ndarray:
    """codes [T, r] int8, scales [T, r/block] fp16 -> float64 values code*scale."""
    T, r = codes.shape
    s = np.repeat(scales.astype(np.float64), block, axis=1)
    return codes.astype(np.float64) * s


# --------------------------------------------------------------------------
# 4-bit coefficients (Sec. 4.5 and Table 4 combine the method with 4-bit
# quantisation "following KVQuant"; that scheme's non-uniform, calibrated code
# book needs data that is not available, so the reading taken here is the plain
# uniform one, with the block structure of the int8 format)
# --------------------------------------------------------------------------

def quantize_i4(C: np.ndarray, block: int = 64) -> Tuple[np.ndarray, np.ndarray]:
    """Per-token, per-`block`-column symmetric 4-bit codes with an fp16 scale.

    amax = max|c| over the block;  scale = fp16(fp32(amax) / 7f);  scale == 0 ->
    all codes 0;  code = clamp(rint(fp32(c) / fp32(scale)), -7, 7), IEEE
    division, round-half-to-even.  Two codes per byte: byte i of a row holds
    column 2i in its low nibble and column 2i+1 in its high nibble, each nibble
    the code plus 8 (1 .. 15).

    C [T, r] float16 (or float32), r % block == 0.
    Returns (packed [T, r/2] uint8, scales [T, r/block] float16).
    """
    C = np.asarray(C)
    T, r = C.shape
    assert r % block == 0 and block % 2 == 0
    c32 = C.astype(np.float32).reshape(T, r // block, block)
    amax = np.abs(c32).max(axis=2)
    scale16 = (amax / np.float32(7.0)).astype(np.float16)
    s32 = scale16.astype(np.float32)
    safe = np.where(s32 == 0, np.float32(1.0), s32)
    code = np.clip(np.rint(c32 / safe[:, :, None]), -7.0, 7.0)
    code = np.where((s32 == 0)[:, :, None], 0.0, code).astype(np.int32).reshape(T, r)
    u = (code + 8).astype(np.uint8)
    packed = (u[:, 0::2] | (u[:, 1::2] << 4)).astype(np.uint8)
    return packed, scale16


def unpack_i4(packed: np.ndarray) -> np.ndarray:
    """packed [T, r/2] uint8 -> integer codes [T, r] in -7 .. 7 (int32)."""
    packed = np.asarray(packed, np.uint8)
    T, half = packed.shape
    codes = np.empty((T, 2 * half), np.int32)
    codes[:, 0::2] = (packed & 0x0F).astype(np.int32) - 8
    codes[:, 1::2] = (packed >> 4).astype(np.int32) - 8
    return codes


def dequantize_i4(packed: np.ndarray, scales: np.ndarray, block: int = 64) -> np.ndarray:
    """packed [T, r/2] uint8, scales [T, r/block] fp16 -> float64 values code*scale."""
    codes = unpack_i4(packed)
    s = np.repeat(scales.astype(np.float64), block, axis=1)
    return codes.astype(np.float64) * s


# --------------------------------------------------------------------------
# closed-form accounting used in the paper's text and tables
# --------------------------------------------------------------------------

def compression_ratio(T: int, HD: int, R: int) -> float:
    """Sec. 3.1: c = T*HD / (T*R + R*HD) for one matrix of one layer."""
    return (T * HD) / (T * R + R * HD)


def decompression_flops(T: int, HD: int, fractions: Sequence[float],
                        ranks: Sequence[int]) -> float:
    """Sec. 3.2: 2*T*HD*sum_f r_f R^(f) flops to rebuild one cache matrix."""
    return 2.0 * T * HD * sum(f * R for f, R in zip(fractions, ranks))


def cache_bytes(L: int, HD: int, T_v: int, T_t: int, R_k: Optional[int],
                R_v: Optional[int], bytes_per_elt: float = 2) -> float:
    """Whole-model KV cache of one sample: visual tokens compressed to rank
    R_k / R_v (None = uncompressed), textual tokens kept uncompressed
    (experiment setup).  Per layer and per matrix: T_v*R + R*HD (Sec. 3.1)."""
    def one(R):
        vis = T_v * HD if R is None else T_v * R + R * HD
        return vis + T_t * HD
    return float(L * bytes_per_elt * (one(R_k) + one(R_v)))
