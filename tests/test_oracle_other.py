"""Pins for the oracle's compaction, rank selection, int8 quantisation and the
paper's closed-form accounting."""
from fractions import Fraction

import numpy as np
import pytest

import oracle


# ------------------------------------------------------------------ compaction

def test_compaction_is_truncated_svd():
    """Sec. 3.1: Kbar = U_r Sigma_r (columns scaled by singular values), D_k =
    V_r^T; the residual of the rank-r reconstruction is the Eckart-Young one."""
    rng = np.random.default_rng(0)
    T, HD, r = 30, 24, 7
    K = rng.standard_normal((T, HD)) @ np.diag(np.linspace(2, 0.1, HD)) @ rng.standard_normal((HD, HD))
    D = oracle.bases(K, r)
    C = oracle.compact(K, D)
    U, S, Vt = np.linalg.svd(K, full_matrices=False)
    assert np.abs(D @ D.T - np.eye(r)).max() < 1e-12
    # singular values strictly ordered: columns of C match U_r Sigma_r up to sign
    ref = U[:, :r] * S[:r]
    for j in range(r):
        assert min(np.abs(C[:, j] - ref[:, j]).max(), np.abs(C[:, j] + ref[:, j]).max()) < 1e-10
    # column norms are the singular values, in decreasing order
    norms = np.linalg.norm(C, axis=0)
    assert np.abs(norms - S[:r]).max() < 1e-10
    assert (np.diff(norms) < 0).all()
    # residual energy = sum of the discarded sigma^2
    res = np.linalg.norm(K - C @ D) ** 2
    assert abs(res - np.sum(S[r:] ** 2)) < 1e-9 * np.sum(S ** 2)
    assert C.shape == (T, r) and D.shape == (r, HD)


def test_compact_single_row_matches_projection():
    rng = np.random.default_rng(1)
    D = np.linalg.qr(rng.standard_normal((12, 4)))[0].T
    x = rng.standard_normal((1, 12))
    c = oracle.compact(x, D)
    assert c.shape == (1, 4)
    for j in range(4):
        assert abs(c[0, j] - sum(x[0, i] * D[j, i] for i in range(12))) < 1e-14


# -------------------------------------------------------------- rank selection

def brute_select(mass, group_rank, cum_num, den):
    T = len(mass)
    order = sorted(range(T), key=lambda t: (-float(mass[t]), t))
    bounds = [0] + [(T * c) // den for c in cum_num]
    rank = [None] * T
    idx = []
    for f in range(len(group_rank)):
        members = sorted(order[bounds[f]:bounds[f + 1]])
        for t in members:
            rank[t] = group_rank[f]
        idx += members
    return rank, bounds, idx


@pytest.mark.parametrize("T", [1, 2, 7, 64, 257])
@pytest.mark.parametrize("ties", [False, True])
def test_select_ranks_against_python_sorted(T, ties):
    rng = np.random.default_rng(T + 1000 * ties)
    mass = rng.random(T).astype(np.float32)
    if ties:
        mass = (np.floor(mass * 4) / 4).astype(np.float32)
    gr, cn, den = [512, 256, 128, 64], [1, 2, 3, 4], 4
    rank, off, idx = oracle.select_ranks(mass, gr, cn, den)
    brank, boff, bidx = brute_select(mass, gr, cn, den)
    assert rank.tolist() == brank
    assert off.tolist() == boff
    assert idx.tolist() == bidx
    assert rank.dtype == np.int32 and off.dtype == np.int32 and idx.dtype == np.int32


def test_select_ranks_invariants():
    rng = np.random.default_rng(5)
    T = 1000
    mass = rng.random(T).astype(np.float32)
    gr, cn, den = [64, 16], [1, 10], 10            # the paper's example: 10 % at R=64, 90 % at R=16
    rank, off, idx = oracle.select_ranks(mass, gr, cn, den)
    assert off.tolist() == [0, 100, 1000]
    assert sorted(idx.tolist()) == list(range(T))
    assert (np.diff(rank[idx]) <= 0).all()
    for f in range(2):
        seg = idx[off[f]:off[f + 1]]
        assert (np.diff(seg) > 0).all()
        assert (rank[seg] == gr[f]).all()
    # the high-rank group holds exactly the 100 largest masses
    assert set(idx[:100].tolist()) == set(np.argsort(-mass, kind="stable")[:100].tolist())


def test_select_ranks_degenerate():
    mass = np.full(10, 0.1, dtype=np.float32)      # all equal: groups are index ranges
    rank, off, idx = oracle.select_ranks(mass, [8, 4], [1, 2], 2)
    assert idx.tolist() == list(range(10)) and off.tolist() == [0, 5, 10]
    assert rank.tolist() == [8] * 5 + [4] * 5
    rank, off, idx = oracle.select_ranks(mass, [8], [1], 1)   # F = 1: everything at full rank
    assert rank.tolist() == [8] * 10 and off.tolist() == [0, 10]
    rank, off, idx = oracle.select_ranks(np.array([3, 1, 2], np.float32), [8, 4, 2, 1], [1, 2, 3, 4], 4)
    assert off.tolist() == [0, 0, 1, 2, 3]         # floor(3*f/4): first group empty
    assert rank.tolist() == [4, 1, 2]


# ---------------------------------------------------------------- quantisation

def exact_codes(block16):
    """The recipe evaluated with exact rationals, rounding each step to the
    stated binary format by brute force."""
    vals = [Fraction(float(x)) for x in block16]
    amax = max(abs(v) for v in vals)
    q32 = np.float32(float(amax)) / np.float32(127.0)          # reference fp32 divide ...
    # ... cross-checked: q32 must be the binary32 nearest to the exact quotient
    exact = amax / 127
    lo, hi = np.nextafter(q32, np.float32(-np.inf)), np.nextafter(q32, np.float32(np.inf))
    assert abs(Fraction(float(q32)) - exact) <= min(abs(Fraction(float(lo)) - exact),
                                                     abs(Fraction(float(hi)) - exact))
    scale = Fraction(float(np.float16(q32)))
    if scale == 0:
        return [0] * len(vals), 0.0
    codes = []
    for v in vals:
        quo = v / scale
        quo32 = Fraction(float(np.float32(float(v)) / np.float32(float(scale))))
        # exact quotient is far from a rounding tie compared with fp32 spacing,
        # so rounding the exact value must agree with rounding the fp32 one
        fl = quo.numerator // quo.denominator
        frac = quo - fl
        near = fl + (1 if frac > Fraction(1, 2) or (frac == Fraction(1, 2) and fl % 2 == 1) else 0)
        near32 = int(np.rint(float(quo32)))
        assert near == near32
        codes.append(max(-127, min(127, near)))
    return codes, float(scale)


def test_quantize_i8_exact_small():
    rng = np.random.default_rng(0)
    C = (rng.standard_normal((5, 128)) * np.array([10.0, 1.0, 0.1, 1e-3, 50.0])[:, None]).astype(np.float16)
    C[1, :64] = 0                                  # an all-zero block
    C[2, 3] = np.float16(0.5)
    codes, scales = oracle.quantize_i8(C)
    assert codes.dtype == np.int8 and scales.dtype == np.float16
    assert codes.shape == (5, 128) and scales.shape == (5, 2)
    for t in range(5):
        for blk in range(2):
            ref, sc = exact_codes(C[t, blk * 64:(blk + 1) * 64])
            assert codes[t, blk * 64:(blk + 1) * 64].tolist() == ref
            assert float(scales[t, blk]) == sc
    assert (codes[1, :64] == 0).all() and scales[1, 0] == 0


def test_quantize_i8_properties():
    rng = np.random.default_rng(1)
    C = (rng.standard_normal((64, 512)) * rng.uniform(0.01, 40, size=(64, 1))).astype(np.float16)
    codes, scales = oracle.quantize_i8(C)
    assert np.abs(codes.astype(np.int32)).max() <= 127
    deq = oracle.dequantize_i8(codes, scales)
    s = np.repeat(scales.astype(np.float64), 64, axis=1)
    unclamped = np.abs(C.astype(np.float64) / s) <= 127.0
    assert (np.abs(C.astype(np.float64) - deq)[unclamped] <= 0.5 * s[unclamped] * (1 + 1e-6)).all()
    # the block's largest element lands on +-127 or +-126 (fp16 rounding of the scale)
    blk = np.abs(C.astype(np.float64)).reshape(64, 8, 64)
    am = np.take_along_axis(np.abs(codes.astype(np.int32)).reshape(64, 8, 64),
                            blk.argmax(axis=2)[..., None], axis=2)
    assert am.min() >= 126 and am.max() <= 127
    # dequantise is exactly code*scale
    assert deq[3, 70] == float(codes[3, 70]) * float(scales[3, 1])


def exact_codes4(block):
    """4-bit recipe in exact rational arithmetic, except where it fixes binary32 / binary16."""
    vals = [Fraction(float(x)) for x in block]
    amax = max(abs(v) for v in vals)
    scale = np.float16(np.float32(float(amax)) / np.float32(7.0))
    if float(scale) == 0.0:
        return [0] * len(block), 0.0
    codes = []
    for x in block:
        quo = Fraction(float(np.float32(np.float32(x) / np.float32(scale))))     # the fp32 quotient, exactly
        fl = quo.numerator // quo.denominator
        frac = quo - fl
        near = fl if frac < Fraction(1, 2) else fl + 1
        if frac == Fraction(1, 2):
            near = fl if fl % 2 == 0 else fl + 1
        codes.append(max(-7, min(7, near)))
    return codes, float(scale)


def test_quantize_i4_exact_small_and_packing():
    rng = np.random.default_rng(2)
    C = (rng.standard_normal((4, 128)) * np.array([10.0, 1.0, 1e-3, 50.0])[:, None]).astype(np.float16)
    C[1, 64:] = 0                                  # an all-zero block
    C[0, :8] = np.array([3.5, -3.5, 7, -7, 0.5, -0.5, 1.5, 2.5], np.float16)   # ties at scale 1 (amax 7)
    C[0, 8:64] = np.clip(C[0, 8:64], -7, 7)
    packed, scales = oracle.quantize_i4(C)
    assert packed.dtype == np.uint8 and packed.shape == (4, 64) and scales.shape == (4, 2)
    codes = oracle.unpack_i4(packed)
    for t in range(4):
        for blk in range(2):
            ref, sc = exact_codes4(C[t, blk * 64:(blk + 1) * 64])
            assert codes[t, blk * 64:(blk + 1) * 64].tolist() == ref
            assert float(scales[t, blk]) == sc
    # half-to-even at scale exactly 1: 3.5 -> 4, -3.5 -> -4, 0.5 -> 0, 1.5 -> 2, 2.5 -> 2
    assert float(scales[0, 0]) == 1.0 and codes[0, :8].tolist() == [4, -4, 7, -7, 0, 0, 2, 2]
    # layout: byte i = (column 2i + 8) | (column 2i+1 + 8) << 4, written out by hand
    assert packed[0, 0] == (4 + 8) | ((-4 + 8) << 4) and packed[0, 1] == (7 + 8) | ((-7 + 8) << 4)
    assert (packed[1, 32:] == 0x88).all() and scales[1, 1] == 0 and (codes[1, 64:] == 0).all()
    assert np.abs(codes).max() <= 7 and packed.min() >= 0x11


def test_quantize_i4_properties():
    rng = np.random.default_rng(3)
    C = (rng.standard_normal((32, 256)) * rng.uniform(0.01, 40, size=(32, 1))).astype(np.float16)
    packed, scales = oracle.quantize_i4(C)
    deq = oracle.dequantize_i4(packed, scales)
    s = np.repeat(scales.astype(np.float64), 64, axis=1)
    inside = np.abs(C.astype(np.float64) / s) <= 7.0
    assert (np.abs(C.astype(np.float64) - deq)[inside] <= 0.5 * s[inside] * (1 + 1e-6)).all()
    codes = oracle.unpack_i4(packed)
    blk = np.abs(C.astype(np.float64)).reshape(32, 4, 64)
    am = np.take_along_axis(np.abs(codes).reshape(32, 4, 64), blk.argmax(axis=2)[..., None], axis=2)
    assert (am == 7).all()                          # amax/7 rounded to fp16 keeps the largest element at +-7
    assert deq[3, 70] == float(codes[3, 70]) * float(scales[3, 1])
    # 4 bits carry less than 8: the error is about 127 / 7 times the int8 one
    c8, s8 = oracle.quantize_i8(C)
    e8 = np.abs(oracle.dequantize_i8(c8, s8) - C.astype(np.float64)).mean()
    e4 = np.abs(deq - C.astype(np.float64)).mean()
    assert 10 < e4 / e8 < 30


# ------------------------------------------------------ the paper's own numbers

def test_paper_closed_forms(paper_values):
    pv = paper_values

    def check(key, got):
        val, tol = pv[key]
        assert abs(got - val) <= tol, (key, got, val)

    check("compression_ratio_T1000_H40_D128_R64", oracle.compression_ratio(1000, 40 * 128, 64))
    full = oracle.decompression_flops(1000, 5120, [1.0], [64])
    part = oracle.decompression_flops(1000, 5120, [0.1, 0.9], [64, 16])
    check("flop_reduction_F2_r0.1_R64_R16", 1 - part / full)
    vonly = full + oracle.decompression_flops(1000, 5120, [0.25, 0.75], [64, 16])
    check("flop_reduction_vonly_r0.25_R64_R16", 1 - vonly / (2 * full))
    check("kv_bytes_13B_16img_b64_GB", 64 * oracle.cache_bytes(40, 5120, 16 * 256, 0, None, None) / 1e9)

    # LLaVA-1.5-7B: 32 layers, HD 4096, 576 visual tokens; 50 text tokens reproduce the tables
    L, HD, Tv, Tt = 32, 4096, 576, 50
    f7 = oracle.cache_bytes(L, HD, Tv, Tt, None, None)
    check("llava7b_full_MB", f7 / 1e6)
    check("llava7b_R64_MB", oracle.cache_bytes(L, HD, Tv, Tt, 64, 64) / 1e6)
    check("llava7b_R64_4bit_MB", oracle.cache_bytes(L, HD, Tv, Tt, 64, 64, bytes_per_elt=0.5) / 1e6)
    for R in (128, 64, 32, 16):
        check(f"llava7b_R{R}_reduction", f7 / oracle.cache_bytes(L, HD, Tv, Tt, R, R))
    check("llava7b_Rk64_Rv128_reduction", f7 / oracle.cache_bytes(L, HD, Tv, Tt, 64, 128))
    check("llava7b_Rk128_Rv256_reduction", f7 / oracle.cache_bytes(L, HD, Tv, Tt, 128, 256))
    check("llava7b_batch32_full_GB", 32 * f7 / 1e9)
    check("llava7b_batch32_R64_GB", 32 * oracle.cache_bytes(L, HD, Tv, Tt, 64, 64) / 1e9)
    check("llava7b_batch32_R32_GB", 32 * oracle.cache_bytes(L, HD, Tv, Tt, 32, 32) / 1e9)
    # LLaVA-1.5-13B: 40 layers, HD 5120
    f13 = oracle.cache_bytes(40, 5120, Tv, Tt, None, None)
    check("llava13b_R64_reduction", f13 / oracle.cache_bytes(40, 5120, Tv, Tt, 64, 64))
    check("llava13b_R32_reduction", f13 / oracle.cache_bytes(40, 5120, Tv, Tt, 32, 32))
    # VideoLLaVA-7B: 8 frames x 257 tokens, 70 text tokens
    fv = oracle.cache_bytes(L, HD, 8 * 257, 70, None, None)
    check("videollava_full_MB", fv / 1e6)
    check("videollava_R128_MB", oracle.cache_bytes(L, HD, 8 * 257, 70, 128, 128) / 1e6)
    check("videollava_R128_reduction", fv / oracle.cache_bytes(L, HD, 8 * 257, 70, 128, 128))


def test_cache_bytes_reduces_to_ratio_formula():
    """One layer, one matrix, no text: cache_bytes ratio == Sec. 3.1's c."""
    T, HD, R = 1000, 5120, 64
    full = oracle.cache_bytes(1, HD, T, 0, None, None)
    comp = oracle.cache_bytes(1, HD, T, 0, R, R)
    assert abs(full / comp - oracle.compression_ratio(T, HD, R)) < 1e-12
