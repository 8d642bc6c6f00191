"""Pins for the decode-attention oracle: each test checks it against something
the paper or the mathematics fixes, not against itself."""
import math
from fractions import Fraction

import numpy as np
import pytest
import scipy.special

import oracle
from paper_2603_23914_amd import workloads as wl


def textbook_attention(q, K, V, scale):
    """Uncompressed multi-head attention of one query with library softmax."""
    H, d = q.shape
    out = np.empty((H, d))
    for h in range(H):
        s = K[:, h * d:(h + 1) * d] @ q[h] * scale
        out[h] = scipy.special.softmax(s) @ V[:, h * d:(h + 1) * d]
    return out


def small_case(seed, H=3, d=8, T=11, r=5):
    rng = np.random.default_rng(seed)
    HD = H * d
    Ck = rng.standard_normal((T, r))
    Cv = rng.standard_normal((T, r))
    Bk = rng.standard_normal((r, HD))
    Bv = rng.standard_normal((r, HD))
    q = rng.standard_normal((H, d))
    return q, Ck, Cv, Bk, Bv


def test_full_rank_equals_uncompressed_attention():
    """r = HD with the exact right-singular basis: compression is lossless, so
    the oracle must reproduce plain attention on K, V (Sec. 3.1, Alg. 1)."""
    rng = np.random.default_rng(1)
    H, d, T = 2, 8, 40
    K = rng.standard_normal((T, H * d))
    V = rng.standard_normal((T, H * d))
    q = rng.standard_normal((H, d))
    Bk = oracle.bases(K, H * d)
    Bv = oracle.bases(V, H * d)
    Ck = oracle.compact(K, Bk)
    Cv = oracle.compact(V, Bv)
    ref = textbook_attention(q, K, V, 1.0 / math.sqrt(d))
    got = oracle.decode_attn(q, Ck, Cv, Bk, Bv)
    assert np.abs(got - ref).max() < 1e-12
    got2 = oracle.decode_attn_absorbed(q, Ck, Cv, Bk, Bv)
    assert np.abs(got2 - ref).max() < 1e-12


def test_default_scale_is_inverse_sqrt_head_dim():
    """Alg. 1 divides by sqrt(D), D the per-head dimension (not H*D, not r)."""
    q, Ck, Cv, Bk, Bv = small_case(2, H=4, d=16, T=9, r=6)
    a = oracle.decode_attn(q, Ck, Cv, Bk, Bv)
    b = oracle.decode_attn(q, Ck, Cv, Bk, Bv, sm_scale=0.25)
    assert np.abs(a - b).max() < 1e-14
    c = oracle.decode_attn(q, Ck, Cv, Bk, Bv, sm_scale=1.0 / math.sqrt(64))
    assert np.abs(a - c).max() > 1e-3


@pytest.mark.parametrize("seed", range(4))
def test_absorbed_equals_reconstruct(seed):
    q, Ck, Cv, Bk, Bv = small_case(seed)
    T, r = Ck.shape
    rng = np.random.default_rng(100 + seed)
    rk = rng.integers(0, r + 1, size=T)
    rv = rng.integers(0, r + 1, size=T)
    a, la = oracle.decode_attn(q, Ck, Cv, Bk, Bv, rk, rv, return_lse=True)
    b, lb = oracle.decode_attn_absorbed(q, Ck, Cv, Bk, Bv, rk, rv, return_lse=True)
    assert np.abs(a - b).max() < 1e-12
    assert np.abs(la - lb).max() < 1e-12


def test_brute_force_scalar_loops():
    """Pure-Python triple loops written from Alg. 1, with per-token ranks."""
    q, Ck, Cv, Bk, Bv = small_case(7, H=2, d=4, T=6, r=3)
    H, d = q.shape
    T, r = Ck.shape
    rk = [3, 1, 2, 0, 3, 2]
    rv = [1, 3, 0, 2, 2, 3]
    scale = 1.0 / math.sqrt(d)
    out = [[0.0] * d for _ in range(H)]
    for h in range(H):
        scores = []
        for t in range(T):
            acc = 0.0
            for i in range(d):
                kti = sum(Ck[t, j] * Bk[j, h * d + i] for j in range(rk[t]))
                acc += q[h, i] * kti
            scores.append(acc * scale)
        mx = max(scores)
        ex = [math.exp(s - mx) for s in scores]
        z = sum(ex)
        for i in range(d):
            tot = 0.0
            for t in range(T):
                vti = sum(Cv[t, j] * Bv[j, h * d + i] for j in range(rv[t]))
                tot += ex[t] / z * vti
            out[h][i] = tot
    got = oracle.decode_attn(q, Ck, Cv, Bk, Bv, np.array(rk), np.array(rv))
    assert np.abs(got - np.array(out)).max() < 1e-13


def test_softmax_rows_sum_to_one_and_lse():
    q, Ck, Cv, Bk, Bv = small_case(3, T=50)
    A = oracle.attention_probs(q, Ck, Bk)
    assert A.shape == (q.shape[0], 50)
    assert np.abs(A.sum(axis=1) - 1.0).max() < 1e-14
    assert (A >= 0).all()
    # lse against the library logsumexp of the same scores
    _, lse = oracle.decode_attn(q, Ck, Cv, Bk, Bv, return_lse=True)
    H, d = q.shape
    K = Ck @ Bk
    for h in range(H):
        s = K[:, h * d:(h + 1) * d] @ q[h] / math.sqrt(d)
        assert abs(lse[h] - scipy.special.logsumexp(s)) < 1e-12


def _scalar_loop_weights(q, Ck, Bk, rk, scale, Hkv):
    """Attention weights written out from Alg. 1's score step with scalar loops:
    rebuild key element (t, column) from the leading rk[t] coefficients, dot it
    with the query of head h over the columns of key/value head h // (H/Hkv),
    scale, library softmax over the tokens."""
    H, d = q.shape
    T = Ck.shape[0]
    A = np.empty((H, T))
    for h in range(H):
        g = h // (H // Hkv)
        s = []
        for t in range(T):
            acc = 0.0
            for i in range(d):
                acc += q[h, i] * sum(Ck[t, j] * Bk[j, g * d + i] for j in range(rk[t]))
            s.append(acc * scale)
        A[h] = scipy.special.softmax(np.array(s))
    return A


def test_attention_probs_against_scalar_loops_and_library_softmax():
    """Values of the attention weights (the reference of every importance check):
    per-token key ranks, a scale that is not 1/sqrt(d), fewer key/value heads
    than query heads."""
    rng = np.random.default_rng(21)
    H, Hkv, d, T, r = 4, 2, 4, 7, 5
    q = rng.standard_normal((H, d))
    Ck = rng.standard_normal((T, r))
    Bk = rng.standard_normal((r, Hkv * d))
    rk = [5, 2, 0, 3, 1, 5, 4]
    scale = 0.37
    ref = _scalar_loop_weights(q, Ck, Bk, rk, scale, Hkv)
    got = oracle.attention_probs(q, Ck, Bk, rank_k=np.array(rk), sm_scale=scale, kv_heads=Hkv)
    assert np.abs(got - ref).max() < 1e-14
    # each of the plausible mistakes moves the reference by far more than that
    assert np.abs(_scalar_loop_weights(q, Ck, Bk, rk, 0.5, Hkv) - ref).max() > 1e-3       # scale
    assert np.abs(_scalar_loop_weights(q, Ck, Bk, [r] * T, scale, Hkv) - ref).max() > 1e-3  # truncation
    wrong_heads = _scalar_loop_weights(q[[0, 2, 1, 3]], Ck, Bk, rk, scale, Hkv)[[0, 2, 1, 3]]
    assert np.abs(wrong_heads - ref).max() > 1e-3                                          # head slice
    # default scale is 1/sqrt(d) (Alg. 1 divides by the square root of the head width)
    ref_d = _scalar_loop_weights(q, Ck, Bk, rk, 1.0 / math.sqrt(d), Hkv)
    got_d = oracle.attention_probs(q, Ck, Bk, rank_k=np.array(rk), kv_heads=Hkv)
    assert np.abs(got_d - ref_d).max() < 1e-14
    # multi-head default (kv_heads=None) with uniform rank
    Bk4 = rng.standard_normal((r, H * d))
    ref_m = _scalar_loop_weights(q, Ck, Bk4, [r] * T, 1.0 / math.sqrt(d), H)
    assert np.abs(oracle.attention_probs(q, Ck, Bk4) - ref_m).max() < 1e-14


@pytest.mark.parametrize("kv_heads", [None, 1])
def test_attention_probs_are_exp_of_score_minus_lse(kv_heads):
    """A[h,t] = exp(s[h,t] - lse[h]) with the log-sum-exp decode_attn returns, and
    decode_attn's output is A applied to the rebuilt values (ties the weights to
    the pinned attention output)."""
    rng = np.random.default_rng(22)
    H, d, T, r = 3, 8, 12, 6
    Hkv = H if kv_heads is None else kv_heads
    q = rng.standard_normal((H, d))
    Ck = rng.standard_normal((T, r))
    Cv = rng.standard_normal((T, r))
    Bk = rng.standard_normal((r, Hkv * d))
    Bv = rng.standard_normal((r, Hkv * d))
    rk = rng.integers(0, r + 1, size=T)
    rv = rng.integers(0, r + 1, size=T)
    scale = 0.21
    out, lse = oracle.decode_attn(q, Ck, Cv, Bk, Bv, rk, rv, sm_scale=scale, return_lse=True,
                                  kv_heads=kv_heads)
    A = oracle.attention_probs(q, Ck, Bk, rank_k=rk, sm_scale=scale, kv_heads=kv_heads)
    for h in range(H):
        g = h // (H // Hkv)
        s = np.array([(Ck[t, :rk[t]] @ Bk[:rk[t], g * d:(g + 1) * d]) @ q[h] * scale for t in range(T)])
        assert np.abs(A[h] - np.exp(s - lse[h])).max() < 1e-14
        Vh = np.array([Cv[t, :rv[t]] @ Bv[:rv[t], g * d:(g + 1) * d] for t in range(T)])
        assert np.abs(A[h] @ Vh - out[h]).max() < 1e-13


def test_single_token_returns_its_value_row():
    """T = 1: the softmax weight is 1, so out_h = Vtilde[0, head h] exactly."""
    q, Ck, Cv, Bk, Bv = small_case(4, T=1)
    H, d = q.shape
    got = oracle.decode_attn(q, Ck, Cv, Bk, Bv)
    V = Cv @ Bv
    assert np.abs(got - V[0].reshape(H, d)).max() < 1e-14


def test_two_tokens_closed_form():
    """T = 2: p_0 = sigmoid(s_0 - s_1); checks sign and the 1/sqrt(d) scale."""
    q, Ck, Cv, Bk, Bv = small_case(5, T=2, H=2, d=4, r=4)
    H, d = q.shape
    K = Ck @ Bk
    V = Cv @ Bv
    got = oracle.decode_attn(q, Ck, Cv, Bk, Bv)
    for h in range(H):
        s = [float(K[t, h * d:(h + 1) * d] @ q[h]) / 2.0 for t in range(2)]   # sqrt(4) = 2
        p0 = 1.0 / (1.0 + math.exp(-(s[0] - s[1])))
        ref = p0 * V[0, h * d:(h + 1) * d] + (1 - p0) * V[1, h * d:(h + 1) * d]
        assert np.abs(got[h] - ref).max() < 1e-13


def test_zero_query_gives_mean_value():
    """q = 0 makes every score equal: out = mean over tokens of Vtilde."""
    q, Ck, Cv, Bk, Bv = small_case(6, T=13)
    H, d = q.shape
    got = oracle.decode_attn(np.zeros_like(q), Ck, Cv, Bk, Bv)
    assert np.abs(got - (Cv @ Bv).mean(axis=0).reshape(H, d)).max() < 1e-14


def test_head_slices_follow_merged_layout():
    """Head h uses hidden columns [h*d,(h+1)*d) of the merged axis (Sec. 3.1):
    permuting whole head blocks of q, D_k, D_v permutes the output rows."""
    q, Ck, Cv, Bk, Bv = small_case(8, H=3, d=8)
    H, d = q.shape
    base = oracle.decode_attn(q, Ck, Cv, Bk, Bv)
    perm = [2, 0, 1]
    cols = np.concatenate([np.arange(p * d, (p + 1) * d) for p in perm])
    got = oracle.decode_attn(q[perm], Ck, Cv, Bk[:, cols], Bv[:, cols])
    assert np.abs(got - base[perm]).max() < 1e-13
    # and a transposed basis (wrong operand order) cannot even be expressed:
    with pytest.raises(AssertionError):
        oracle.decode_attn(q, Ck, Cv, Bk.T, Bv)


def test_token_permutation_invariance():
    q, Ck, Cv, Bk, Bv = small_case(9, T=17)
    T, r = Ck.shape
    rng = np.random.default_rng(9)
    rk = rng.integers(1, r + 1, size=T)
    rv = rng.integers(1, r + 1, size=T)
    p = rng.permutation(T)
    a = oracle.decode_attn(q, Ck, Cv, Bk, Bv, rk, rv)
    b = oracle.decode_attn(q, Ck[p], Cv[p], Bk, Bv, rk[p], rv[p])
    assert np.abs(a - b).max() < 1e-13


def test_ragged_equals_zeroed_trailing_columns():
    """Decoding token t at rank r_t == zeroing its coefficient columns >= r_t
    and decoding at full rank (Alg. 1 retrieve step uses leading columns)."""
    q, Ck, Cv, Bk, Bv = small_case(10, T=23, r=8)
    T, r = Ck.shape
    rng = np.random.default_rng(10)
    rk = rng.choice([8, 4, 2, 1], size=T)
    rv = rng.choice([8, 4, 2, 1], size=T)
    Ckz = Ck.copy()
    Cvz = Cv.copy()
    for t in range(T):
        Ckz[t, rk[t]:] = 0
        Cvz[t, rv[t]:] = 0
    a = oracle.decode_attn(q, Ck, Cv, Bk, Bv, rk, rv)
    b = oracle.decode_attn(q, Ckz, Cvz, Bk, Bv)
    assert np.abs(a - b).max() < 1e-13
    full = oracle.decode_attn(q, Ck, Cv, Bk, Bv, np.full(T, r), np.full(T, r))
    assert np.abs(full - oracle.decode_attn(q, Ck, Cv, Bk, Bv)).max() == 0.0
    assert np.abs(a - full).max() > 1e-3          # the ranks do matter


def test_config1_compressed_close_to_uncompressed():
    """Planted rank-16 cache + 1 % noise: rank-16 compression must stay within
    the noise level of uncompressed attention (sanity, not equality)."""
    c = wl.config1(0)
    K, V, q = c["K"], c["V"], c["q"]
    Bk = oracle.bases(K, c["r"])
    Bv = oracle.bases(V, c["r"])
    got = oracle.decode_attn(q, oracle.compact(K, Bk), oracle.compact(V, Bv), Bk, Bv)
    ref = textbook_attention(q, K, V, 1.0 / math.sqrt(c["d"]))
    err = np.abs(got - ref).max()
    assert 1e-6 < err < 0.05 * np.abs(ref).max()
    assert abs(np.std(K) - 1.0) < 0.15            # unit-variance reading of the recipe


def test_batched_wrapper_and_shared_basis():
    rng = np.random.default_rng(11)
    B, H, d, T, r, cap = 3, 2, 4, 7, 3, 9
    q = rng.standard_normal((B, H, d))
    Ck = rng.standard_normal((B, cap, r))
    Cv = rng.standard_normal((B, cap, r))
    Bk = rng.standard_normal((B, r, H * d))
    Bv = rng.standard_normal((r, H * d))
    out = oracle.decode_attn_batched(q, Ck, Cv, Bk, Bv, T)
    for b in range(B):
        ref = oracle.decode_attn(q[b], Ck[b, :T], Cv[b, :T], Bk[b], Bv)
        assert np.abs(out[b] - ref).max() == 0.0
    out2 = oracle.decode_attn_batched(q, Ck, Cv, Bk, Bv, T, absorbed=True)
    assert np.abs(out - out2).max() < 1e-13


def test_promote_is_exact():
    x16 = np.array([1.0, -0.333251953125, 65504.0, 6e-8], dtype=np.float16)
    assert (oracle.promote(x16, "f16") == x16.astype(np.float64)).all()
    # bf16 bit patterns with known values: 0x3F80 = 1.0, 0xC040 = -3.0, 0x3EAB = 0.333984375
    bits = np.array([0x3F80, 0xC040, 0x3EAB], dtype=np.uint16)
    assert oracle.promote(bits, "bf16").tolist() == [1.0, -3.0, float(Fraction(171, 512))]
    # generator-side rounding is round-to-nearest-even onto those patterns
    assert wl.to_bf16_bits(np.array([1.0, -3.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8])).tolist() == \
        [0x3F80, 0xC040, 0x3F80, 0x3F82]


def test_importance_update_eq1():
    """Eq. 1 with T_q = 1 is a plain EMA of the head-averaged weights; with
    alpha = 0 only the newest weights survive."""
    rng = np.random.default_rng(12)
    T, H = 9, 3
    I = rng.random(T)
    A = rng.random((1, H, T))
    got = oracle.importance_update(I, A, 0.25)
    assert np.abs(got - (0.25 * I + 0.75 * A[0].mean(axis=0))).max() < 1e-15
    assert np.abs(oracle.importance_update(I, A, 0.0) - A[0].mean(axis=0)).max() < 1e-15
    A2 = rng.random((2, H, T))
    got2 = oracle.importance_update(I, A2, 0.5)
    ref2 = 0.25 * I + 0.75 * (A2[0].mean(axis=0) + A2[1].mean(axis=0)) / 2
    assert np.abs(got2 - ref2).max() < 1e-15
