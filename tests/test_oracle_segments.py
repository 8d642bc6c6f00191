"""Pins for the multi-segment oracle (Alg. 1's cache: compressed segments next to an
uncompressed one under a single softmax): library softmax, brute force, invariances."""
import math

import numpy as np
import pytest
import scipy.special

import oracle


def rand_case(seed, H=3, d=8, T=13, r=6, Tu=7):
    rng = np.random.default_rng(seed)
    HD = H * d
    return dict(q=rng.standard_normal((H, d)),
                Ck=rng.standard_normal((T, r)), Cv=rng.standard_normal((T, r)),
                Bk=rng.standard_normal((r, HD)), Bv=rng.standard_normal((r, HD)),
                K=rng.standard_normal((Tu, HD)), V=rng.standard_normal((Tu, HD)))


def test_raw_attn_is_library_softmax_attention():
    c = rand_case(1, H=4, d=16, Tu=29)
    H, d = c["q"].shape
    out, lse = oracle.raw_attn(c["q"], c["K"], c["V"], return_lse=True)
    for h in range(H):
        s = c["K"][:, h * d:(h + 1) * d] @ c["q"][h] / math.sqrt(d)
        assert np.abs(out[h] - scipy.special.softmax(s) @ c["V"][:, h * d:(h + 1) * d]).max() < 1e-13
        assert abs(lse[h] - scipy.special.logsumexp(s)) < 1e-12


def test_raw_attn_empty_cache():
    c = rand_case(2)
    out, lse = oracle.raw_attn(c["q"], c["K"][:0], c["V"][:0], return_lse=True)
    assert (out == 0).all() and np.isneginf(lse).all()


def test_segments_brute_force_loops():
    """Scalar loops written from Alg. 1: decompress the compressed tokens at their ranks, append
    the uncompressed ones, one softmax over all of them."""
    c = rand_case(3, H=2, d=4, T=5, r=3, Tu=4)
    H, d = c["q"].shape
    rk, rv = [3, 1, 0, 2, 3], [2, 3, 1, 0, 3]
    scale = 1.0 / math.sqrt(d)
    ref = np.zeros((H, d))
    for h in range(H):
        keys, vals = [], []
        for t in range(5):
            keys.append([sum(c["Ck"][t, j] * c["Bk"][j, h * d + i] for j in range(rk[t])) for i in range(d)])
            vals.append([sum(c["Cv"][t, j] * c["Bv"][j, h * d + i] for j in range(rv[t])) for i in range(d)])
        for t in range(4):
            keys.append([c["K"][t, h * d + i] for i in range(d)])
            vals.append([c["V"][t, h * d + i] for i in range(d)])
        sc = [scale * sum(c["q"][h, i] * k[i] for i in range(d)) for k in keys]
        mx = max(sc)
        ex = [math.exp(x - mx) for x in sc]
        for i in range(d):
            ref[h, i] = sum(e * v[i] for e, v in zip(ex, vals)) / sum(ex)
    got = oracle.decode_attn_segments(c["q"], [
        dict(Ck=c["Ck"], Cv=c["Cv"], Bk=c["Bk"], Bv=c["Bv"], rank_k=np.array(rk), rank_v=np.array(rv)),
        dict(K=c["K"], V=c["V"])])
    assert np.abs(got - ref).max() < 1e-13


def test_one_compressed_segment_is_decode_attn():
    c = rand_case(4)
    a = oracle.decode_attn_segments(c["q"], [dict(Ck=c["Ck"], Cv=c["Cv"], Bk=c["Bk"], Bv=c["Bv"])])
    assert np.abs(a - oracle.decode_attn(c["q"], c["Ck"], c["Cv"], c["Bk"], c["Bv"])).max() < 1e-14


def test_splitting_a_segment_changes_nothing():
    """Token sets are just concatenated: cutting a compressed segment in two, or moving its
    reconstructed rows into the uncompressed segment, gives the same attention."""
    c = rand_case(5, T=17)
    whole = oracle.decode_attn(c["q"], c["Ck"], c["Cv"], c["Bk"], c["Bv"])
    cut = oracle.decode_attn_segments(c["q"], [
        dict(Ck=c["Ck"][:6], Cv=c["Cv"][:6], Bk=c["Bk"], Bv=c["Bv"]),
        dict(Ck=c["Ck"][6:], Cv=c["Cv"][6:], Bk=c["Bk"], Bv=c["Bv"])])
    assert np.abs(cut - whole).max() < 1e-13
    moved = oracle.decode_attn_segments(c["q"], [
        dict(Ck=c["Ck"][:6], Cv=c["Cv"][:6], Bk=c["Bk"], Bv=c["Bv"]),
        dict(K=c["Ck"][6:] @ c["Bk"], V=c["Cv"][6:] @ c["Bv"])])
    assert np.abs(moved - whole).max() < 1e-13


def test_segment_order_does_not_matter():
    c = rand_case(6)
    seg_c = dict(Ck=c["Ck"], Cv=c["Cv"], Bk=c["Bk"], Bv=c["Bv"])
    seg_u = dict(K=c["K"], V=c["V"])
    a = oracle.decode_attn_segments(c["q"], [seg_c, seg_u])
    b = oracle.decode_attn_segments(c["q"], [seg_u, seg_c])
    assert np.abs(a - b).max() < 1e-13


@pytest.mark.parametrize("seed", [7, 8])
def test_merge_of_parts_equals_attention_over_the_union(seed):
    """merge_segments is the log-sum-exp identity: checked against the concatenation."""
    c = rand_case(seed, H=4, d=8, T=19, Tu=9)
    o1, l1 = oracle.decode_attn(c["q"], c["Ck"], c["Cv"], c["Bk"], c["Bv"], return_lse=True)
    o2, l2 = oracle.raw_attn(c["q"], c["K"], c["V"], return_lse=True)
    ref, ref_lse = oracle.decode_attn_segments(c["q"], [dict(Ck=c["Ck"], Cv=c["Cv"], Bk=c["Bk"], Bv=c["Bv"]),
                                                        dict(K=c["K"], V=c["V"])], return_lse=True)
    out, lse = oracle.merge_segments([o1, o2], [l1, l2])
    assert np.abs(out - ref).max() < 1e-13 and np.abs(lse - ref_lse).max() < 1e-12
    # an empty part drops out
    o0, l0 = oracle.raw_attn(c["q"], c["K"][:0], c["V"][:0], return_lse=True)
    out3, lse3 = oracle.merge_segments([o1, o0, o2], [l1, l0, l2])
    assert np.abs(out3 - ref).max() < 1e-13 and np.abs(lse3 - ref_lse).max() < 1e-12


def test_dominant_uncompressed_token_takes_over():
    """A key aligned with the query and scaled up wins the softmax: the output tends to that
    token's value row whatever the compressed segment holds."""
    c = rand_case(9, H=2, d=8)
    H, d = c["q"].shape
    K = c["K"].copy()
    K[3] = 60.0 * c["q"].reshape(-1)
    out = oracle.decode_attn_segments(c["q"], [dict(Ck=c["Ck"], Cv=c["Cv"], Bk=c["Bk"], Bv=c["Bv"]),
                                               dict(K=K, V=c["V"])])
    assert np.abs(out - c["V"][3].reshape(H, d)).max() < 1e-9


# ---------------------------------------------------------------- grouped-query attention

def gqa_case(seed, H=6, Hkv=2, d=8, T=15, r=5, Tu=6):
    rng = np.random.default_rng(seed)
    HDkv = Hkv * d
    return dict(q=rng.standard_normal((H, d)),
                Ck=rng.standard_normal((T, r)), Cv=rng.standard_normal((T, r)),
                Bk=rng.standard_normal((r, HDkv)), Bv=rng.standard_normal((r, HDkv)),
                K=rng.standard_normal((Tu, HDkv)), V=rng.standard_normal((Tu, HDkv)))


def repeat_kv(M, H, Hkv, d):
    """[.., Hkv*d] -> [.., H*d]: every key/value head's slice copied to the query heads that
    share it (what a model without grouped queries would store)."""
    g = H // Hkv
    parts = [M[..., (h // g) * d:(h // g + 1) * d] for h in range(H)]
    return np.concatenate(parts, axis=-1)


@pytest.mark.parametrize("H,Hkv", [(6, 2), (8, 1), (4, 4), (12, 3)])
def test_grouped_queries_equal_multi_head_on_repeated_kv_heads(H, Hkv):
    """Grouped-query attention is multi-head attention whose key/value heads are shared: with
    the shared slices written out once per query head the plain functions must agree."""
    d = 8
    c = gqa_case(11, H=H, Hkv=Hkv, d=d)
    rk = np.array([5, 3, 1, 0, 2, 5, 4, 4, 3, 2, 1, 5, 5, 0, 2])
    Bk_r, Bv_r = repeat_kv(c["Bk"], H, Hkv, d), repeat_kv(c["Bv"], H, Hkv, d)
    for fn in (oracle.decode_attn, oracle.decode_attn_absorbed):
        a, la = fn(c["q"], c["Ck"], c["Cv"], c["Bk"], c["Bv"], rk, rk, return_lse=True, kv_heads=Hkv)
        b, lb = oracle.decode_attn(c["q"], c["Ck"], c["Cv"], Bk_r, Bv_r, rk, rk, return_lse=True)
        assert np.abs(a - b).max() < 1e-13 and np.abs(la - lb).max() < 1e-12
    pa = oracle.attention_probs(c["q"], c["Ck"], c["Bk"], rk, kv_heads=Hkv)
    pb = oracle.attention_probs(c["q"], c["Ck"], Bk_r, rk)
    assert np.abs(pa - pb).max() < 1e-14
    ra = oracle.raw_attn(c["q"], c["K"], c["V"], kv_heads=Hkv)
    rb = oracle.raw_attn(c["q"], repeat_kv(c["K"], H, Hkv, d), repeat_kv(c["V"], H, Hkv, d))
    assert np.abs(ra - rb).max() < 1e-13
    sa = oracle.decode_attn_segments(c["q"], [dict(Ck=c["Ck"], Cv=c["Cv"], Bk=c["Bk"], Bv=c["Bv"]),
                                              dict(K=c["K"], V=c["V"])], kv_heads=Hkv)
    sb = oracle.decode_attn_segments(c["q"], [dict(Ck=c["Ck"], Cv=c["Cv"], Bk=Bk_r, Bv=Bv_r),
                                              dict(K=repeat_kv(c["K"], H, Hkv, d), V=repeat_kv(c["V"], H, Hkv, d))])
    assert np.abs(sa - sb).max() < 1e-13


def test_grouped_queries_head_mapping_is_by_consecutive_groups():
    """Query heads 0..g-1 read key/value head 0, the next g read head 1, ...: make one
    key/value head's keys huge for one token and see which query heads follow it."""
    H, Hkv, d = 6, 3, 4
    c = gqa_case(12, H=H, Hkv=Hkv, d=d, T=1, r=2, Tu=5)
    q = np.ones((H, d))
    K = np.zeros((5, Hkv * d))
    K[2, 1 * d:2 * d] = 50.0                      # token 2 dominates for key/value head 1 only
    out = oracle.raw_attn(q, K, c["V"], kv_heads=Hkv)
    for h in range(H):
        kv = h // 2
        if kv == 1:
            assert np.abs(out[h] - c["V"][2, d:2 * d]).max() < 1e-9
        else:
            assert np.abs(out[h] - c["V"][:, kv * d:(kv + 1) * d].mean(axis=0)).max() < 1e-12


# ---- one-sided compression (appendix "Analysis of Textual Token Compression": keys at R_k = 64, values kept) ----
def test_key_only_segment_brute_force_loops():
    """Scalar loops: keys rebuilt from their coefficients, values taken as stored, grouped heads."""
    rng = np.random.default_rng(21)
    H, Hkv, d, T, r = 4, 2, 3, 6, 4
    q = rng.standard_normal((H, d))
    Ck = rng.standard_normal((T, r))
    Bk = rng.standard_normal((r, Hkv * d))
    V = rng.standard_normal((T, Hkv * d))
    scale = 1.0 / math.sqrt(d)
    ref = np.zeros((H, d))
    ref_lse = np.zeros(H)
    for h in range(H):
        kvh = h // (H // Hkv)
        sc = []
        for t in range(T):
            key = [sum(Ck[t, j] * Bk[j, kvh * d + i] for j in range(r)) for i in range(d)]
            sc.append(scale * sum(q[h, i] * key[i] for i in range(d)))
        mx = max(sc)
        ex = [math.exp(x - mx) for x in sc]
        for i in range(d):
            ref[h, i] = sum(e * V[t, kvh * d + i] for t, e in enumerate(ex)) / sum(ex)
        ref_lse[h] = mx + math.log(sum(ex))
    got, lse = oracle.decode_attn_segments(q, [dict(Ck=Ck, Bk=Bk, V=V)], return_lse=True, kv_heads=Hkv)
    assert np.abs(got - ref).max() < 1e-13 and np.abs(lse - ref_lse).max() < 1e-13


def test_value_only_segment_brute_force_loops():
    rng = np.random.default_rng(22)
    H, d, T, r = 2, 4, 5, 3
    q = rng.standard_normal((H, d))
    K = rng.standard_normal((T, H * d))
    Cv = rng.standard_normal((T, r))
    Bv = rng.standard_normal((r, H * d))
    rv = [3, 0, 2, 1, 3]
    scale = 1.0 / math.sqrt(d)
    ref = np.zeros((H, d))
    for h in range(H):
        sc = [scale * sum(q[h, i] * K[t, h * d + i] for i in range(d)) for t in range(T)]
        mx = max(sc)
        ex = [math.exp(x - mx) for x in sc]
        for i in range(d):
            vals = [sum(Cv[t, j] * Bv[j, h * d + i] for j in range(rv[t])) for t in range(T)]
            ref[h, i] = sum(e * v for e, v in zip(ex, vals)) / sum(ex)
    got = oracle.decode_attn_segments(q, [dict(K=K, Cv=Cv, Bv=Bv, rank_v=np.array(rv))])
    assert np.abs(got - ref).max() < 1e-13


def test_one_sided_segments_reduce_to_the_known_cases():
    """Keys in a complete orthonormal basis lose nothing: key-only compression at r = H*d equals
    plain attention on the raw keys; and a two-sided segment equals the compressed decode."""
    c = rand_case(23, H=3, d=4, T=9, r=12, Tu=9)
    HD = 12
    Qm, _ = np.linalg.qr(np.random.default_rng(5).standard_normal((HD, HD)))
    Bk = Qm.T                                             # orthonormal rows, complete
    Ck = c["K"] @ Bk.T                                    # then Ck Bk = K exactly (up to rounding)
    got = oracle.decode_attn_segments(c["q"], [dict(Ck=Ck, Bk=Bk, V=c["V"])])
    assert np.abs(got - oracle.raw_attn(c["q"], c["K"], c["V"])).max() < 1e-12
    both = oracle.decode_attn_segments(c["q"], [dict(Ck=c["Ck"], Bk=c["Bk"], Cv=c["Cv"], Bv=c["Bv"])])
    assert np.abs(both - oracle.decode_attn(c["q"], c["Ck"], c["Cv"], c["Bk"], c["Bv"])).max() < 1e-12
    with pytest.raises(ValueError):
        oracle.decode_attn_segments(c["q"], [dict(Ck=c["Ck"], Bk=c["Bk"], V=c["V"][:5])])


def test_key_only_segment_next_to_a_raw_tail_is_the_merge_of_the_two():
    c = rand_case(24, H=2, d=8, T=11, r=5, Tu=6)
    Vc = np.random.default_rng(6).standard_normal((11, 16))
    whole, lse = oracle.decode_attn_segments(c["q"], [dict(Ck=c["Ck"], Bk=c["Bk"], V=Vc), dict(K=c["K"], V=c["V"])],
                                             return_lse=True)
    o1, l1 = oracle.decode_attn_segments(c["q"], [dict(Ck=c["Ck"], Bk=c["Bk"], V=Vc)], return_lse=True)
    o2, l2 = oracle.raw_attn(c["q"], c["K"], c["V"], return_lse=True)
    om, lm = oracle.merge_segments([o1, o2], [l1, l2])
    assert np.abs(om - whole).max() < 1e-13 and np.abs(lm - lse).max() < 1e-13
