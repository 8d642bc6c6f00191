"""Pins for the oracle side of the compression step (Sec. 3.1; Alg. 1 compress step; randomized
SVD as the appendix names it): the quality checker against closed forms and planted mistakes, the
randomized scheme against the exact truncated SVD it approximates."""
import numpy as np
import pytest

import oracle


def decaying(T, HD, seed, power=0.7, noise=0.01):
    rng = np.random.default_rng(seed)
    n = min(T, HD)
    U, _ = np.linalg.qr(rng.standard_normal((T, n)))
    V, _ = np.linalg.qr(rng.standard_normal((HD, n)))
    s = np.arange(1, n + 1) ** -power
    return (U * s) @ V.T + noise * rng.standard_normal((T, HD)) / np.sqrt(HD)


def test_checker_on_the_exact_basis_and_closed_form():
    """Diagonal cache: singular values are the diagonal, the leading unit vectors are the basis,
    and the residual is the sum of the squares left out."""
    diag = np.array([5.0, 4.0, 3.0, 2.0, 1.0, 0.5])
    X = np.zeros((8, 6))
    X[:6, :6] = np.diag(diag)
    D = np.eye(6)[:3]
    qv = oracle.basis_quality(X, D)
    assert qv["orth_err"] == 0.0
    assert abs(qv["residual"] - (4.0 + 1.0 + 0.25)) < 1e-12
    assert abs(qv["optimal"] - 5.25) < 1e-12 and abs(qv["ratio"] - 1.0) < 1e-12
    assert np.abs(qv["energy"] - np.array([25.0, 16.0, 9.0])).max() < 1e-12
    assert abs(qv["lead_capture"] - 1.0) < 1e-12 and qv["order_violation"] == 0.0
    assert qv["sin_angle"] < 1e-12
    # the exact truncated SVD of a generic matrix scores the same
    Xg = decaying(40, 24, 1)
    qg = oracle.basis_quality(Xg, oracle.bases(Xg, 7))
    assert qg["orth_err"] < 1e-12 and abs(qg["ratio"] - 1.0) < 1e-10
    assert abs(qg["lead_capture"] - 1.0) < 1e-10 and qg["sin_angle"] < 1e-8


def test_checker_catches_planted_mistakes():
    X = decaying(60, 32, 2)
    D = oracle.bases(X, 8)
    good = oracle.basis_quality(X, D)
    # rows in the wrong order: the subspace is optimal, its leading truncations are not
    swapped = D[[1, 0, 2, 3, 4, 5, 6, 7]]
    qs = oracle.basis_quality(X, swapped)
    assert abs(qs["ratio"] - 1.0) < 1e-10 and qs["order_violation"] > 1e-3 and qs["lead_capture"] < 0.999
    # a row scaled: not orthonormal
    scaled = D.copy()
    scaled[3] *= 1.01
    assert oracle.basis_quality(X, scaled)["orth_err"] > 1e-2
    # a random orthonormal basis: far from optimal
    R = np.linalg.qr(np.random.default_rng(3).standard_normal((32, 8)))[0].T
    qr_ = oracle.basis_quality(X, R)
    assert qr_["orth_err"] < 1e-12 and qr_["ratio"] > 1.5 and qr_["sin_angle"] > 0.5
    # a transposed operand cannot be expressed
    with pytest.raises(ValueError):
        oracle.basis_quality(X, D.T)
    # one singular vector replaced by a discarded one: the residual grows by exactly the difference
    S = good["sigma"]
    Vt = np.linalg.svd(X, full_matrices=False)[2]
    wrong = D.copy()
    wrong[7] = Vt[12]
    qw = oracle.basis_quality(X, wrong)
    assert abs(qw["residual"] - (good["optimal"] + S[7] ** 2 - S[12] ** 2)) < 1e-10


def test_randomized_scheme_tends_to_the_truncated_svd():
    """More power iterations: the residual falls to the Eckart-Young minimum and the rows to the
    singular vectors (up to sign); with a start block that already spans the leading directions
    one pass is exact."""
    X = decaying(120, 64, 4, power=1.0)
    r, l = 8, 16
    Om = np.random.default_rng(5).standard_normal((l, 64))
    ratios = []
    for q in (0, 1, 3, 12):
        D, sig = oracle.randomized_bases(X, Om, r, q)
        qv = oracle.basis_quality(X, D)
        assert qv["orth_err"] < 1e-10 and qv["order_violation"] < 1e-12
        ratios.append(qv["ratio"])
        assert np.abs(sig ** 2 - qv["energy"]).max() < 1e-9 * qv["energy"][0]     # sigma_i = ||X d_i||
    assert ratios[0] > ratios[1] > ratios[2] >= ratios[3] - 1e-12 and ratios[3] < 1.0005
    exact = oracle.bases(X, r)
    D, sig = oracle.randomized_bases(X, Om, r, 40)
    assert np.abs(np.abs(np.sum(D * exact, axis=1)) - 1.0).max() < 1e-6
    assert np.abs(sig - np.linalg.svd(X, compute_uv=False)[:r]).max() < 1e-8
    # a start block spanning the l leading right singular vectors (mixed by any invertible matrix)
    Vt = np.linalg.svd(X, full_matrices=False)[2]
    mix = np.random.default_rng(6).standard_normal((l, l))
    D0, _ = oracle.randomized_bases(X, mix @ Vt[:l], r, 0)
    assert np.abs(np.abs(np.sum(D0 * exact, axis=1)) - 1.0).max() < 1e-9
    # the published expectation bound for the plain range finder (no power iteration), Frobenius
    # norm: E||X - X P^T P||_F <= sqrt(1 + r/(p-1)) * sqrt(sum_{i>r} sigma_i^2) with p = l - r
    res = [oracle.basis_quality(X, oracle.randomized_bases(X, np.random.default_rng(10 + s).standard_normal((l, 64)), r, 0)[0])["ratio"]
           for s in range(20)]
    assert np.mean(np.sqrt(res)) <= np.sqrt(1 + r / (l - r - 1))


def test_decompress_is_the_retrieve_step():
    rng = np.random.default_rng(7)
    C = rng.standard_normal((5, 4))
    D = rng.standard_normal((4, 6))
    assert np.abs(oracle.decompress(C, D) - C @ D).max() < 1e-14
    rk = np.array([4, 2, 0, 1, 3])
    got = oracle.decompress(C, D, rk)
    for t in range(5):
        ref = [sum(C[t, j] * D[j, c] for j in range(rk[t])) for c in range(6)]
        assert np.abs(got[t] - np.array(ref)).max() < 1e-14
