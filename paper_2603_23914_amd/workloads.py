"""Seeded synthetic inputs for the five benchmark/parity configurations.

This module holds NO arithmetic of the method (no projection, no attention,
no rank selection, no quantisation): only random draws, the planted low-rank
structure the configurations prescribe, and storage-format conversion.  Both
the CPU oracle's tests and the HIP path's tests/bench take their inputs here,
so the two sides always see identical stored bits.

The data stand in for LLaVA-1.5 / VideoLLaVA KV caches, which are not
available offline; only shapes follow those models (256 visual tokens per
image or frame, H=32/40 heads of d=128).
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Dict, Optional

import numpy as np

# ---------------------------------------------------------------------------
# storage formats
# ---------------------------------------------------------------------------

def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float array -> uint16 bfloat16 bit patterns, round-to-nearest-even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def store(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round a float64/float32 array to the storage dtype tag
    ("f32" | "f16" | "bf16").  bf16 is returned as uint16 bit patterns."""
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "f16":
        return np.ascontiguousarray(x, dtype=np.float16)
    if dtype == "bf16":
        return to_bf16_bits(x)
    raise ValueError(dtype)


def rng_for(seed: int, *path: int) -> np.random.Generator:
    """Independent PCG64 stream for (seed, path...)."""
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, *path])))


# ---------------------------------------------------------------------------
# building blocks
# ---------------------------------------------------------------------------

def spectrum(r: int, HD: int) -> np.ndarray:
    """kappa * sigma_j with sigma_j = j^-0.7 (j=1..r) and kappa chosen so that
    a cache row reconstructed with orthonormal bases has unit rms per hidden
    element (so raw logits q.k/sqrt(d) have unit variance for q ~ N(0,1))."""
    sigma = np.arange(1, r + 1, dtype=np.float64) ** -0.7
    kappa = math.sqrt(HD / float(np.sum(sigma ** 2)))
    return kappa * sigma


def coefficient_rows(rng: np.random.Generator, T: int, r: int, HD: int) -> np.ndarray:
    """[T, r] float64: C[t,j] = kappa*sigma_j*g + 0.01*n, g, n ~ N(0,1)."""
    ks = spectrum(r, HD)
    return rng.standard_normal((T, r)) * ks[None, :] + 0.01 * rng.standard_normal((T, r))


def orthonormal_rows(rng: np.random.Generator, r: int, HD: int) -> np.ndarray:
    """[r, HD] float64 with orthonormal rows: Q^T from the QR of a Gaussian [HD, r]."""
    qmat, _ = np.linalg.qr(rng.standard_normal((HD, r)))
    return np.ascontiguousarray(qmat.T)


def vary_basis(rng: np.random.Generator, base: np.ndarray) -> np.ndarray:
    """A per-sequence basis derived from `base` by a seeded permutation and sign
    flip of its hidden columns.  Rows stay orthonormal; one QR serves a batch."""
    HD = base.shape[1]
    perm = rng.permutation(HD)
    sign = rng.integers(0, 2, size=HD) * 2.0 - 1.0
    return np.ascontiguousarray(base[:, perm] * sign[None, :])


# ---------------------------------------------------------------------------
# configuration 1: tiny fp32 case
# ---------------------------------------------------------------------------

def config1(seed: int = 0) -> Dict[str, np.ndarray]:
    """B=1, H=4, d=32, T=64, r=16.  K = U W + 0.01 N(0,1) with U [64,16],
    W [16,128] i.i.d. N(0, variance 1/sqrt(16)) so that entries of U W have
    unit variance; V likewise from independent draws; q ~ N(0,1).
    Bases are NOT produced here (they are an SVD, i.e. part of the method)."""
    rng = rng_for(seed, 1)
    H, d, T, r = 4, 32, 64, 16
    std = math.sqrt(1.0 / math.sqrt(16.0))
    out = {}
    for name in ("K", "V"):
        U = rng.standard_normal((T, r)) * std
        W = rng.standard_normal((r, H * d)) * std
        out[name] = U @ W + 0.01 * rng.standard_normal((T, H * d))
    out["q"] = rng.standard_normal((H, d))
    out.update(H=H, d=d, T=T, r=r)
    return out


# ---------------------------------------------------------------------------
# configurations 2, 3, 4: decode over directly generated coefficients
# ---------------------------------------------------------------------------

@dataclass
class DecodeCase:
    """Stored inputs of a decode workload (host arrays, already rounded)."""
    dtype: str
    B: int
    H: int
    d: int
    r: int
    T0: int                 # tokens cached before the first step
    T_cap: int
    steps: int
    Ck: np.ndarray          # [B, T_cap, r] storage dtype (rows >= T0 zero)
    Cv: np.ndarray
    Bk: np.ndarray          # [B, r, HD] (per-sequence) or [r, HD] (shared)
    Bv: np.ndarray
    seed: int

    @property
    def HD(self) -> int:
        return self.H * self.d


def decode_case(dtype: str, B: int, H: int, d: int, r: int, T0: int, steps: int,
                seed: int = 0, shared_basis: bool = False, append: bool = True,
                batch_subset: Optional[range] = None) -> DecodeCase:
    """Coefficients drawn in the law compaction of a planted-basis cache would
    give; bases orthonormal (one QR per K and V, varied per sequence)."""
    HD = H * d
    T_cap = T0 + (steps if append else 0)
    zero = store(np.zeros(1), dtype)[0]
    Ck = np.full((B, T_cap, r), zero, dtype=store(np.zeros(1), dtype).dtype)
    Cv = Ck.copy()
    base_k = orthonormal_rows(rng_for(seed, 20), r, HD)
    base_v = orthonormal_rows(rng_for(seed, 21), r, HD)
    if shared_basis:
        Bk = store(base_k, dtype)
        Bv = store(base_v, dtype)
    else:
        Bk = np.empty((B, r, HD), dtype=Ck.dtype)
        Bv = np.empty((B, r, HD), dtype=Ck.dtype)
    for b in (range(B) if batch_subset is None else batch_subset):
        Ck[b, :T0] = store(coefficient_rows(rng_for(seed, 22, b), T0, r, HD), dtype)
        Cv[b, :T0] = store(coefficient_rows(rng_for(seed, 23, b), T0, r, HD), dtype)
        if not shared_basis:
            Bk[b] = store(vary_basis(rng_for(seed, 24, b), base_k), dtype)
            Bv[b] = store(vary_basis(rng_for(seed, 25, b), base_v), dtype)
    return DecodeCase(dtype, B, H, d, r, T0, T_cap, steps, Ck, Cv, Bk, Bv, seed)


def step_query(case: DecodeCase, step: int) -> np.ndarray:
    """q [B, H, d] ~ N(0,1) for a decode step, rounded to the storage dtype."""
    return store(rng_for(case.seed, 30, step).standard_normal((case.B, case.H, case.d)), case.dtype)


def step_new_token(case: DecodeCase, step: int, Bk64: np.ndarray, Bv64: np.ndarray):
    """Raw key/value rows [B, HD] of the token appended at `step`:
    x = c_new . B + 0.01 N(0,1) with c_new from the coefficient law.
    Bk64/Bv64: the bases as float64 ([B, r, HD] or [r, HD])."""
    rng = rng_for(case.seed, 31, step)
    ks = spectrum(case.r, case.HD)
    outs = []
    for Bm in (Bk64, Bv64):
        c = rng.standard_normal((case.B, case.r)) * ks[None, :]
        if Bm.ndim == 3:
            x = np.einsum("br,brh->bh", c, Bm)
        else:
            x = c @ Bm
        x = x + 0.01 * rng.standard_normal((case.B, case.HD))
        outs.append(store(x, case.dtype))
    return outs[0], outs[1]


def config2(seed: int = 0, **kw) -> DecodeCase:
    """LLaVA-1.5-7B-shaped: B=8, H=32, d=128, T=4*256+64=1088 (+128 appended), r=512, fp16."""
    return decode_case("f16", 8, 32, 128, 512, 1088, 128, seed, **kw)


def config3(seed: int = 0, **kw) -> DecodeCase:
    """LLaVA-13B-shaped batch decode: B=64, H=40, d=128, T=16*256+128=4224 (+64), r=640, bf16."""
    return decode_case("bf16", 64, 40, 128, 640, 4224, 64, seed, **kw)


def config4(seed: int = 0, **kw) -> DecodeCase:
    """Long-context video: B=1, H=32, d=128, T=128*256=32768, r_max=512, fp16, no append."""
    return decode_case("f16", 1, 32, 128, 512, 32768, 128, seed, append=False, **kw)


C4_GROUP_RANK = (512, 256, 128, 64)
C4_CUM_NUM = (1, 2, 3, 4)
C4_DEN = 4
C4_RESELECT_EVERY = 32
C4_ALPHA = 0.25


def zipf_mass(T: int, seed: int, epoch: int) -> np.ndarray:
    """Attention-mass draw for configuration 4: w_t = (1+pi(t))^-1.1 with pi a
    seeded permutation of positions; +1 on the first 8 and the last 256
    positions (attention sinks and recency); normalised to sum 1.  float64."""
    rng = rng_for(seed, 40, epoch)
    w = (1.0 + rng.permutation(T).astype(np.float64)) ** -1.1
    w[:8] += 1.0
    w[T - min(256, T):] += 1.0
    return w / w.sum()


def config4_mass(T: int, seed: int, epoch: int) -> np.ndarray:
    """float32 importance fed to rank selection at reselect number `epoch`
    (0 = before the first step).  Epoch e>0 mixes a fresh draw into the
    previous mass with weights (alpha, 1-alpha), alpha = 0.25 (moving average
    of the paper's Eq. 1, supplied here as data)."""
    m = zipf_mass(T, seed, 0)
    for e in range(1, epoch + 1):
        m = C4_ALPHA * m + (1.0 - C4_ALPHA) * zipf_mass(T, seed, e)
    return m.astype(np.float32)


# ---------------------------------------------------------------------------
# configuration 5: materialised K, V for compaction (+ int8 coefficients)
# ---------------------------------------------------------------------------

def config5_sequence(b: int, seed: int = 0, T: int = 4224, HD: int = 4096, r: int = 512,
                     dtype: str = "f16"):
    """One sequence of configuration 5.  K = G diag(kappa sigma) B2 + 0.01 N
    with r2 = 2r planted orthonormal directions B2 (energy beyond rank r is
    real); the basis handed to compaction is the first r rows of B2.
    Returns (K, V, Bk, Bv) rounded to `dtype`."""
    r2 = 2 * r
    out = []
    for which in (0, 1):
        B2 = orthonormal_rows(rng_for(seed, 50 + which), r2, HD)
        B2 = vary_basis(rng_for(seed, 52 + which, b), B2)
        ks = spectrum(r2, HD)
        rng = rng_for(seed, 54 + which, b)
        G = rng.standard_normal((T, r2)) * ks[None, :]
        X = G @ B2 + 0.01 * rng.standard_normal((T, HD))
        out.append((store(X, dtype), store(B2[:r], dtype)))
    (K, Bk), (V, Bv) = out
    return K, V, Bk, Bv
