"""Acceptance test, residual resampling and bonus token of SSD (test oracle).

Notation: pt = target distribution (the paper's q^s), pd = draft distribution (the paper's p^d),
x_i = draft tokens, r_i ~ U[0,1) acceptance uniforms, u the one uniform used to draw the emitted token.
 - Eq. 5 / Alg. 1: accept x_i iff r_i < min(1, pt_i(x_i) / pd_i(x_i)) + beta, scanning i = 1..K and
   stopping at the first failure; the ratio is the scalar ratio at the drafted token and beta is added
   outside the min.
 - Eq. 6: at the first rejection i, emit a token drawn from normalize(max(0, pt_i - pd_i)).
 - Alg. 1, all accepted: emit a token drawn from pt_{K+1}.
Two forms are given.  `*_plain` is the definition in fp64.  `*_canonical` is the same rule in the fixed
arithmetic a parallel machine can reproduce bit-for-bit: fp32 round-to-nearest divide/add for the
threshold, and an integer (2^40 fixed-point) inverse CDF so that the order of summation cannot matter.
Readings where the paper is silent: pd(x)=0 or pt(x)>=pd(x) gives threshold 1+beta (never a division by
zero); a residual with zero total mass falls back to drawing from pt_i; categorical draws use the inverse
CDF in index order (smallest j whose cumulative weight exceeds the target)."""
import numpy as np

FIX = 40                      # fixed-point fraction bits of the canonical sampler
UBITS = 24                    # uniforms live on the 2^-24 grid


# ----------------------------------------------------------------------------- plain fp64 definition
def threshold_plain(pt_x, pd_x, beta):
    """min(1, pt/pd) + beta   (Eq. 5), with the pd=0 reading above."""
    ratio = 1.0 if pd_x <= pt_x else pt_x / pd_x
    return min(1.0, ratio) + beta


def residual_plain(pt_row, pd_row):
    """Unnormalised max(0, pt - pd)   (Eq. 6)."""
    return np.maximum(0.0, np.asarray(pt_row, dtype=np.float64) - np.asarray(pd_row, dtype=np.float64))


def inverse_cdf_plain(weights, u):
    """Smallest j with (w_0 + .. + w_j) / sum(w) > u."""
    w = np.asarray(weights, dtype=np.float64)
    c = np.cumsum(w)
    j = int(np.searchsorted(c, u * c[-1], side="right"))
    return min(j, len(w) - 1)


def accept_plain(pt, pd, x, r, u, beta):
    """pt [K+1,V], pd [K,V], x [K] draft tokens, r [K] uniforms, u sampling uniform.
    Returns (n_accepted, emitted token)."""
    K = len(x)
    n = 0
    while n < K and r[n] < threshold_plain(pt[n][x[n]], pd[n][x[n]], beta):
        n += 1
    if n == K:
        return n, inverse_cdf_plain(pt[K], u)
    w = residual_plain(pt[n], pd[n])
    if w.sum() <= 0.0:
        w = np.asarray(pt[n], dtype=np.float64)
    return n, inverse_cdf_plain(w, u)


# ------------------------------------------------------------------- canonical fp32 / integer form
def threshold_canonical(pt_x, pd_x, beta):
    """fp32: pd > pt ? RN(RN(pt / pd) + beta) : RN(1 + beta)."""
    pt_x, pd_x, beta = np.float32(pt_x), np.float32(pd_x), np.float32(beta)
    if pd_x > pt_x:
        return np.float32(np.float32(pt_x / pd_x) + beta)
    return np.float32(np.float32(1.0) + beta)


def fixed_weights(w32):
    """floor(w * 2^40) of non-negative fp32 weights as exact Python-int-valued uint64 array."""
    w = np.asarray(w32, dtype=np.float32).astype(np.float64) * float(1 << FIX)      # exact scaling
    return np.floor(w).astype(np.uint64)


def inverse_cdf_fixed(W, u):
    """W uint64 fixed-point weights, u on the 2^-24 grid.  Returns (token, total); token is the smallest j
    with W_0 + .. + W_j > floor(total * (u * 2^24) / 2^24).  total == 0 returns token -1."""
    total = int(W.sum(dtype=np.uint64))
    if total == 0:
        return -1, 0
    Ru = int(round(float(u) * (1 << UBITS)))
    assert 0 <= Ru < (1 << UBITS) and Ru * 2.0 ** -UBITS == float(u), "uniform must lie on the 2^-24 grid"
    t = (total * Ru) >> UBITS
    c = np.cumsum(W, dtype=np.uint64)
    return int(np.searchsorted(c, np.uint64(t), side="right")), total


def accept_canonical(pt, pd, x, r, u, beta):
    """Same rule as accept_plain on fp32 inputs.  Returns (n_accepted, token, used_fallback)."""
    pt = np.asarray(pt, dtype=np.float32)
    pd = np.asarray(pd, dtype=np.float32).reshape(-1, pt.shape[1])
    K = len(x)
    n = 0
    while n < K and np.float32(r[n]) < threshold_canonical(pt[n, x[n]], pd[n, x[n]], beta):
        n += 1
    if n == K:
        tok, total = inverse_cdf_fixed(fixed_weights(pt[K]), u)
        return n, (tok if total else 0), False
    w = pt[n] - pd[n]                                   # fp32 subtraction, round to nearest
    tok, total = inverse_cdf_fixed(fixed_weights(np.maximum(w, np.float32(0.0))), u)
    if total:
        return n, tok, False
    tok, total = inverse_cdf_fixed(fixed_weights(pt[n]), u)
    return n, (tok if total else 0), True


def sample_canonical(p_row, u):
    """Draw from one fp32 probability row with the canonical sampler (draft tokens, AR decoding)."""
    tok, total = inverse_cdf_fixed(fixed_weights(np.asarray(p_row, dtype=np.float32)), u)
    return tok if total else 0
