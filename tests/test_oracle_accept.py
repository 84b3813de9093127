"""Pins of the oracle's acceptance / resampling rule (Eq. 5-6, Alg. 1).  CPU only."""
import itertools
import os

import numpy as np
import pytest

import synth_inputs as si
from oracle import accept as A

GOLD = os.path.join(os.path.dirname(__file__), "golden", "accept_worked_examples.txt")


def grid(u):
    """Snap to the 2^-24 grid the canonical form requires."""
    return round(u * (1 << 24)) / (1 << 24)


def load_examples():
    out = []
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        f = [s.strip() for s in line.split(";")]
        rows = lambda s: np.array([[float(v) for v in r.split()] for r in s.split(",")])
        out.append(dict(beta=float(f[0]), pt=rows(f[1]), pd=rows(f[2]), x=[int(v) for v in f[3].split()],
                        r=[float(v) for v in f[4].split()], u=float(f[5]), n=int(f[6]), tok=int(f[7]), why=f[8]))
    return out


@pytest.mark.parametrize("ex", load_examples(), ids=lambda e: e["why"][:40])
def test_hand_worked_examples(ex):
    n, tok = A.accept_plain(ex["pt"], ex["pd"], ex["x"], ex["r"], ex["u"], ex["beta"])
    assert (n, tok) == (ex["n"], ex["tok"])
    n, tok, fb = A.accept_canonical(ex["pt"], ex["pd"], ex["x"], [grid(v) for v in ex["r"]], grid(ex["u"]), ex["beta"])
    assert (n, tok, fb) == (ex["n"], ex["tok"], False)


def cycle_law(pt_of, pd_of, V, K, beta):
    """Exact law over strings of length K+1 of: the tokens one SSD cycle emits, completed by the target's
    own conditionals where the cycle emitted fewer than K+1.  Integrates the uniforms analytically
    (P(r < thr) = clip(thr, 0, 1)) and enumerates every draft string and rejection position, using the
    oracle's threshold and residual functions."""
    law = {s: 0.0 for s in itertools.product(range(V), repeat=K + 1)}

    def complete(prefix, mass):
        if mass == 0.0:
            return
        if len(prefix) == K + 1:
            law[prefix] += mass
            return
        p = pt_of(prefix)
        for y in range(V):
            complete(prefix + (y,), mass * p[y])

    def cycle(ctx, mass):
        """`ctx` = draft tokens accepted so far in this cycle, reached with probability `mass`."""
        pt = pt_of(ctx)
        if len(ctx) == K:                                      # all accepted: bonus token from pt_{K+1}
            for y in range(V):
                complete(ctx + (y,), mass * pt[y])
            return
        pd = pd_of(ctx)
        for x in range(V):
            mass_x = mass * pd[x]                              # the draft proposes x
            if mass_x == 0.0:
                continue
            a = min(1.0, max(0.0, A.threshold_plain(pt[x], pd[x], beta)))
            if a < 1.0:                                        # rejected with probability 1 - a
                w = A.residual_plain(pt, pd)
                if w.sum() <= 0:
                    w = pt
                for y in range(V):
                    complete(ctx + (y,), mass_x * (1 - a) * w[y] / w.sum())
            cycle(ctx + (x,), mass_x * a)

    cycle((), 1.0)
    return law


def random_tables(V, K, seed, zeros):
    rng = np.random.default_rng(seed)
    tabs = {}
    for n in range(K + 1):
        for ctx in itertools.product(range(V), repeat=n):
            tabs[ctx] = (si.make_probs(rng, 1, V, 0.7, zeros)[0].astype(np.float64),
                         si.make_probs(rng, 1, V, 0.7, zeros)[0].astype(np.float64))
    for k in tabs:
        tabs[k] = (tabs[k][0] / tabs[k][0].sum(), tabs[k][1] / tabs[k][1].sum())
    return tabs


@pytest.mark.parametrize("V,K,zeros", [(4, 1, 0.0), (5, 2, 0.3), (4, 3, 0.2), (8, 2, 0.0)])
def test_beta0_cycle_law_equals_target_law(V, K, zeros):
    """Sec. 2.2: with the strict rule (beta = 0) the emitted tokens follow the target's distribution."""
    tabs = random_tables(V, K, 11 + V + K, zeros)
    law = cycle_law(lambda c: tabs[c][0], lambda c: tabs[c][1], V, K, 0.0)
    for s, got in law.items():
        want = np.prod([tabs[s[:i]][0][s[i]] for i in range(K + 1)])
        assert abs(got - want) < 1e-12
    assert abs(sum(law.values()) - 1) < 1e-12


def test_beta_positive_law_is_a_distribution_and_leans_to_the_draft():
    V, K = 4, 2
    tabs = random_tables(V, K, 5, 0.0)
    law0 = cycle_law(lambda c: tabs[c][0], lambda c: tabs[c][1], V, K, 0.0)
    law4 = cycle_law(lambda c: tabs[c][0], lambda c: tabs[c][1], V, K, 0.4)
    assert abs(sum(law4.values()) - 1) < 1e-12
    first = lambda law, y: sum(m for s, m in law.items() if s[0] == y)
    pt, pd = tabs[()]
    for y in range(V):
        # tolerance moves mass only from "target" toward "draft" on the first token
        lo, hi = min(pt[y], pd[y]) - 1e-12, max(pt[y], pd[y]) + 1e-12
        assert lo <= first(law4, y) <= hi
        assert abs(first(law0, y) - pt[y]) < 1e-12
    assert max(abs(first(law4, y) - pt[y]) for y in range(V)) > 1e-3


def test_decisions_integrate_to_the_target_distribution():
    """Brute force over a fine grid of (r, u): the decision function itself (strict <, inverse CDF
    direction, canonical fixed point) emits y with frequency pt(y) when the draft token is drawn from pd."""
    rng = np.random.default_rng(9)
    V, N = 5, 192
    pt = si.make_probs(rng, 2, V, 0.8)
    pd = si.make_probs(rng, 1, V, 0.8)
    us = [grid((i + 0.5) / N) for i in range(N)]
    freq = np.zeros(V)
    for x in range(V):
        for r in us:
            for u in us:
                n, tok, _ = A.accept_canonical(pt, pd, [x], [r], u, 0.0)
                freq[x if n == 1 else tok] += pd[0, x] / (N * N)
    assert np.abs(freq - pt[0]).max() < 2.0 / N


def test_draft_equals_target_accepts_everything():
    rng = np.random.default_rng(4)
    V, K = 37, 6
    for trial in range(50):
        p = si.make_probs(rng, K + 1, V, 0.5, zeros=0.2)
        x = [int(rng.choice(V, p=p[i].astype(np.float64) / p[i].astype(np.float64).sum())) for i in range(K)]
        r = [grid(1 - 2.0 ** -24)] * K                        # the largest uniform there is
        n, _, _ = A.accept_canonical(p, p[:K], x, r, grid(rng.random()), 0.0)
        assert n == K
        assert A.accept_plain(p, p[:K], x, r, 0.3, 0.0)[0] == K


def test_beta_saturation_and_monotonicity():
    rng = np.random.default_rng(6)
    V, K = 23, 5
    for trial in range(100):
        pt = si.make_probs(rng, K + 1, V, 0.4, zeros=0.3)
        pd = si.make_probs(rng, K, V, 0.4)
        x = [int(rng.integers(V)) for _ in range(K)]
        r = [grid(rng.random()) for _ in range(K)]
        u = grid(rng.random())
        ns = [A.accept_canonical(pt, pd, x, r, u, b)[0] for b in (0.0, 0.1, 0.2, 0.3, 0.4, 1.0)]
        assert ns == sorted(ns)                               # more tolerance never accepts fewer
        assert ns[-1] == K                                    # beta >= 1 accepts all, even pt(x) = 0


def test_rejected_token_is_never_reemitted():
    rng = np.random.default_rng(7)
    V, K = 11, 3
    seen = 0
    for trial in range(400):
        pt = si.make_probs(rng, K + 1, V, 0.5)
        pd = si.make_probs(rng, K, V, 0.5)
        x = [int(rng.integers(V)) for _ in range(K)]
        r = [grid(rng.random()) for _ in range(K)]
        n, tok, fb = A.accept_canonical(pt, pd, x, r, grid(rng.random()), 0.0)
        if n < K:
            seen += 1
            assert not fb
            assert pt[n, x[n]] < pd[n, x[n]]                  # a rejection implies pt(x) < pd(x)
            assert tok != x[n] and pt[n, tok] > pd[n, tok]    # emitted token has positive residual
    assert seen > 100


def test_canonical_matches_plain_away_from_boundaries():
    rng = np.random.default_rng(8)
    V, K = 300, 4
    agree = total = 0
    for trial in range(300):
        pt = si.make_probs(rng, K + 1, V, 0.5)
        pd = si.make_probs(rng, K, V, 0.5)
        x = [int(rng.choice(V, p=pd[i].astype(np.float64) / pd[i].astype(np.float64).sum())) for i in range(K)]
        r = [grid(rng.random()) for _ in range(K)]
        u = grid(rng.random())
        beta = [0.0, 0.4][trial % 2]
        a = A.accept_plain(pt.astype(np.float64), pd.astype(np.float64), x, r, u, beta)
        b = A.accept_canonical(pt, pd, x, r, u, beta)[:2]
        total += 1
        agree += (a == b)
    assert agree >= total - 1          # a uniform may fall within rounding of a boundary, rarely


def test_inverse_cdf_fixed_brute_force():
    """Exhaustive check of the integer inverse CDF against rational arithmetic on small cases."""
    from fractions import Fraction
    rng = np.random.default_rng(10)
    for trial in range(200):
        V = int(rng.integers(1, 9))
        w = (rng.random(V) * (rng.random(V) > 0.3)).astype(np.float32)
        W = A.fixed_weights(w)
        Wi = [int(Fraction(float(v)) * (1 << 40)) for v in w]         # floor for non-negative values
        assert [int(v) for v in W] == Wi
        u = grid(rng.random())
        tok, total = A.inverse_cdf_fixed(W, u)
        if sum(Wi) == 0:
            assert tok == -1
            continue
        t = (sum(Wi) * int(u * (1 << 24))) >> 24
        want = next(j for j in range(V) if sum(Wi[:j + 1]) > t)
        assert tok == want and Wi[tok] > 0


def test_zero_residual_falls_back_to_target_row():
    # rows that are equal in fp32 except that the drafted token is (inconsistently) rejected cannot occur in
    # exact arithmetic; the API accepts arbitrary rows, so construct one: residual identically zero.
    pt = np.array([[0.25, 0.25, 0.5], [1.0, 0.0, 0.0]], dtype=np.float32)
    pd = np.array([[0.5, 0.5, 1.0]], dtype=np.float32)                 # unnormalised on purpose: pd >= pt
    n, tok, fb = A.accept_canonical(pt, pd, [2], [grid(0.9)], grid(0.6), 0.0)
    assert (n, tok, fb) == (0, 2, True)


def test_subnormal_probabilities():
    tiny = np.float32(1e-41)                                           # subnormal in fp32
    pt = np.array([[tiny, 1.0, 0.0], [0.0, 1.0, 0.0]], dtype=np.float32)
    pd = np.array([[np.float32(4e-41), 1.0, 0.0]], dtype=np.float32)
    thr = A.threshold_canonical(pt[0, 0], pd[0, 0], 0.0)
    assert abs(float(thr) - 0.25) < 1e-3                               # gradual underflow is honoured
    assert A.accept_canonical(pt, pd, [0], [grid(0.2)], 0.0, 0.0)[0] == 1
    assert A.accept_canonical(pt, pd, [0], [grid(0.3)], 0.0, 0.0)[0] == 0
