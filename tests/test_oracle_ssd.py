"""Pins of the oracle's SSD cycle (Alg. 1) and of the paged-allocator model.  CPU only."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import decoder as D
from oracle import ssd as S
from oracle.kv_alloc import PagedAllocator
from oracle.warp import warp_probs


def setup(tname, dname, tseed, dseed, n_prefix=24, cap=160):
    ts, ds = si.model_shape(tname), si.model_shape(dname)
    t, d = D.Model(ts, si.make_weights(ts, tseed)), D.Model(ds, si.make_weights(ds, dseed))
    toks = si.make_prefix(ts, 0, n_prefix, 102)
    tc, dc = D.Cache(ts, cap), D.Cache(ds, cap)
    D.prefill(t, tc, toks[:-1])
    D.prefill(d, dc, toks[:-1])
    return t, d, tc, dc, int(toks[-1])


def test_greedy_ssd_reproduces_greedy_autoregressive_decoding():
    """beta = 0 with one-hot distributions: SSD emits exactly the target's greedy continuation,
    whatever the draft proposes."""
    t, d, tc, dc, pend = setup("tiny", "tiny_draft", 100, 101)
    cfg = S.sample_cfg(greedy=True, seed=1)
    ar = S.ar_generate(t, tc.copy(), pend, cfg, 24)
    for K in (1, 3, 4):
        out, ns = S.ssd_generate(t, d, tc.copy(), dc.copy(), pend, K, cfg, S.sample_cfg(greedy=True, seed=2), 24)
        assert out == ar
        assert all(0 <= n <= K for n in ns)
    assert len(set(ar)) > 3


def test_draft_equal_to_target_accepts_all_and_matches_its_own_ar_stream():
    """Draft == target: every cycle accepts K tokens (ratio 1), including the two-token catch-up path."""
    t, _, tc, _, pend = setup("tiny", "tiny_draft", 100, 101)
    cfg, dcfg = S.sample_cfg(seed=5), S.sample_cfg(seed=6)
    out, ns = S.ssd_generate(t, t, tc.copy(), tc.copy(), pend, 3, cfg, dcfg, 20)
    assert ns == [3] * len(ns) and len(out) == 20


def test_sampling_ssd_cycle_bookkeeping():
    t, d, tc, dc, pend = setup("tiny", "tiny_draft", 100, 101)
    cfg, dcfg = S.sample_cfg(beta=0.4, seed=1234), S.sample_cfg(seed=1235)
    L0 = tc.length
    tc2, dc2 = tc.copy(), dc.copy()
    out, ns = S.ssd_generate(t, d, tc2, dc2, pend, 4, cfg, dcfg, 40)
    emitted = sum(n + 1 for n in ns)
    assert tc2.length == L0 + emitted                       # L_acc grows by n+1 per cycle
    assert emitted >= 40 and len(out) == 40
    assert all(0 <= tok < t.shape["vocab"] for tok in out)
    # replay: teacher-forcing the emitted tokens through the target reproduces the cache it built
    tc3 = tc.copy()
    D.prefill(t, tc3, [pend] + out[:10])
    np.testing.assert_allclose(tc3.k[:, :L0 + 10], tc2.k[:, :L0 + 10], atol=1e-12)


def test_beta_increases_mean_accepted_length():
    """Table 3's trend: a larger tolerance accepts more draft tokens (same models, same uniforms)."""
    t, d, tc, dc, pend = setup("tiny", "tiny_draft", 100, 101)
    means = []
    for beta in (0.0, 0.2, 0.4):
        _, ns = S.ssd_generate(t, d, tc.copy(), dc.copy(), pend, 4, S.sample_cfg(beta=beta, temperature=0.05, seed=3),
                               S.sample_cfg(temperature=0.05, seed=4), 60)
        means.append(np.mean(ns))
    assert means[0] <= means[1] <= means[2] and means[0] + 0.2 < means[2]


def test_verify_step_k0_is_an_ar_step():
    t, _, tc, _, pend = setup("tiny", "tiny_draft", 100, 101)
    c = tc.copy()
    res = S.verify_step(t, c, pend, [], None, S.sample_cfg(), [], 0.5)
    assert res["n"] == 0 and c.length == tc.length + 1
    ref = warp_probs(D.forward_rows(t, tc.copy(), [pend]))
    np.testing.assert_allclose(res["pt"], ref, atol=1e-15)


# ---------------------------------------------------------------------------- allocator model
def test_allocator_model():
    a = PagedAllocator(n_blocks=10, block_tokens=16, max_seqs=2, max_blocks_per_seq=6)
    a.reserve(0, 20)                 # needs 2 blocks
    a.reserve(1, 5)                  # 1 block
    assert a.table[0][:2] == [0, 1] and a.table[1][:1] == [2]
    a.set_length(0, 20); a.set_length(1, 5)
    a.reserve(0, 13)                 # 33 positions -> 3 blocks
    assert a.table[0][:3] == [0, 1, 3]
    a.set_length(0, 32)              # exactly two full blocks: the third goes back
    assert a.owned[0] == 2 and a.free[-1] == 3
    a.reserve(0, 5)
    assert a.table[0][2] == 3        # re-allocation returns the same id
    a.set_length(0, 37)
    a.set_length(0, 3)               # rollback across blocks frees highest index first
    assert a.owned[0] == 1 and a.free[-2:] == [3, 1]
    assert a.slot(0, 2) == (0, 2)
    ids = a.table[0][:1] + a.table[1][:1] + a.free
    assert sorted(ids) == list(range(10))                    # nothing lost, nothing duplicated
    b = PagedAllocator(n_blocks=4, block_tokens=16, max_seqs=1, max_blocks_per_seq=8)
    with pytest.raises(MemoryError):
        b.reserve(0, 16 * 5)


def _first_token_law(draft_slot0, seed=2024, cycles=40000):
    """Empirical law of the first token a cycle emits when draft and target use ONE seed: x ~ pd drawn with the
    uniform of slot draft_slot0, then Eq. 5-6 with the verification's slots 0 (r_1) and 1 (the emitted token)."""
    from oracle.accept import accept_canonical, sample_canonical
    from oracle.philox import uniform24
    pd = np.array([[0.55, 0.25, 0.15, 0.05]], np.float32)
    pt = np.array([[0.10, 0.30, 0.20, 0.40], [0.25, 0.25, 0.25, 0.25]], np.float32)
    counts = np.zeros(4)
    for step in range(cycles):
        x = sample_canonical(pd[0], uniform24(seed, 0, step, draft_slot0))
        r, u = S.verify_uniforms(seed, 0, step, 1)
        n, nxt, _ = accept_canonical(pt, pd, [x], r, u, 0.0)
        counts[x if n == 1 else nxt] += 1
    return counts / cycles, pt[0].astype(np.float64)


def test_one_seed_for_draft_and_target_keeps_the_target_law():
    """Alg. 1 draws r_i afresh: with the draft's draws on slots of their own (oracle.ssd.DRAFT_SLOT0), a caller who
    gives both models the same seed still emits the target's law at beta = 0.  The mistake this guards against -
    drawing x_1 with the uniform that Eq. 5 then compares, i.e. slot 0 - couples the two and visibly bends the law."""
    law, pt = _first_token_law(S.DRAFT_SLOT0)
    assert np.abs(law - pt).max() < 0.01                    # 40000 cycles: three sigma is 0.0075
    assert S.draft_uniform(5, 1, 2, 3) != S.verify_uniforms(5, 1, 2, 4)[0][3]
    bent, _ = _first_token_law(0)                           # the planted mistake
    assert np.abs(bent - pt).max() > 0.05
