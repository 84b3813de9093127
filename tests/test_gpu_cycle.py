"""GPU tests of the pieces around the verification: draft steps and whole SSD cycles in lockstep with the
oracle, batches with ragged lengths, rollback, pool exhaustion, and row-count invariance (greedy SSD ==
greedy autoregressive decoding on the GPU itself)."""
import numpy as np
import pytest
import torch

import synth_inputs as si

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2505_15380_amd as pkg
    pkg.load_library()


def make_session(workload, K, beta=0.0, greedy=False, n_prefix=40, steps=12, temperature=None, draft_is_target=False,
                 models=None):
    """`models` = (target shape, target weights, draft shape, draft weights) replaces the workload's own pair."""
    import paper_2505_15380_amd as ssd
    wl = si.workload(workload)
    if models is not None:
        ts, tw, ds, dw = models
    else:
        ts, ds = si.model_shape(wl["target"]), si.model_shape(wl["draft"])
        tw, dw = si.make_weights(ts, wl["seeds"]["target"]), si.make_weights(ds, wl["seeds"]["draft"])
    if draft_is_target:
        ds, dw = ts, tw
    toks = si.make_prefix(ts, 5, n_prefix, wl["seeds"]["prefix"])
    T = wl["temperature"] if temperature is None else temperature
    cfg = dict(beta=beta, temperature=T, top_k=0, greedy=greedy, seed=77)
    dcfg = dict(beta=0.0, temperature=T, top_k=0, greedy=greedy, seed=78)
    max_pos = len(toks) + steps * (K + 1) + 40
    sess = ssd.SSDSession(ts, tw, ds, dw, 1, K, max_pos, ssd.sample_config(**cfg), ssd.sample_config(**dcfg))
    sess.prefill(0, torch.from_numpy(toks).cuda())
    return sess, (ts, tw, ds, dw, toks, cfg, dcfg, max_pos)


@pytest.mark.parametrize("workload,tol", [("tiny", 1e-5), ("mini", 2e-2)])
@pytest.mark.parametrize("beta", [0.0, 0.4])
def test_ssd_cycles_in_lockstep_with_oracle(workload, tol, beta):
    """Draft steps (Eq. 2-3) and verification (Eq. 4-6) over several cycles, including the two-token catch-up
    after a fully accepted cycle.  Every draft distribution and target distribution is compared; every drawn
    token and decision must equal the oracle's canonical rule applied to the GPU's own fp32 probabilities."""
    run_cycles_in_lockstep(workload, tol, beta, K=3, steps=10, require_both=True)


def run_cycles_in_lockstep(workload, tol, beta, K, steps, require_both, n_prefix=40, sharp_steps=True, models=None):
    import paper_2505_15380_amd as ssd
    from oracle import decoder as OD, ssd as OS
    from oracle.accept import sample_canonical, accept_canonical
    from oracle.philox import uniform24
    from oracle.warp import warp_probs
    sess, (ts, tw, ds, dw, toks, cfg, dcfg, max_pos) = make_session(workload, K, beta=beta, steps=steps, n_prefix=n_prefix,
                                                                    models=models)
    t, d = OD.Model(ts, tw), OD.Model(ds, dw)
    tc, dc = OD.Cache(ts, max_pos), OD.Cache(ds, max_pos)
    OD.prefill(t, tc, toks[:-1]); OD.prefill(d, dc, toks[:-1])
    pending, dpend = int(toks[-1]), [int(toks[-1])]
    V = ts["vocab"]
    seen_full = seen_reject = False
    draft_paths = set()
    ns = []
    for step in range(steps):
        # alternate a flat and a sharp temperature so that full acceptance and rejection both occur
        # (a temperature of 0.05 multiplies the logits' error by 20: only where the tolerance has that room)
        cfg["temperature"] = dcfg["temperature"] = 1.0 if (step % 2 == 0 or not sharp_steps) else 0.05
        sess.cfg, sess.dcfg = ssd.sample_config(**cfg), ssd.sample_config(**dcfg)
        out = dict(n_accepted=torch.zeros(1, dtype=torch.int32, device="cuda"),
                   next_token=torch.zeros(1, dtype=torch.int32, device="cuda"),
                   probs=torch.zeros((1, K + 1, V), dtype=torch.float32, device="cuda"), logits=None)
        sess.cycle(step, out=out)
        torch.cuda.synchronize()
        draft_paths.add(sess.kv_d.last_forward_path())
        gx, gpd = sess.x.cpu().numpy()[0], sess.pd.cpu().numpy()[0]
        # oracle draft steps, teacher-forced with the GPU's tokens
        for i in range(K):
            lg = OD.forward_rows(d, dc, dpend)
            dc.length += len(dpend)
            ref = warp_probs(lg[-1:], dcfg["temperature"])[0]
            assert np.abs(gpd[i] - ref).max() <= tol, (step, i)
            tok = sample_canonical(gpd[i], OS.draft_uniform(dcfg["seed"], 0, step, i))
            assert tok == int(gx[i]), (step, i)
            dpend = [tok]
        r, u = OS.verify_uniforms(cfg["seed"], 0, step, K)
        L = tc.length
        gp = out["probs"].cpu().numpy()[0]
        res = OS.verify_step(t, tc, pending, list(gx), gpd, OS.sample_cfg(**cfg), r, u, pt32=gp)
        assert np.abs(gp - res["pt"]).max() <= tol
        assert (int(out["n_accepted"][0]), int(out["next_token"][0])) == (res["n"], res["next"])
        n, pending = res["n"], res["next"]
        ns.append(n)
        if n < K:
            dc.length = L + 1 + n; dpend = [pending]; seen_reject = True
        else:
            dpend = [int(gx[-1]), pending]; seen_full = True
        st, sd = sess.kv.state(0), sess.kv_d.state(0)
        assert st["len"] == tc.length and st["pending"] == [pending]
        assert sd["len"] == dc.length and sd["pending"] == dpend
    assert (seen_reject and seen_full) or not require_both, ns
    sess.draft_paths_seen = draft_paths
    sess.accepted_seen = ns
    return sess


def test_cycles_with_a_layer_inheritance_draft_in_lockstep_with_oracle():
    """The draft the paper builds (Sec. 2.3): the target's lower and upper layers, its embeddings and its head, here
    without the fine-tuning: a 6-layer target of the small bf16 shape with a peaked head, draft = layers 0, 1, 4, 5.
    Cycles in lockstep with the oracle as above; such a draft agrees with its target far more often than an unrelated
    one, so full acceptances and rejections both occur at beta = 0."""
    ts = si.model_shape("mini_bf16")
    ts["n_layers"] = 6
    tw = si.make_weights(ts, 9100)
    tw["head"] = si.round_to_bf16(tw["head"] * np.float32(6.0))           # peaked distributions
    ds, dw = si.correlated_draft_weights(ts, tw, 4, n_lower=2)
    sess = run_cycles_in_lockstep("mini", 2e-2, 0.0, K=3, steps=14, require_both=True, sharp_steps=False,
                                  models=(ts, tw, ds, dw))
    assert sess.kv.last_forward_path() == 3
    # and the same pair under the tolerance of Eq. 5: more is accepted (Table 3's trend), still in lockstep
    sess2 = run_cycles_in_lockstep("mini", 2e-2, 0.4, K=3, steps=14, require_both=False, sharp_steps=False,
                                   models=(ts, tw, ds, dw))
    assert sum(sess2.accepted_seen) >= sum(sess.accepted_seen)


@pytest.mark.parametrize("workload", ["tiny", "mini"])
def test_greedy_ssd_equals_greedy_ar_on_gpu(workload):
    """beta = 0, greedy: the SSD output is the target's own greedy continuation token for token; on the GPU this
    also requires that a row verified among K+1 rows has the bits it has when decoded alone."""
    K, n_tok = 4, 24
    sess, _ = make_session(workload, K, greedy=True, steps=n_tok + 4)
    ar = []
    for s in range(n_tok):
        out = sess.ar_step(s)
        ar.append(int(out["next_token"][0]))
    sess2, _ = make_session(workload, K, greedy=True, steps=n_tok + 4)
    got = []
    step = 0
    while len(got) < n_tok:
        out = sess2.cycle(step)
        torch.cuda.synchronize()
        n = int(out["n_accepted"][0])
        got += [int(v) for v in sess2.x[0, :n]] + [int(out["next_token"][0])]
        step += 1
    assert got[:n_tok] == ar
    assert len(set(ar)) > 2


def test_draft_equal_to_target_accepts_everything():
    K = 4
    sess, _ = make_session("mini", K, beta=0.0, draft_is_target=True, steps=8)
    for step in range(6):
        out = sess.cycle(step)
        assert int(out["n_accepted"][0]) == K
    assert sess.kv.state(0)["len"] == sess.kv_d.state(0)["len"] + 1      # the draft owes x_K


@pytest.mark.parametrize("workload,tol", [("tiny", 1e-5), ("mini", 2e-2)])
def test_batched_ragged_verify_parity(workload, tol):
    """Several sequences of different lengths in one call; per-sequence accept counts differ, blocks are shared
    from one pool (block size 16), and the allocator state must follow the model exactly."""
    from tests.parity import Pair, verify_parity_step
    wl = si.workload(workload)
    shape = si.model_shape(wl["target"])
    B, K, steps = 3, 4, 5
    lens = [23, 70, 49]
    pair = Pair(wl["target"], wl["seeds"]["target"], 70 + steps * (K + 1) + 20, max_seqs=B, max_rows=8,
                n_blocks=3 * 8 + 2, block_tokens=16)
    for b in range(B):
        pair.prefill(b, si.make_prefix(shape, 3, lens[b] - 3, 900 + b))
    for b in range(B):
        pair.check_state(b, tol)
    pair.check_free_stack()
    rng = np.random.default_rng(5)
    cfg = dict(beta=0.1, temperature=1.0, top_k=0, greedy=False, seed=4321)
    ns = []
    for s in range(steps):
        res = verify_parity_step(pair, cfg, K, s, rng, tol, tol, seqs=tuple(range(B)))
        ns.append([r["n"] for r in res])
        for b in range(B):
            pair.check_state(b, tol, layers=[shape["n_layers"] - 1])
        pair.check_free_stack()
    assert len({tuple(n) for n in ns}) > 1 and any(len(set(n)) > 1 for n in ns)


def test_draft_attention_mode_changes_with_the_prefix():
    """The draft's launches take attention without parts while the host's bound of the cached length allows it (1520
    positions) and attention in parts beyond: cycles in lockstep with the oracle across that length."""
    sess = run_cycles_in_lockstep("mini", 2e-2, 0.4, K=3, steps=12, require_both=False, n_prefix=1490)
    assert sess.draft_paths_seen == {3, 4}
    assert sess.kv_d.state(0)["len"] > 1520


@pytest.mark.parametrize("B,K,target_path", [(4, 3, 3), (16, 2, 1)])
def test_batched_cycles_in_lockstep_with_oracle(B, K, target_path):
    """Whole SSD cycles of several sequences at once: after a verification some sequences have one pending draft row and
    some two (everything accepted), so one draft launch mixes active and inactive rows, the draft caches roll back by
    different amounts, and every sequence is followed by an oracle of its own.  Four sequences stay on the persistent
    kernels throughout; sixteen have 16-row draft steps there, 32-row first steps and the verification per operator."""
    import paper_2505_15380_amd as ssd
    from oracle import decoder as OD, ssd as OS
    from oracle.accept import sample_canonical
    from oracle.philox import uniform24
    from oracle.warp import warp_probs
    wl = si.workload("mini")
    ts, ds = si.model_shape(wl["target"]), si.model_shape(wl["draft"])
    tw, dw = si.make_weights(ts, wl["seeds"]["target"]), si.make_weights(ds, wl["seeds"]["draft"])
    steps, tol = 8, 2e-2
    lens = [21, 40, 33, 64, 17, 90, 48, 31, 16, 75, 52, 29, 63, 44, 36, 81][:B]
    toks = [si.make_prefix(ts, 4, n - 4, 500 + b) for b, n in enumerate(lens)]
    cfg = dict(beta=0.5, temperature=1.0, top_k=0, greedy=False, seed=31)
    dcfg = dict(beta=0.0, temperature=1.0, top_k=0, greedy=False, seed=32)
    max_pos = max(lens) + steps * (K + 1) + 40
    sess = ssd.SSDSession(ts, tw, ds, dw, B, K, max_pos, ssd.sample_config(**cfg), ssd.sample_config(**dcfg))
    t, d = OD.Model(ts, tw), OD.Model(ds, dw)
    tc, dc, pending, dpend = [], [], [], []
    for b in range(B):
        sess.prefill(b, torch.from_numpy(toks[b]).cuda())
        tc.append(OD.Cache(ts, max_pos)); dc.append(OD.Cache(ds, max_pos))
        OD.prefill(t, tc[b], toks[b][:-1]); OD.prefill(d, dc[b], toks[b][:-1])
        pending.append(int(toks[b][-1])); dpend.append([int(toks[b][-1])])
    V = ts["vocab"]
    mixed = False
    for step in range(steps):
        out = dict(n_accepted=torch.zeros(B, dtype=torch.int32, device="cuda"),
                   next_token=torch.zeros(B, dtype=torch.int32, device="cuda"),
                   probs=torch.zeros((B, K + 1, V), dtype=torch.float32, device="cuda"), logits=None)
        sess.cycle(step, out=out)
        torch.cuda.synchronize()
        assert sess.kv.last_forward_path() == target_path and sess.kv_d.last_forward_path() in (3, 4)
        gx, gpd, gp = sess.x.cpu().numpy(), sess.pd.cpu().numpy(), out["probs"].cpu().numpy()
        ns = []
        for b in range(B):
            for i in range(K):                            # the oracle's draft steps, teacher-forced with the GPU's tokens
                lg = OD.forward_rows(d, dc[b], dpend[b])
                dc[b].length += len(dpend[b])
                ref = warp_probs(lg[-1:], dcfg["temperature"])[0]
                assert np.abs(gpd[b, i] - ref).max() <= tol, (step, b, i)
                tok = sample_canonical(gpd[b, i], OS.draft_uniform(dcfg["seed"], b, step, i))
                assert tok == int(gx[b, i]), (step, b, i)
                dpend[b] = [tok]
            r, u = OS.verify_uniforms(cfg["seed"], b, step, K)
            L = tc[b].length
            res = OS.verify_step(t, tc[b], pending[b], list(gx[b]), gpd[b], OS.sample_cfg(**cfg), r, u, pt32=gp[b])
            assert np.abs(gp[b] - res["pt"]).max() <= tol, (step, b)
            assert (int(out["n_accepted"][b]), int(out["next_token"][b])) == (res["n"], res["next"]), (step, b)
            n, pending[b] = res["n"], res["next"]
            ns.append(n)
            if n < K:
                dc[b].length = L + 1 + n; dpend[b] = [pending[b]]
            else:
                dpend[b] = [int(gx[b, -1]), pending[b]]
            st, sd = sess.kv.state(b), sess.kv_d.state(b)
            assert st["len"] == tc[b].length and st["pending"] == [pending[b]], (step, b)
            assert sd["len"] == dc[b].length and sd["pending"] == dpend[b], (step, b)
        mixed = mixed or (K in ns and any(n < K for n in ns))
    assert mixed                                          # one and two pending draft rows occurred in the same launch


def test_many_sequences_reserve_blocks_in_one_launch():
    """Eight sequences x two rows = 16 rows on the barrier-free kernel, whose reservation takes one lane per sequence:
    lengths chosen so that in the same launch some sequences need no new block, some one, and several at once; the
    block tables and the order of the free stack must follow the serial allocator model through every step."""
    from tests.parity import Pair, verify_parity_step
    wl = si.workload("mini")
    shape = si.model_shape(wl["target"])
    B, K, steps = 8, 1, 10
    lens = [15, 16, 17, 30, 31, 32, 47, 9]             # block size 16: boundaries are crossed at different steps, often together
    pair = Pair(wl["target"], wl["seeds"]["target"], 47 + steps * (K + 1) + 20, max_seqs=B, max_rows=2,
                n_blocks=B * 5 + 1, block_tokens=16)
    for b in range(B):
        pair.prefill(b, si.make_prefix(shape, 2, lens[b] - 2, 700 + b))
    pair.check_free_stack()
    rng = np.random.default_rng(11)
    cfg = dict(beta=0.3, temperature=1.0, top_k=0, greedy=False, seed=99)
    together = 0
    for s in range(steps):
        owned_before = [pair.alloc.owned[b] for b in range(B)]
        verify_parity_step(pair, cfg, K, s, rng, 2e-2, 2e-2, seqs=tuple(range(B)))
        assert pair.kv.last_forward_path() == 3
        for b in range(B):
            pair.check_state(b, 2e-2, layers=[shape["n_layers"] - 1])
        pair.check_free_stack()
        together = max(together, sum(pair.alloc.owned[b] != owned_before[b] for b in range(B)))
    assert together >= 2                                  # at least once several sequences changed their block count in one step


def test_batched_verify_beyond_one_row_tile_uses_matrix_core_attention():
    """Five ragged sequences x (K+1 = 5) rows = 25 rows: more than the persistent kernels take, so every operator is
    its own launch and attention runs as 256-key parts on the matrix cores.  Lengths put new positions on both sides
    of a part boundary (250 -> 256), in a second and third part, and inside the first chunk."""
    from tests.parity import Pair, verify_parity_step
    wl = si.workload("mini")
    shape = si.model_shape(wl["target"])
    B, K, steps = 5, 4, 3
    lens = [23, 250, 300, 515, 64]
    cap = max(lens) + steps * (K + 1) + 20
    pair = Pair(wl["target"], wl["seeds"]["target"], cap, max_seqs=B, max_rows=8, block_tokens=16)
    for b in range(B):
        pair.prefill(b, si.make_prefix(shape, 3, lens[b] - 3, 700 + b))
    rng = np.random.default_rng(6)
    cfg = dict(beta=0.2, temperature=1.0, top_k=0, greedy=False, seed=99)
    worst = 0.0
    for s in range(steps):
        res = verify_parity_step(pair, cfg, K, s, rng, 2e-2, 2e-2, seqs=tuple(range(B)))
        assert pair.kv.last_forward_path() == 1
        worst = max(worst, max(r["dlogits"] for r in res))
        for b in range(B):
            pair.check_state(b, 2e-2, layers=[shape["n_layers"] - 1])
        pair.check_free_stack()
    assert 0 < worst < 2e-2


@pytest.mark.parametrize("shape_name,gemm,attn", [("mini_bf16", "", ""), ("mini128_bf16", "", ""), ("mini_bf16", "narrow", ""),
                                                  ("mini128_bf16", "", "valu")])
def test_batched_verify_many_rows_kernels(shape_name, gemm, attn, monkeypatch):
    """Five ragged sequences x (K+1 = 8) rows = 40 rows: three row tiles, so the batched kernels run (matrix-core
    attention for head_dim 64 and 128, the LDS-shared gate/up GEMM with a ragged last row group), and the generic
    kernels they replace when switched off; all against the oracle."""
    from tests.parity import Pair, verify_parity_step
    for k, v in (("SSD_GEMM", gemm), ("SSD_ATTN", attn)):
        if v:
            monkeypatch.setenv(k, v)
        else:
            monkeypatch.delenv(k, raising=False)
    shape = si.model_shape(shape_name)
    B, K, steps = 5, 7, 2
    lens = [40, 250, 300, 515, 64]
    cap = max(lens) + steps * (K + 1) + 20
    pair = Pair(shape_name, 777, cap, max_seqs=B, max_rows=K + 1, block_tokens=16)
    for b in range(B):
        pair.prefill(b, si.make_prefix(shape, 3, lens[b] - 3, 710 + b))
    rng = np.random.default_rng(8)
    cfg = dict(beta=0.2, temperature=1.0, top_k=0, greedy=False, seed=11)
    worst = 0.0
    for s in range(steps):
        res = verify_parity_step(pair, cfg, K, s, rng, 2e-2, 2e-2, seqs=tuple(range(B)))
        assert pair.kv.last_forward_path() == 1
        worst = max(worst, max(r["dlogits"] for r in res))
        for b in range(B):
            pair.check_state(b, 2e-2, layers=[shape["n_layers"] - 1])
        pair.check_free_stack()
    assert 0 < worst < 2e-2


@pytest.mark.parametrize("shape_name,max_rows,n_tokens", [("mini_bf16", 256, 700), ("mini128_bf16", 256, 700),
                                                          ("mini_bf16", 400, 777), ("mini128_bf16", 300, 777),
                                                          ("mini_bf16", 1024, 1100), ("mini128_bf16", 1024, 1100)])
def test_prefill_in_large_chunks_then_verify(shape_name, max_rows, n_tokens):
    """Prefill in chunks of 256 rows (700 tokens), of 400 and 300 rows (777 tokens: launches whose last row tile is
    ragged, 400 + 376 and 300 + 300 + 176 rows) and of 1024 rows (1100 tokens: one launch of 1024 rows, the most the
    library takes, and a ragged one of 75) - many row tiles per sequence: groups of tiles per attention workgroup, causal
    skipping of tiles that do not reach a part, the GEMM kernels for 256 rows and more at each of their tile heights -
    cache contents against the oracle's, then two verifications on top of it."""
    from tests.parity import Pair, verify_parity_step
    shape = si.model_shape(shape_name)
    K = 4
    pair = Pair(shape_name, 778, n_tokens + 100, max_seqs=1, max_rows=max_rows, block_tokens=16)
    pair.prefill(0, si.make_prefix(shape, 50, n_tokens - 50, 720))
    assert pair.kv.last_forward_path() == 1
    pair.check_state(0, 2e-2)
    pair.check_free_stack()
    rng = np.random.default_rng(9)
    cfg = dict(beta=0.2, temperature=1.0, top_k=0, greedy=False, seed=12)
    for s in range(2):
        verify_parity_step(pair, cfg, K, s, rng, 2e-2, 2e-2)
        pair.check_state(0, 2e-2, layers=[shape["n_layers"] - 1])


def test_rollback_and_reverify():
    """After a verification that rejected drafts, positions below the new length are untouched, stale positions
    are overwritten by the next call, and an explicit rollback frees whole blocks in the documented order."""
    import paper_2505_15380_amd as ssd
    from tests.parity import Pair, verify_parity_step
    pair = Pair("tiny", 100, 200, max_seqs=1, max_rows=16, n_blocks=13, block_tokens=16)
    shape = pair.shape
    pair.prefill(0, si.make_prefix(shape, 0, 60, 1))
    rng = np.random.default_rng(2)
    cfg = dict(beta=0.0, temperature=0.2, top_k=0, greedy=False, seed=9)       # sharp: mostly rejections
    for s in range(4):
        verify_parity_step(pair, cfg, 6, s, rng, 1e-5, 1e-5)
        pair.check_state(0, 1e-5)
    L = pair.ocache[0].length
    k_before, _ = pair.kv.gather(0, 1, 40)
    ssd.ssd_kv_rollback(pair.kv, 0, 20, 17)
    pair.ocache[0].length = 20; pair.pending[0] = 17; pair.alloc.set_length(0, 20)
    pair.check_state(0, 1e-5)
    pair.check_free_stack()
    k_after, _ = pair.kv.gather(0, 1, 20)
    assert (k_after == k_before[:20]).all()
    for s in range(4, 7):
        verify_parity_step(pair, cfg, 6, s, rng, 1e-5, 1e-5)
        pair.check_state(0, 1e-5)
        pair.check_free_stack()
    with pytest.raises(ssd.SSDError):
        ssd.ssd_kv_rollback(pair.kv, 0, L + 100, 0)


def test_errors_are_reported_not_faulted():
    import paper_2505_15380_amd as ssd
    from tests.parity import Pair
    pair = Pair("tiny", 100, 64, max_seqs=1, max_rows=8, n_blocks=3, block_tokens=16)
    shape = pair.shape
    pair.prefill(0, si.make_prefix(shape, 0, 40, 1))            # 39 cached positions -> 3 blocks
    V = shape["vocab"]
    x = torch.zeros((1, 7), dtype=torch.int32, device="cuda")
    pd = torch.full((1, 7, V), 1.0 / V, dtype=torch.float32, device="cuda")
    cfg = ssd.sample_config()
    with pytest.raises(ssd.SSDError) as e:                      # 39 + 8 rows need 3 blocks: fits; 39+8=47 <= 48
        ssd.ssd_verify(pair.gmodel, pair.kv, 1, x, pd, 7, cfg, 0, prefix_len=[38])
    assert e.value.code == -1                                   # wrong prefix_len
    ssd.ssd_verify(pair.gmodel, pair.kv, 1, x, pd, 7, cfg, 0, prefix_len=[39])
    with pytest.raises(ssd.SSDError) as e:                      # pool (3 blocks = 48 positions) cannot take 8 more
        for s in range(1, 4):
            ssd.ssd_verify(pair.gmodel, pair.kv, 1, x, pd, 7, cfg, s)
    assert e.value.code == -2
    free, err = pair.kv.free_stack()
    assert err == 0                                             # refused on the host, the device never overflowed
    with pytest.raises(ssd.SSDError):
        ssd.ssd_verify(pair.gmodel, pair.kv, 1, torch.zeros((1, 9), dtype=torch.int32, device="cuda"),
                       torch.full((1, 9, V), 1.0 / V, dtype=torch.float32, device="cuda"), 9, cfg, 0)          # K + 1 > max_rows
    with pytest.raises(ssd.SSDError):
        ssd.ssd_verify(pair.gmodel, pair.kv, 2, torch.zeros((2, 7), dtype=torch.int32, device="cuda"),
                       torch.full((2, 7, V), 1.0 / V, dtype=torch.float32, device="cuda"), 7, cfg, 0)          # n_seqs > max_seqs
    with pytest.raises(ssd.SSDError):                           # more than 1024 rows per forward
        ssd.KVCache(pair.gmodel, 65, 16, 80, 16, 4, 1)


@pytest.mark.parametrize("workload,K,cycles", [("mini", 3, 80), ("tiny", 2, 0)])
def test_captured_cycle_replays_like_the_eager_cycle(workload, K, cycles):
    """One SSD cycle captured as a graph (ssd_cycle_create) and replayed: every replay must leave what the same cycle
    enqueued call by call leaves on a second, identical session - draft tokens, draft rows, accepted count, emitted
    token, both caches' lengths - bit for bit, over enough cycles that the graph is captured again for longer prefixes
    (shapes are captured 256 positions ahead).  The eager cycle is the one the lockstep tests hold against the oracle."""
    import paper_2505_15380_amd as ssd
    side = torch.cuda.Stream()                             # HIP cannot capture the default stream
    if cycles == 0:                                        # fp32 storage runs one launch per operator: no capture
        sess, _ = make_session(workload, K, beta=0.2, steps=4)
        torch.cuda.synchronize()
        with pytest.raises(ssd.SSDError) as e:
            sess.graph_cycle()
        assert e.value.code == -4
        return
    a, _ = make_session(workload, K, beta=0.3, steps=cycles + 2, n_prefix=200)
    b, _ = make_session(workload, K, beta=0.3, steps=cycles + 2, n_prefix=200)
    a.cfg = b.cfg = ssd.sample_config(beta=0.3, seed=77)
    a.dcfg = b.dcfg = ssd.sample_config(seed=77)           # one seed for both models: the slots keep them apart
    torch.cuda.synchronize()
    g = a.graph_cycle(first_step=5)
    with pytest.raises(ssd.SSDError):
        g.launch()                                         # on the default stream: refused
    ns = []
    with torch.cuda.stream(side):
        for c in range(cycles):
            g.launch()
            b.cycle(5 + c)
            side.synchronize()
            assert torch.equal(a.x, b.x), c
            assert torch.equal(a.pd, b.pd), c
            assert int(a.n_acc[0]) == int(b.n_acc[0]) and int(a.next[0]) == int(b.next[0]), c
            ns.append(int(a.n_acc[0]))
            if c % 16 == 0:                                # eager work on the captured caches between replays
                sa, sb = a.kv.state(0), b.kv.state(0)
                assert sa["len"] == sb["len"] and sa["pending"] == sb["pending"]
                da, db = a.kv_d.state(0), b.kv_d.state(0)
                assert da["len"] == db["len"] and da["pending"] == db["pending"]
        assert g.captures() >= 2 and len(set(ns)) > 1
        assert a.kv.state(0)["table"] == b.kv.state(0)["table"]
        assert a.kv.free_stack() == b.kv.free_stack()
    torch.cuda.synchronize()


@pytest.mark.parametrize("B", [64, 128])
def test_verify_of_many_sequences_against_the_oracle(B):
    """64 or 128 ragged sequences x (K+1 = 8) rows = 512 or 1024 rows (the most one verification takes) on the small bf16 shape: every
    sequence's logits, probabilities and decision against the oracle, block tables and free stack against the allocator
    model, two steps (the second after 64 different commits)."""
    from tests.parity import Pair, verify_parity_step
    shape = si.model_shape("mini_bf16")
    K, steps = 7, 2
    rng0 = np.random.default_rng(64)
    lens = [int(n) for n in rng0.integers(18, 140, size=B)]
    cap = max(lens) + steps * (K + 1) + 20
    pair = Pair("mini_bf16", 778, cap, max_seqs=B, max_rows=K + 1, block_tokens=16)
    for b in range(B):
        pair.prefill(b, si.make_prefix(shape, 3, lens[b] - 3, 1200 + b))
    rng = np.random.default_rng(9)
    cfg = dict(beta=0.2, temperature=1.0, top_k=0, greedy=False, seed=13)
    worst, ns = 0.0, []
    for s in range(steps):
        res = verify_parity_step(pair, cfg, K, s, rng, 2e-2, 2e-2, seqs=tuple(range(B)))
        assert pair.kv.last_forward_path() == 1
        worst = max(worst, max(r["dlogits"] for r in res))
        ns += [r["n"] for r in res]
        for b in (0, 17, B - 1):
            pair.check_state(b, 2e-2, layers=[shape["n_layers"] - 1])
        pair.check_free_stack()
    assert 0 < worst < 2e-2 and len(set(ns)) > 2
