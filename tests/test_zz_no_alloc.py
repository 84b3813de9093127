"""GPU test of ssd_verify_noalloc (the entry point for callers that cannot allocate): through the C ABI, against
ssd_verify on an identical cache, two calls in a row - the second with a smaller input - and the size limit."""
import numpy as np
import pytest
import torch

import synth_inputs as si

pytestmark = pytest.mark.gpu


def _caches(B, max_rows, lens, seed=640):
    import paper_2505_15380_amd as ssd
    shape = si.model_shape("mini_bf16")
    w = si.make_weights(shape, 150)
    max_pos = max(lens) + 3 * max_rows + 32
    model = ssd.Model(shape, ssd.upload_weights(shape, w), max_pos)
    mbps = -(-max_pos // 16)
    kvs = [ssd.KVCache(model, B, max_rows, B * mbps, 16, mbps, 1) for _ in range(2)]
    for kv in kvs:
        for b, n in enumerate(lens):
            ssd.ssd_prefill(model, kv, b, torch.from_numpy(si.make_prefix(shape, 2, n - 2, seed + b)).cuda())
    return shape, model, kvs


def _drafts(rng, B, K, V):
    pd = si.make_probs(rng, B * K, V, 2.0).reshape(B, K, V)
    x = np.stack([[int(rng.choice(V, p=pd[b, i].astype(np.float64) / pd[b, i].astype(np.float64).sum())) for i in range(K)]
                  for b in range(B)]).astype(np.int32)
    return torch.from_numpy(x).cuda(), torch.from_numpy(pd).cuda()


def _same_state(kv_a, kv_b, n_seqs):
    for b in range(n_seqs):
        assert kv_a.state(b) == kv_b.state(b)
    assert kv_a.free_stack() == kv_b.free_stack()
    assert torch.equal(kv_a.pool, kv_b.pool)               # same block ids on both sides: the pools agree bit for bit


def test_verify_noalloc_matches_verify_twice_and_refuses_oversize():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2505_15380_amd as ssd
    lens = [45, 130, 300]
    shape, model, (kv_a, kv_b) = _caches(3, 8, lens)
    V = shape["vocab"]
    rng = np.random.default_rng(21)
    cfg = ssd.sample_config(beta=0.3, temperature=1.0, seed=17)
    for step, (B, K) in enumerate([(3, 6), (1, 2)]):       # the second call is smaller than the first
        x, pd = _drafts(rng, B, K, V)
        ref = ssd.ssd_verify(model, kv_a, B, x, pd, K, cfg, step)
        n = torch.full((B,), -1, dtype=torch.int32, device="cuda")
        nxt = torch.full((B,), -1, dtype=torch.int32, device="cuda")
        ssd.ssd_verify_noalloc(model, kv_b, B, x, pd, K, cfg, step, n, nxt)
        torch.cuda.synchronize()
        assert torch.equal(n, ref["n_accepted"]) and torch.equal(nxt, ref["next_token"]), (step, n, ref["n_accepted"])
        assert kv_a.last_forward_path() == kv_b.last_forward_path()
        _same_state(kv_a, kv_b, 3)
    # an autoregressive step (K = 0) through both
    ref = ssd.ssd_verify(model, kv_a, 3, None, None, 0, cfg, 9)
    n = torch.zeros(3, dtype=torch.int32, device="cuda")
    nxt = torch.zeros(3, dtype=torch.int32, device="cuda")
    ssd.ssd_verify_noalloc(model, kv_b, 3, None, None, 0, cfg, 9, n, nxt)
    torch.cuda.synchronize()
    assert torch.equal(nxt, ref["next_token"])
    _same_state(kv_a, kv_b, 3)


def test_verify_noalloc_refuses_what_its_static_staging_cannot_hold():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2505_15380_amd as ssd
    B, K = 32, 8                                           # 32 x 9 rows x 1000 = 288000 floats > 2^18
    shape, model, (kv_a, kv_b) = _caches(B, K + 1, [20] * B)
    V = shape["vocab"]
    x = torch.zeros((B, K), dtype=torch.int32, device="cuda")
    pd = torch.full((B, K, V), 1.0 / V, dtype=torch.float32, device="cuda")
    n = torch.zeros(B, dtype=torch.int32, device="cuda")
    nxt = torch.zeros(B, dtype=torch.int32, device="cuda")
    before = kv_b.state(5)
    with pytest.raises(ssd.SSDError) as e:
        ssd.ssd_verify_noalloc(model, kv_b, B, x, pd, K, ssd.sample_config(seed=1), 0, n, nxt)
    assert e.value.code == -2 and "static staging" in str(e.value)
    assert kv_b.state(5) == before
    ssd.ssd_verify_noalloc(model, kv_b, 16, x[:16].contiguous(), pd[:16].contiguous(), K, ssd.sample_config(seed=1), 0, n, nxt)
    ref = ssd.ssd_verify(model, kv_a, 16, x[:16].contiguous(), pd[:16].contiguous(), K, ssd.sample_config(seed=1), 0)
    torch.cuda.synchronize()
    assert torch.equal(n[:16], ref["n_accepted"]) and torch.equal(nxt[:16], ref["next_token"])
