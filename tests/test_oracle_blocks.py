"""Pins of the oracle's decoder blocks and whole forward against library routines and invariants.
CPU only."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import synth_inputs as si
from oracle import decoder as D
from oracle.warp import warp_probs

F64 = torch.float64


def test_rmsnorm_vs_torch():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((5, 96))
    g = 1 + 0.1 * rng.standard_normal(96)
    ref = F.rms_norm(torch.tensor(x), (96,), torch.tensor(g), eps=1e-6).numpy()
    np.testing.assert_allclose(D.rmsnorm(x, g, 1e-6), ref, rtol=0, atol=1e-13)
    # closed form: a constant row c normalises to sign(c) * gain (eps -> 0)
    np.testing.assert_allclose(D.rmsnorm(np.full((1, 8), -3.0), np.arange(8.0), 0.0), -np.arange(8.0)[None])


def test_silu_vs_torch():
    x = np.linspace(-20, 20, 101)
    np.testing.assert_allclose(D.silu(x), F.silu(torch.tensor(x)).numpy(), atol=1e-14)


def test_attention_row_vs_torch_sdpa():
    rng = np.random.default_rng(1)
    q, k, v = rng.standard_normal(16), rng.standard_normal((9, 16)), rng.standard_normal((9, 16))
    ref = F.scaled_dot_product_attention(torch.tensor(q)[None, None], torch.tensor(k)[None], torch.tensor(v)[None])
    np.testing.assert_allclose(D.attention_row(q, k, v), ref[0, 0].numpy(), atol=1e-13)


def test_rope_invariants():
    rng = np.random.default_rng(2)
    hd, base = 32, 1.0e4
    q = rng.standard_normal((1, 1, hd))
    k = rng.standard_normal((1, 1, hd))
    # position 0 is the identity; norms are preserved
    np.testing.assert_allclose(D.rope(q, [0], base), q, atol=0)
    np.testing.assert_allclose(np.linalg.norm(D.rope(q, [37], base)), np.linalg.norm(q), rtol=1e-13)
    # the score depends only on the position difference
    s1 = (D.rope(q, [5], base) * D.rope(k, [2], base)).sum()
    s2 = (D.rope(q, [105], base) * D.rope(k, [102], base)).sum()
    assert abs(s1 - s2) < 1e-12
    # complex form: pair (i, i+hd/2) is a complex number multiplied by exp(i * pos * base^(-2i/hd))
    z = q[0, 0, :hd // 2] + 1j * q[0, 0, hd // 2:]
    w = z * np.exp(1j * 11 * base ** (-np.arange(hd // 2) / (hd // 2)))
    got = D.rope(q, [11], base)[0, 0]
    np.testing.assert_allclose(got, np.concatenate([w.real, w.imag]), atol=1e-13)
    # slowest pair of a 64-wide head at base 1e6, position 1: angle = 1e6^(-62/64)
    x = np.zeros((1, 1, 64)); x[0, 0, 31] = 1.0
    got = D.rope(x, [1], 1.0e6)[0, 0]
    ang = 1.0e6 ** (-62 / 64)
    assert abs(got[31] - np.cos(ang)) < 1e-15 and abs(got[63] - np.sin(ang)) < 1e-15


def torch_full_sequence_logits(shape, w, tokens):
    """Independent formulation: the whole sequence at once, no cache, torch CPU fp64 library ops
    (F.embedding, F.rms_norm, F.linear, F.scaled_dot_product_attention(is_causal), F.silu), RoPE as a
    complex multiplication."""
    nq, nkv, hd = shape["n_q_heads"], shape["n_kv_heads"], shape["head_dim"]
    t = {k: (None if v is None else torch.tensor(np.asarray(v, dtype=np.float64))) for k, v in w.items()}
    S = len(tokens)
    h = F.embedding(torch.tensor(np.asarray(tokens, dtype=np.int64)), t["embed"])
    pos = torch.arange(S, dtype=F64)
    freqs = shape["rope_base"] ** (-torch.arange(hd // 2, dtype=torch.float64) / (hd // 2))
    rot = torch.polar(torch.ones(S, hd // 2, dtype=F64), pos[:, None] * freqs[None, :])       # [S, hd/2] complex

    def rope(x):                                                                    # x [S, H, hd]
        z = torch.complex(x[..., : hd // 2], x[..., hd // 2:]) * rot[:, None, :]
        return torch.cat([z.real, z.imag], dim=-1)

    for l in range(shape["n_layers"]):
        p = f"l{l}."
        x = F.rms_norm(h, (h.shape[-1],), t[p + "ln1"], eps=shape["rms_eps"])
        qkv = F.linear(x, t[p + "wqkv"], t[p + "bqkv"])
        q, k, v = qkv.split([nq * hd, nkv * hd, nkv * hd], dim=-1)
        q = rope(q.view(S, nq, hd)).transpose(0, 1)
        k = rope(k.view(S, nkv, hd)).transpose(0, 1).repeat_interleave(nq // nkv, dim=0)
        v = v.view(S, nkv, hd).transpose(0, 1).repeat_interleave(nq // nkv, dim=0)
        a = F.scaled_dot_product_attention(q[None], k[None], v[None], is_causal=True)[0]
        h = h + F.linear(a.transpose(0, 1).reshape(S, nq * hd), t[p + "wo"])
        x = F.rms_norm(h, (h.shape[-1],), t[p + "ln2"], eps=shape["rms_eps"])
        h = h + F.linear(F.silu(F.linear(x, t[p + "wgate"])) * F.linear(x, t[p + "wup"]), t[p + "wdown"])
    return F.linear(F.rms_norm(h, (h.shape[-1],), t["final_norm"], eps=shape["rms_eps"]), t["head"]).numpy()


@pytest.mark.parametrize("name,seed", [("tiny", 100), ("mini_bf16", 150)])
def test_cached_forward_equals_full_sequence_torch(name, seed):
    """Prefill in ragged chunks + one multi-row verify forward == full-sequence library forward
    (covers cache indexing, the causal mask inside the draft block, GQA head mapping, bias, RoPE positions)."""
    shape = si.model_shape(name)
    w = si.make_weights(shape, seed)
    toks = si.make_prefix(shape, 7, 30, seed + 2)
    ref = torch_full_sequence_logits(shape, w, toks)
    m = D.Model(shape, w)
    c = D.Cache(shape, 64)
    D.prefill(m, c, toks[:32], chunk=13)
    assert c.length == 32
    got = D.forward_rows(m, c, toks[32:])                 # 5 rows: "pending + 4 drafts"
    np.testing.assert_allclose(got, ref[32:], rtol=0, atol=1e-12)
    assert np.abs(ref[32:]).max() > 0.1                    # the comparison is not vacuous


def test_verify_rows_equal_autoregressive_rows():
    """Row i of the parallel pass equals the logits of feeding the same tokens one at a time (Eq. 4)."""
    shape = si.model_shape("tiny")
    m = D.Model(shape, si.make_weights(shape, 100))
    toks = si.make_prefix(shape, 0, 24, 5)
    c = D.Cache(shape, 64)
    D.prefill(m, c, toks[:19])
    par = D.forward_rows(m, c.copy(), toks[19:])
    for j in range(5):
        row = D.forward_rows(m, c, toks[19 + j: 20 + j])
        c.length += 1
        np.testing.assert_allclose(row[0], par[j], atol=1e-13)


def test_stale_rows_beyond_length_are_ignored():
    """After a rollback the rejected positions hold stale keys; the next forward must not see them."""
    shape = si.model_shape("tiny")
    m = D.Model(shape, si.make_weights(shape, 100))
    toks = si.make_prefix(shape, 0, 12, 6)
    c = D.Cache(shape, 32)
    D.prefill(m, c, toks[:8])
    clean = D.forward_rows(m, c.copy(), toks[8:10])
    D.forward_rows(m, c, [1, 2, 3, 4])                    # writes positions 8..11, not committed
    np.testing.assert_allclose(D.forward_rows(m, c, toks[8:10]), clean, atol=0)


# ------------------------------------------------------------------------------------- warp
def test_warp_vs_torch_softmax_topk():
    rng = np.random.default_rng(3)
    z = rng.standard_normal((4, 50)) * 3
    np.testing.assert_allclose(warp_probs(z, 0.8), F.softmax(torch.tensor(z) / 0.8, dim=-1).numpy(), atol=1e-15)
    p = warp_probs(z, 1.3, top_k=7)
    vals, idx = torch.topk(torch.tensor(z), 7, dim=-1)
    ref = torch.zeros(4, 50, dtype=F64).scatter(1, idx, F.softmax(vals / 1.3, dim=-1)).numpy()
    np.testing.assert_allclose(p, ref, atol=1e-15)
    assert ((p > 0).sum(axis=1) == 7).all()
    np.testing.assert_allclose(p.sum(axis=1), 1.0, atol=1e-14)


def test_warp_ties_and_greedy():
    z = np.array([[1.0, 3.0, 3.0, 2.0, 3.0, 0.0]])
    p = warp_probs(z, 1.0, top_k=2)
    assert (p[0] > 0).tolist() == [False, True, True, False, False, False]      # lower index wins the tie
    np.testing.assert_allclose(p[0, 1:3], 0.5)
    g = warp_probs(z, 1.0, greedy=True)
    assert g[0].tolist() == [0, 1, 0, 0, 0, 0]
    # top_k >= V and top_k = 0 both mean "no truncation"
    np.testing.assert_allclose(warp_probs(z, 1.0, top_k=6), warp_probs(z, 1.0, top_k=0))


def test_bf16_storage_option_only_rounds_keys_and_values():
    """store="bf16" rounds what is written to the cache (round to nearest even on the upper 16 bits) and nothing
    else: the rounding function agrees with torch's bfloat16 cast, cached values are exactly representable,
    the first row's logits are unchanged (its own key/value rounding aside, checked against the exact cache within
    the size of that rounding), and the exact cache is untouched by default."""
    import numpy as np
    import torch
    import synth_inputs as si
    from oracle import decoder as OD
    x = np.random.default_rng(0).standard_normal(4096) * np.array([1e-3, 1.0, 50.0, 1e4]).repeat(1024)
    want = torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(OD.round_to_bf16_storage(x), want)
    shape = si.model_shape("tiny")
    m = OD.Model(shape, si.make_weights(shape, 3))
    toks = si.make_prefix(shape, 0, 24, 1)
    ce, cb = OD.Cache(shape, 32), OD.Cache(shape, 32, store="bf16")
    le, lb = OD.forward_rows(m, ce, toks), OD.forward_rows(m, cb, toks)
    assert ce.store is None
    assert np.array_equal(cb.k, OD.round_to_bf16_storage(cb.k)) and np.array_equal(cb.v, OD.round_to_bf16_storage(cb.v))
    assert not np.array_equal(ce.k, cb.k)
    d = np.abs(le - lb).max()
    assert 0 < d < 5e-3                          # bf16 keys/values perturb the logits a little, and only a little
