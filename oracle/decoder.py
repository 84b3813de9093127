"""fp64 decoder forward with a contiguous KV cache (test oracle; see oracle/__init__.py).

The paper names the network only as a 24-layer Transformer adapted from a 0.5B LM with 14 heads
(Sec. 3.1); the block below is the standard pre-norm decoder of that family: RMSNorm, rotary position
embedding on half-split pairs, grouped-query attention with 1/sqrt(head_dim) scaling, SwiGLU FFN,
untied output head.  The target's parallel verification (Eq. 4) is `forward_rows` called once with the
pending token followed by the K draft tokens: row j attends to every cached position and to rows <= j.
"""
import numpy as np


class Model:
    """Weights widened to fp64 (their stored fp32/bf16 values, exactly) plus the shape dictionary."""

    def __init__(self, shape, weights):
        self.shape = dict(shape)
        self.w = {k: (None if v is None else np.asarray(v, dtype=np.float64)) for k, v in weights.items()}


def round_to_bf16_storage(x):
    """Values as a bf16 cache would hold them: rounded to nearest even on the upper 16 bits of their fp32 form."""
    u = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).astype(np.float64)


class Cache:
    """Contiguous per-layer key/value store: k[l], v[l] are [capacity, n_kv_heads, head_dim] fp64;
    positions 0..length-1 are valid.  The definition keeps keys and values exact (store=None).  store="bf16"
    models the storage format of the bf16 configurations instead: every key/value is rounded to bf16 when it is
    written, everything else stays fp64.  Tests use it to separate what the cache format costs (a property of the
    configuration) from what the arithmetic of an implementation costs."""

    def __init__(self, shape, capacity, store=None):
        nl, nkv, hd = shape["n_layers"], shape["n_kv_heads"], shape["head_dim"]
        self.k = np.zeros((nl, capacity, nkv, hd))
        self.v = np.zeros((nl, capacity, nkv, hd))
        self.length = 0
        self.store = store

    def copy(self):
        c = Cache.__new__(Cache)
        c.k, c.v, c.length, c.store = self.k.copy(), self.v.copy(), self.length, self.store
        return c


def rmsnorm(x, gain, eps):
    """x / sqrt(mean(x^2) + eps) * gain over the last axis."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * gain


def rope(x, positions, base):
    """Rotate the pairs (i, i + hd/2) of x[..., rows, heads, hd] by angle pos * base^(-2i/hd)."""
    hd = x.shape[-1]
    half = hd // 2
    inv_freq = base ** (-(np.arange(half, dtype=np.float64) * 2.0 / hd))
    ang = np.asarray(positions, dtype=np.float64)[:, None] * inv_freq[None, :]      # [rows, half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def silu(x):
    return x / (1.0 + np.exp(-x))


def attention_row(q, keys, values):
    """One query head against its keys: softmax(q.k / sqrt(hd)) weighted sum of values.
    q [hd], keys/values [n, hd]."""
    s = keys @ q / np.sqrt(q.shape[0])
    s = s - s.max()
    p = np.exp(s)
    return (p / p.sum()) @ values


def forward_rows(model, cache, tokens, with_head=True):
    """Run `tokens` (ids, length R) at positions cache.length .. cache.length+R-1.  Writes their keys and
    values into the cache at those positions (cache.length is NOT advanced: the caller commits).
    Returns logits [R, vocab] fp64 (None when with_head is False)."""
    sh, w = model.shape, model.w
    nq, nkv, hd = sh["n_q_heads"], sh["n_kv_heads"], sh["head_dim"]
    group = nq // nkv
    L = cache.length
    R = len(tokens)
    pos = np.arange(L, L + R)
    h = w["embed"][np.asarray(tokens, dtype=np.int64)].copy()                      # [R, d]
    for l in range(sh["n_layers"]):
        p = f"l{l}."
        x = rmsnorm(h, w[p + "ln1"], sh["rms_eps"])
        qkv = x @ w[p + "wqkv"].T
        if w[p + "bqkv"] is not None:
            qkv = qkv + w[p + "bqkv"]
        q = qkv[:, : nq * hd].reshape(R, nq, hd)
        k = qkv[:, nq * hd: (nq + nkv) * hd].reshape(R, nkv, hd)
        v = qkv[:, (nq + nkv) * hd:].reshape(R, nkv, hd)
        q = rope(q, pos, sh["rope_base"])
        k = rope(k, pos, sh["rope_base"])
        if getattr(cache, "store", None) == "bf16":
            k, v = round_to_bf16_storage(k), round_to_bf16_storage(v)
        cache.k[l, L:L + R] = k
        cache.v[l, L:L + R] = v
        att = np.empty((R, nq, hd))
        for j in range(R):                       # row j sees positions 0 .. L+j
            n = L + j + 1
            for hq in range(nq):
                g = hq // group
                att[j, hq] = attention_row(q[j, hq], cache.k[l, :n, g], cache.v[l, :n, g])
        h = h + att.reshape(R, nq * hd) @ w[p + "wo"].T
        x = rmsnorm(h, w[p + "ln2"], sh["rms_eps"])
        h = h + (silu(x @ w[p + "wgate"].T) * (x @ w[p + "wup"].T)) @ w[p + "wdown"].T
    if not with_head:
        return None
    return rmsnorm(h, w["final_norm"], sh["rms_eps"]) @ w["head"].T


def prefill(model, cache, tokens, chunk=256):
    """Put the keys/values of `tokens` into the cache and advance its length."""
    for i in range(0, len(tokens), chunk):
        part = tokens[i:i + chunk]
        forward_rows(model, cache, part, with_head=False)
        cache.length += len(part)
