"""Seeded generators: weights, token prefixes, probability rows. No arithmetic of the method."""
import numpy as np


def round_to_bf16(x):
    """Round fp32 values to the nearest bf16 (ties to even) and return them widened back to fp32."""
    return (bf16_bits(x).astype(np.uint32) << 16).view(np.float32)


def bf16_bits(x):
    """The 16-bit patterns of the nearest-even bf16 roundings of an fp32 array."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> 16) & 1
    return ((u + 0x7FFF + lsb) >> 16).astype(np.uint16)


def weight_names(shape):
    """Canonical tensor names, in the order the C-ABI expects its pointer array."""
    names = ["embed", "final_norm", "head"]
    for l in range(shape["n_layers"]):
        names += [f"l{l}.{n}" for n in ("ln1", "wqkv", "bqkv", "wo", "ln2", "wgate", "wup", "wdown")]
    return names


def make_weights(shape, seed):
    """All tensors of one decoder, canonical layout: linear weights are [out_features, in_features]
    row-major; `wqkv` stacks query heads, then key heads, then value heads along the out axis.
    Matrices and biases ~ N(0, 0.02); norm gains ~ 1 + N(0, 0.1) so that a dropped gain shows.
    Values of matrices/embeddings are rounded to the model's storage type; gains and biases stay fp32.
    Returns a dict name -> fp32 ndarray."""
    rng = np.random.Generator(np.random.PCG64(seed))
    d, hd = shape["d_model"], shape["head_dim"]
    nq, nkv, ffn = shape["n_q_heads"], shape["n_kv_heads"], shape["d_ffn"]
    store = round_to_bf16 if shape["dtype"] == "bf16" else (lambda a: a)

    def mat(o, i):
        return store((rng.standard_normal((o, i), dtype=np.float32) * np.float32(0.02)))

    def gain(n):
        return (1.0 + 0.1 * rng.standard_normal(n, dtype=np.float32)).astype(np.float32)

    w = {"embed": mat(shape["n_embed"], d), "final_norm": gain(d), "head": mat(shape["vocab"], d)}
    for l in range(shape["n_layers"]):
        p = f"l{l}."
        w[p + "ln1"] = gain(d)
        w[p + "wqkv"] = mat((nq + 2 * nkv) * hd, d)
        if shape["qkv_bias"]:
            w[p + "bqkv"] = (rng.standard_normal((nq + 2 * nkv) * hd, dtype=np.float32) * np.float32(0.02))
        else:
            w[p + "bqkv"] = None
        w[p + "wo"] = mat(d, nq * hd)
        w[p + "ln2"] = gain(d)
        w[p + "wgate"] = mat(ffn, d)
        w[p + "wup"] = mat(ffn, d)
        w[p + "wdown"] = mat(d, ffn)
    return w


def correlated_draft_weights(target_shape, target_w, n_draft_layers, n_lower=2):
    """A draft that inherits the target's lower `n_lower` and upper `n_draft_layers - n_lower` layers,
    embeddings, final norm and head (the layer-inheritance construction of Sec. 2.3 / 3.1, without the
    fine-tuning, which needs data this repository does not have). Returns (draft_shape, weights)."""
    L = target_shape["n_layers"]
    keep = list(range(n_lower)) + list(range(L - (n_draft_layers - n_lower), L))
    shape = dict(target_shape)
    shape["n_layers"] = n_draft_layers
    w = {k: target_w[k] for k in ("embed", "final_norm", "head")}
    for new, old in enumerate(keep):
        for n in ("ln1", "wqkv", "bqkv", "wo", "ln2", "wgate", "wup", "wdown"):
            w[f"l{new}.{n}"] = target_w[f"l{old}.{n}"]
    return shape, w


def make_prefix(shape, n_text, n_speech, seed):
    """Token ids of one prompt: `n_text` text ids (embedding rows vocab .. n_embed-1) followed by
    `n_speech` speech ids (rows 0 .. vocab-1), the single concatenated sequence of Sec. 2.1."""
    rng = np.random.Generator(np.random.PCG64(seed))
    V, E = shape["vocab"], shape["n_embed"]
    text = rng.integers(V, E, size=n_text, dtype=np.int64) if (n_text and E > V) else \
        rng.integers(0, V, size=n_text, dtype=np.int64)
    speech = rng.integers(0, V, size=n_speech, dtype=np.int64)
    return np.concatenate([text, speech]).astype(np.int32)


def make_probs(rng, rows, V, alpha=0.5, zeros=0.0):
    """Random fp32 probability rows: Dirichlet(alpha) draws from `rng` (smaller alpha = peakier), optionally
    with a fraction of entries forced to exactly zero before renormalising. Row sums are 1 up to fp32
    rounding."""
    p = rng.gamma(alpha, size=(rows, V)) + 1e-300
    if zeros > 0:
        p = p * (rng.random((rows, V)) >= zeros)
        p[:, 0] += (p.sum(axis=1) == 0)
    p = p / p.sum(axis=1, keepdims=True)
    return p.astype(np.float32)
