"""Workload shapes. The paper's target is a 24-layer, 14-head decoder derived from a 0.5B LM with
an 8-layer draft (Sec. 3.1); the five workloads below are synthetic stand-ins that take that
shape (and a tiny fp32 one for exact parity work). Architecture details the paper leaves open
(norm type, RoPE base, bias, FFN width) are configuration fields.
"""
from copy import deepcopy

# dtype: "fp32" or "bf16" (storage type of weights and KV cache)
MODEL_SHAPES = {
    # tiny fp32 target / draft
    "tiny": dict(n_layers=2, d_model=128, n_q_heads=4, n_kv_heads=4, head_dim=32, d_ffn=512,
                 vocab=512, n_embed=512, dtype="fp32", qkv_bias=0, rope_base=1.0e4, rms_eps=1e-6),
    "tiny_draft": dict(n_layers=1, d_model=64, n_q_heads=2, n_kv_heads=2, head_dim=32, d_ffn=256,
                       vocab=512, n_embed=512, dtype="fp32", qkv_bias=0, rope_base=1.0e4, rms_eps=1e-6),
    # a small bf16 shape with grouped-query attention, bias and a ragged vocabulary: several MFMA tiles
    # and a ragged tail, yet the oracle finishes in well under a second
    "mini_bf16": dict(n_layers=2, d_model=256, n_q_heads=6, n_kv_heads=2, head_dim=64, d_ffn=768,
                      vocab=1000, n_embed=1100, dtype="bf16", qkv_bias=1, rope_base=1.0e6, rms_eps=1e-6),
    "mini_bf16_draft": dict(n_layers=1, d_model=256, n_q_heads=6, n_kv_heads=2, head_dim=64, d_ffn=768,
                            vocab=1000, n_embed=1100, dtype="bf16", qkv_bias=1, rope_base=1.0e6, rms_eps=1e-6),
    # the same with head_dim 128 (the 1.5B shape's head size) for the kernels that are specialised on it
    "mini128_bf16": dict(n_layers=2, d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=128, d_ffn=768,
                         vocab=1000, n_embed=1100, dtype="bf16", qkv_bias=1, rope_base=1.0e6, rms_eps=1e-6),
    # 0.5B-shaped target and its 4-layer draft
    "half_b": dict(n_layers=24, d_model=896, n_q_heads=14, n_kv_heads=2, head_dim=64, d_ffn=4864,
                   vocab=6564, n_embed=6564 + 4096, dtype="bf16", qkv_bias=1, rope_base=1.0e6, rms_eps=1e-6),
    "half_b_draft": dict(n_layers=4, d_model=896, n_q_heads=14, n_kv_heads=2, head_dim=64, d_ffn=4864,
                         vocab=6564, n_embed=6564 + 4096, dtype="bf16", qkv_bias=1, rope_base=1.0e6, rms_eps=1e-6),
    # 1.5B-shaped target and its 6-layer, narrower draft
    "one_half_b": dict(n_layers=28, d_model=1536, n_q_heads=12, n_kv_heads=2, head_dim=128, d_ffn=8960,
                       vocab=6564, n_embed=6564 + 4096, dtype="bf16", qkv_bias=1, rope_base=1.0e6, rms_eps=1e-6),
    "one_half_b_draft": dict(n_layers=6, d_model=896, n_q_heads=14, n_kv_heads=2, head_dim=64, d_ffn=4864,
                             vocab=6564, n_embed=6564 + 4096, dtype="bf16", qkv_bias=1, rope_base=1.0e6, rms_eps=1e-6),
}

# One entry per workload of the benchmark plan. `prefix` gives (n_text_ids, n_speech_ids) or a range
# (lo, hi) for ragged batches; seeds are frozen here.
WORKLOADS = {
    "tiny": dict(target="tiny", draft="tiny_draft", seeds=dict(target=100, draft=101, prefix=102, rng=1234),
                 batch=1, prefix=(0, 64), K=4, temperature=1.0, top_k=0, steps=16),
    "mini": dict(target="mini_bf16", draft="mini_bf16_draft", seeds=dict(target=150, draft=151, prefix=152, rng=1234),
                 batch=1, prefix=(20, 77), K=4, temperature=1.0, top_k=0, steps=8),
    "half_b_k4": dict(target="half_b", draft="half_b_draft", seeds=dict(target=200, draft=201, prefix=202, rng=1234),
                      batch=1, prefix=(256, 768), K=4, temperature=1.0, top_k=0, gen_tokens=200),
    "half_b_long": dict(target="half_b", draft="half_b_draft", seeds=dict(target=200, draft=201, prefix=302, rng=1234),
                        batch=1, prefix=(1024, 3072), K=(2, 4, 8, 12), temperature=1.0, top_k=25, gen_tokens=500),
    "half_b_batch16": dict(target="half_b", draft="half_b_draft", seeds=dict(target=200, draft=201, prefix=402, rng=1234),
                           batch=16, prefix_range=(256, 4096), K=6, temperature=1.0, top_k=0, steps=64,
                           block_tokens=16),
    # beyond the benchmark plan's five: 64 sequences x 8 rows = 512 rows in one verification
    "half_b_batch64": dict(target="half_b", draft="half_b_draft", seeds=dict(target=200, draft=201, prefix=602, rng=1234),
                           batch=64, prefix_range=(256, 2048), K=7, temperature=1.0, top_k=0, steps=16,
                           block_tokens=16),
    "one_half_b_batch8": dict(target="one_half_b", draft="one_half_b_draft",
                              seeds=dict(target=500, draft=501, prefix=502, rng=1234),
                              batch=8, prefix_range=(1024, 2048), K=8, temperature=0.8, top_k=0, steps=64,
                              block_tokens=16),
}


def model_shape(name):
    return deepcopy(MODEL_SHAPES[name])


def workload(name):
    return deepcopy(WORKLOADS[name])
