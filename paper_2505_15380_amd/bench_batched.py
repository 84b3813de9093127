"""Latency of ONE batched verification (Eq. 4-6 over B sequences x (K+1) rows) on the full-size batched workloads.

    python -m paper_2505_15380_amd.bench_batched [--workload half_b_batch16|one_half_b_batch8] [--iters N] [--cycles C]

The batched workloads have more rows than the persistent kernels take, so every operator is its own launch; this
prints one JSON line with the whole verification's latency (HIP events, the cache rolled back to the same state
before every call, rollback time subtracted), the time per operator kind from the library's own event pairs, and
the rates those imply.  `bench.py` stays the headline benchmark (batch 1); this is the second configuration's
measurement, and the command the batched rocprofv3 summary under profiles/ was taken with.  With --cycles C it also
runs C whole SSD cycles of the batch (K draft steps of the workload's draft model for all sequences, one batched
verification, the draft caches following the decisions) and adds the aggregate emitted tokens/s."""
import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="half_b_batch16")
    ap.add_argument("--iters", type=int, default=10)
    ap.add_argument("--cycles", type=int, default=0)
    ap.add_argument("--beta", type=float, default=0.2)
    args = ap.parse_args()
    print(json.dumps(measure(args)))


def measure(args, weights=None):
    """The record of one batched workload (args: workload, iters, cycles, beta).  `weights`: the target's tensors when the
    caller has them already."""
    import numpy as np
    import torch
    import paper_2505_15380_amd as ssd
    import synth_inputs as si

    wl = si.workload(args.workload)
    shape = si.model_shape(wl["target"])
    w = weights if weights is not None else si.make_weights(shape, wl["seeds"]["target"])
    B, K = wl["batch"], wl["K"]
    rng = np.random.default_rng(wl["seeds"]["prefix"])
    lo, hi = wl["prefix_range"]
    lens = [int(n) for n in rng.integers(lo, hi + 1, size=B)]                 # ragged prefixes, as the parity test draws them
    toks = [si.make_prefix(shape, n // 4, n - n // 4, wl["seeds"]["prefix"] + 1 + b) for b, n in enumerate(lens)]
    bt = 16
    max_pos = max(lens) + 4 * (K + 1) + 32
    n_blocks = sum(-(-(n + 4 * (K + 1)) // bt) for n in lens) + 4
    model = ssd.Model(shape, ssd.upload_weights(shape, w), max_pos)
    kv = ssd.KVCache(model, B, K + 1, n_blocks, bt, -(-max_pos // bt), 1)
    for b in range(B):
        ssd.ssd_prefill(model, kv, b, torch.from_numpy(toks[b]).cuda())
    V = shape["vocab"]
    drng = np.random.default_rng(wl["seeds"]["rng"])
    pd = si.make_probs(drng, B * K, V, 2.0).reshape(B, K, V)
    x = drng.integers(0, V, size=(B, K)).astype(np.int32)
    x, pd = torch.from_numpy(x).cuda(), torch.from_numpy(pd).cuda()
    cfg = ssd.sample_config(beta=0.2, temperature=wl["temperature"], top_k=wl["top_k"], seed=wl["seeds"]["rng"])
    n_acc = torch.zeros(B, dtype=torch.int32, device="cuda")
    nxt = torch.zeros(B, dtype=torch.int32, device="cuda")

    def rollback():
        for b in range(B):
            ssd.ssd_kv_rollback(kv, b, len(toks[b]) - 1, int(toks[b][-1]))

    def once(i):
        rollback()
        ssd.ssd_verify(model, kv, B, x, pd, K, cfg, i, out=dict(n_accepted=n_acc, next_token=nxt, probs=None, logits=None))

    for i in range(3):
        once(i)
    torch.cuda.synchronize()
    per_kind = {}
    for kind in ("qkv", "attention", "o", "gate_up", "down", "head"):
        ssd.ssd_profile_begin(kind)
        for i in range(args.iters):
            once(i)
        ms, n = ssd.ssd_profile_end()
        per_kind[kind] = {"us_per_verify": round(ms / args.iters * 1e3, 1), "launches": n // args.iters}
    stream = torch.cuda.current_stream()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed(fn):
        torch.cuda.synchronize()
        e0.record(stream)
        for i in range(args.iters):
            fn(i)
        e1.record(stream)
        e1.synchronize()
        return e0.elapsed_time(e1) / args.iters

    t_rb = timed(lambda i: rollback())
    t_ms = timed(once) - t_rb
    fwd_path = kv.last_forward_path()
    es = 2 if shape["dtype"] == "bf16" else 4
    d, hd, nq, nkv, ffn, L = (shape[k] for k in ("d_model", "head_dim", "n_q_heads", "n_kv_heads", "d_ffn", "n_layers"))
    rows = B * (K + 1)
    per_layer = d * (nq + 2 * nkv) * hd + nq * hd * d + 3 * d * ffn
    weight_bytes = (L * per_layer + V * d) * es
    kv_bytes = sum(lens) * 2 * nkv * hd * es * L
    gemm_flops = 2 * rows * (L * per_layer + V * d)
    attn_flops = sum(4 * (K + 1) * nq * hd * n for n in lens) * L
    cyc = None
    if args.cycles > 0:
        import time
        del kv, model
        torch.cuda.empty_cache()
        dshape = si.model_shape(wl["draft"])
        dw = si.make_weights(dshape, wl["seeds"]["draft"])
        C, warm = args.cycles, 4
        cap = max(lens) + (C + warm + 2) * (K + 1) + 32
        nb = sum(-(-(n + (C + warm + 2) * (K + 1)) // bt) for n in lens) + 4
        ccfg = ssd.sample_config(beta=args.beta, temperature=wl["temperature"], top_k=wl["top_k"], seed=wl["seeds"]["rng"])
        dcfg = ssd.sample_config(temperature=wl["temperature"], top_k=wl["top_k"], seed=wl["seeds"]["rng"] + 1)
        sess = ssd.SSDSession(shape, w, dshape, dw, B, K, cap, ccfg, dcfg, n_blocks=nb)
        for b in range(B):
            sess.prefill(b, torch.from_numpy(toks[b]).cuda())
        n_log = torch.zeros((warm + C, B), dtype=torch.int32, device="cuda")
        t_log = torch.zeros((warm + C, B), dtype=torch.int32, device="cuda")
        for c in range(warm):
            sess.cycle(c, out=dict(n_accepted=n_log[c], next_token=t_log[c], probs=None, logits=None))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for c in range(warm, warm + C):
            sess.cycle(c, out=dict(n_accepted=n_log[c], next_token=t_log[c], probs=None, logits=None))
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        n_acc = n_log[warm:].cpu().numpy()
        emitted = int((n_acc + 1).sum())
        cyc = {"cycles": C, "beta": args.beta, "cycle_ms": round(dt / C * 1e3, 3), "emitted_tokens_per_s": round(emitted / dt, 1),
               "mean_accepted_per_sequence_and_cycle": round(float(n_acc.mean()), 3),
               "accepted_min_max_in_one_cycle": [int(n_acc.min()), int(n_acc.max())],
               "draft_forward_path": sess.kv_d.last_forward_path(), "target_forward_path": sess.kv.last_forward_path()}
    return ({
        "workload": args.workload, "batch": B, "K": K, "rows": rows, "prefix_lengths": sorted(lens),
        "forward_path": fwd_path, "verify_us": round(t_ms * 1e3, 1), "per_operator": per_kind,
        "weight_bytes": weight_bytes, "kv_bytes": kv_bytes, "gemm_flops": gemm_flops, "attention_flops": attn_flops,
        "achieved_TFLOPs": round((gemm_flops + attn_flops) / (t_ms * 1e-3) / 1e12, 2),
        "frac_of_bf16_mfma_peak": round((gemm_flops + attn_flops) / (t_ms * 1e-3) / 2.5e15, 4),
        "achieved_GBps": round((weight_bytes + kv_bytes) / (t_ms * 1e-3) / 1e9, 1),
        "frac_of_hbm_peak": round((weight_bytes + kv_bytes) / (t_ms * 1e-3) / 8e12, 4),
        "verified_rows_per_s": round(rows / (t_ms * 1e-3), 1), "ssd_cycles": cyc,
    })


if __name__ == "__main__":
    main()
