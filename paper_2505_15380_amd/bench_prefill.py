"""Latency of a prompt prefill (the decoder forward over the prefix that fills the cache before the first SSD cycle).

    python -m paper_2505_15380_amd.bench_prefill [--workload half_b_k4] [--tokens 4096] [--rows 1024] [--iters 3]

Prefills `--tokens` positions of the workload's target shape in launches of up to `--rows` rows (every operator its
own launch: more rows than the persistent kernels take) and prints one JSON line: the whole prefill's time, tokens/s,
the time per operator kind from the library's own event pairs, and the GEMM rate those imply.  This is the command the
prefill's rocprofv3 summary under profiles/ was taken with; `bench.py` stays the headline benchmark."""
import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="half_b_k4")
    ap.add_argument("--tokens", type=int, default=4096)
    ap.add_argument("--rows", type=int, default=1024)
    ap.add_argument("--iters", type=int, default=3)
    print(json.dumps(measure(ap.parse_args())))


def measure(args, weights=None):
    """The record of one prefill (args: workload, tokens, rows, iters).  `weights`: the target's tensors when the caller has
    them already."""
    import torch
    import paper_2505_15380_amd as ssd
    import synth_inputs as si

    wl = si.workload(args.workload)
    shape = si.model_shape(wl["target"])
    w = weights if weights is not None else si.make_weights(shape, wl["seeds"]["target"])
    n = args.tokens + 1                                   # the last token stays pending: n - 1 positions are written
    toks = torch.from_numpy(si.make_prefix(shape, n // 4, n - n // 4, wl["seeds"]["prefix"])).cuda()
    bt = 16
    model = ssd.Model(shape, ssd.upload_weights(shape, w), n + 64)
    kv = ssd.KVCache(model, 1, args.rows, (n + 64) // bt + 2, bt, (n + 64) // bt + 1, 1)
    ssd.ssd_prefill(model, kv, 0, toks)                   # warm-up; a prefill of a sequence starts it over
    torch.cuda.synchronize()
    stream = torch.cuda.current_stream()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(args.iters):
        ssd.ssd_prefill(model, kv, 0, toks)
    e1.record(stream)
    e1.synchronize()
    ms = e0.elapsed_time(e1) / args.iters
    per_kind = {}
    for kind in ("qkv", "attention", "o", "gate_up", "down"):
        ssd.ssd_profile_begin(kind)
        ssd.ssd_prefill(model, kv, 0, toks)
        t, cnt = ssd.ssd_profile_end()
        per_kind[kind] = {"us_per_launch": round(t / cnt * 1e3, 1), "launches": cnt}
    d, hd, nq, nkv, ffn, L = (shape[k] for k in ("d_model", "head_dim", "n_q_heads", "n_kv_heads", "d_ffn", "n_layers"))
    gemm_flops = 2 * (n - 1) * L * (d * (nq + 2 * nkv) * hd + nq * hd * d + 3 * d * ffn)
    gemm_s = sum(per_kind[k]["us_per_launch"] * per_kind[k]["launches"] for k in ("qkv", "o", "gate_up", "down")) * 1e-6
    return {
        "workload": args.workload, "tokens": n - 1, "rows_per_launch": args.rows, "forward_path": kv.last_forward_path(),
        "prefill_ms": round(ms, 2), "tokens_per_s": round((n - 1) / (ms * 1e-3), 1), "per_operator": per_kind,
        "gemm_flops": gemm_flops, "gemm_TFLOPs_between_events": round(gemm_flops / gemm_s / 1e12, 1),
        "gemm_frac_of_bf16_mfma_peak": round(gemm_flops / gemm_s / 2.5e15, 4),
    }


if __name__ == "__main__":
    main()
