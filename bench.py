#!/usr/bin/env python3
"""Benchmark of the SSD hot path on one MI355X.

A step is one SSD cycle of Alg. 1 at batch 1 on the 0.5B-shaped workload: K=4 draft steps (Eq. 2-3), one
parallel verification of the K+1 rows (Eq. 4) with acceptance / resampling (Eq. 5-6) and the cache commit,
and the draft cache following the decision, replayed as one captured graph per cycle.  `value` is the number of
speech tokens the sequence grows by per second over whole cycles (per cycle: the n accepted draft tokens plus the
resampled or bonus token), inputs resident in HBM.  Extra keys report the accepted draft tokens alone, the same
cycles enqueued call by call, the verification alone (latency, fraction of HBM peak), the same GPU's plain
autoregressive decoding, the roofline of the dominant kernel, the batched configurations and the CPU oracle."""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def algorithmic_bytes(shape, K, L, n_seqs=1):
    """Bytes one verification must move: every weight matrix once, the cached keys/values of the prefix once,
    the K+1 new key/value rows, and the logits / probability rows (2K+1 rows of V fp32)."""
    es = 2 if shape["dtype"] == "bf16" else 4
    d, hd, nq, nkv, ffn, V = (shape[k] for k in ("d_model", "head_dim", "n_q_heads", "n_kv_heads", "d_ffn", "vocab"))
    per_layer = d * (nq + 2 * nkv) * hd + nq * hd * d + 3 * d * ffn
    weights = (shape["n_layers"] * per_layer + V * d) * es
    kv_tok = 2 * nkv * hd * es * shape["n_layers"]
    return weights + n_seqs * (L + K + 1) * kv_tok + n_seqs * (2 * K + 1) * V * 4, weights


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--beta", type=float, default=0.4)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-batched", action="store_true", help="skip the batch-16 and batch-8 verification and the prefill sub-records")
    ap.add_argument("--copy-calibration-mib", type=int, default=0,
                    help="after the benchmark, run a plain elementwise copy kernel over this many MiB (3 launches): the "
                         "known-size reference that scales the profiler's FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2505_15380_amd as ssd
    import synth_inputs as si

    wl = si.workload("half_b_k4")
    K = wl["K"]
    tshape, dshape = si.model_shape(wl["target"]), si.model_shape(wl["draft"])
    tw = si.make_weights(tshape, wl["seeds"]["target"])
    dw = si.make_weights(dshape, wl["seeds"]["draft"])
    prefix = si.make_prefix(tshape, *wl["prefix"], wl["seeds"]["prefix"])
    L0 = len(prefix) - 1
    steps, warmup = args.steps, args.warmup
    max_pos = len(prefix) + 2 * (steps + warmup + 8) * (K + 1) + 64
    cfg = ssd.sample_config(beta=args.beta, temperature=wl["temperature"], top_k=wl["top_k"], seed=wl["seeds"]["rng"])
    dcfg = ssd.sample_config(temperature=wl["temperature"], top_k=wl["top_k"], seed=wl["seeds"]["rng"] + 1)
    sess = ssd.SSDSession(tshape, tw, dshape, dw, 1, K, max_pos, cfg, dcfg)
    dev_prefix = torch.from_numpy(prefix).cuda()
    sess.prefill(0, dev_prefix)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()                      # every launch below goes to this stream (HIP cannot capture the default one)
    torch.cuda.set_stream(side)

    # ---- timed region: whole SSD cycles, one graph replay each ---------------------------------------
    # (a cycle grows the sequence by n + 1 tokens, so the tokens of a run are the growth of the cached length)
    graph = sess.graph_cycle(first_step=0)
    for s in range(warmup):
        graph.launch()
    torch.cuda.synchronize()
    len0 = sess.kv.state(0)["len"]
    t0 = time.perf_counter()
    for s in range(steps):
        graph.launch()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    emitted = sess.kv.state(0)["len"] - len0
    accepted = emitted - steps
    value = emitted / dt
    captures = graph.captures()

    # ---- the same cycles enqueued call by call (twelve launches from the host per cycle) -----------------
    n_log = torch.zeros((steps, 1), dtype=torch.int32, device="cuda")
    t_log = torch.zeros((steps, 1), dtype=torch.int32, device="cuda")
    base = warmup + steps
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(steps):
        sess.cycle(base + s, out=dict(n_accepted=n_log[s], next_token=t_log[s], probs=None, logits=None))
    torch.cuda.synchronize()
    dt_eager = time.perf_counter() - t0
    emitted_eager = int((n_log.cpu().numpy().ravel() + 1).sum())

    # ---- verification alone at the nominal prefix length, HIP events on the launch stream ------------
    stream = torch.cuda.current_stream()

    def time_loop(fn, iters):
        for i in range(5):
            fn(i)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record(stream)
        for i in range(iters):
            fn(i)
        e1.record(stream)
        e1.synchronize()
        return e0.elapsed_time(e1) / iters

    pend = int(prefix[-1])

    def verify_once(i):
        ssd.ssd_kv_rollback(sess.kv, 0, L0, pend)
        ssd.ssd_verify(sess.target, sess.kv, 1, sess.x, sess.pd, K, cfg, 10_000 + i,
                       out=dict(n_accepted=sess.n_acc, next_token=sess.next, probs=None, logits=None))

    def ar_once(i):
        ssd.ssd_kv_rollback(sess.kv, 0, L0, pend)
        sess.ar_step(20_000 + i)

    def draft_once(i):
        ssd.ssd_kv_rollback(sess.kv_d, 0, L0, pend)
        ssd.ssd_draft_step(sess.draft, sess.kv_d, 1, dcfg, 30_000 + i, 0, sess.x[:, 0], K, sess.pd[:, 0], K * sess.V)

    def rollback_only(i):
        ssd.ssd_kv_rollback(sess.kv, 0, L0, pend)

    iters = max(20, min(200, steps))
    rb_ms = time_loop(rollback_only, iters)
    verify_ms = time_loop(verify_once, iters) - rb_ms
    ar_ms = time_loop(ar_once, iters) - rb_ms
    draft_ms = time_loop(draft_once, iters) - rb_ms
    abytes, wbytes = algorithmic_bytes(tshape, K, L0)
    verify_gbs = abytes / (verify_ms * 1e-3) / 1e9

    # ---- dominant kernel: the persistent whole-forward kernel of the verification, events around each launch ----
    ssd.ssd_profile_begin("persistent")
    for i in range(20):
        verify_once(i)
    k_ms, k_n = ssd.ssd_profile_end()
    kernel_name = "k_forward_dataflow"          # the whole-forward kernel of the bf16 path (profile kind "persistent")
    fwd_bytes = abytes - (2 * K + 1) * tshape["vocab"] * 4 + (K + 1) * tshape["vocab"] * 4   # weights + KV + logits out
    if k_n == 0:                                    # shapes the persistent kernel does not cover: gate/up GEMM instead
        ssd.ssd_profile_begin("gate_up")
        for i in range(20):
            verify_once(i)
        k_ms, k_n = ssd.ssd_profile_end()
        kernel_name = "k_gemm_bf16<gate/up + SwiGLU>"
        fwd_bytes = 2 * tshape["d_model"] * tshape["d_ffn"] * 2
    gu_ms = k_ms / max(k_n, 1)
    gu_gbs = fwd_bytes / (gu_ms * 1e-3) / 1e9
    # HBM traffic per launch cannot be counted from inside this process: it is the figure of the committed counter
    # summary (two rocprofv3 --pmc runs of this very command), labelled as such
    traffic, traffic_src = None, None
    tname = "hbm_traffic_k_forward_dataflow_half_b_k4.txt"
    tpath = os.path.join(ROOT, "profiles", tname)
    if kernel_name == "k_forward_dataflow" and os.path.exists(tpath):
        collected = ""
        for line in open(tpath):
            if line.startswith("traffic_bytes_per_launch"):
                traffic = float(line.split()[1])
            if line.startswith("collected"):
                collected = line.split(None, 1)[1].strip()
        traffic_src = f"profiles/{tname} (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, collected {collected}; not measured by this run)"

    rec = {
        "metric": "accepted speech tokens/sec/GPU (batch 1, K=4)", "value": round(value, 1), "unit": "tokens/s",
        "metric_note": "tokens the sequence grows by per second: per cycle the n accepted draft tokens + the resampled or bonus "
                       "token (= emitted tokens); accepted draft tokens alone are in accepted_draft_tokens_per_s",
        "emitted_tokens_per_s": round(value, 1),
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": round(dt / steps * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "half_b_k4: 0.5B-shaped bf16 target (24 layers, d=896, 14q/2kv x64, FFN 4864, V=6564), "
                               "4-layer draft, batch 1, prefix 1024, K=4, T=1", "beta": args.beta,
                   "weights": "independent N(0,0.02) target and draft"},
        "accepted_draft_tokens_per_s": round(accepted / dt, 1),
        "launch": "one captured graph per cycle (ssd_cycle_launch)", "graph_captures": captures,
        "eager_cycle_ms": round(dt_eager / steps * 1e3, 4), "eager_emitted_tokens_per_s": round(emitted_eager / dt_eager, 1),
        # the same measured cycle time at other acceptance levels (tau = emitted tokens per cycle, 1 .. K+1): the
        # acceptance of unrelated random draft/target weights says nothing about a trained pair
        "tokens_per_s_if_tau": {str(t): round(t / (dt / steps), 1) for t in range(1, K + 2)},
        "mean_accepted_per_cycle": round(accepted / steps, 3),
        "emitted_per_cycle": round(emitted / steps, 3),
        "verify_us": round(verify_ms * 1e3, 1),
        "verify_algorithmic_GBps": round(verify_gbs, 1),
        "verify_frac_hbm_peak": round(verify_gbs / HBM_PEAK_GBS, 4),
        "draft_step_us": round(draft_ms * 1e3, 1),
        "ar_step_us": round(ar_ms * 1e3, 1),
        "ar_tokens_per_s": round(1e3 / ar_ms, 1),
        "speedup_vs_same_gpu_ar": round(value / (1e3 / ar_ms), 3),
        "roofline": {"bound": "hbm", "kernel": kernel_name, "algorithmic_bytes_per_launch": fwd_bytes, "achieved": round(gu_gbs, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(gu_gbs / HBM_PEAK_GBS, 4),
                     "traffic": traffic, "traffic_source": traffic_src, "launches_timed": k_n, "avg_us": round(gu_ms * 1e3, 2)},
    }

    if args.copy_calibration_mib > 0:               # reads N MiB and writes N MiB per launch, nothing else
        n = args.copy_calibration_mib * (1 << 20) // 4
        src = torch.ones(n, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        rec["copy_calibration_bytes_each_way"] = n * 4

    # ---- the batched configurations: one verification of 16 x 7 and of 8 x 9 rows --------------------------
    if not args.no_batched:
        from paper_2505_15380_amd import bench_batched
        del graph, sess
        torch.cuda.empty_cache()
        for key, name, w in (("batch16", "half_b_batch16", tw), ("batch8", "one_half_b_batch8", None)):
            r = bench_batched.measure(argparse.Namespace(workload=name, iters=10, cycles=0, beta=0.2), weights=w)
            rec[key] = {"workload": name, "rows": r["rows"], "verify_us": r["verify_us"], "forward_path": r["forward_path"],
                        "algorithmic_bytes": r["weight_bytes"] + r["kv_bytes"], "frac_hbm_peak": r["frac_of_hbm_peak"],
                        "flops": r["gemm_flops"] + r["attention_flops"], "frac_mfma_bf16_peak": r["frac_of_bf16_mfma_peak"],
                        "per_operator_us": {k: v["us_per_verify"] for k, v in r["per_operator"].items()}}
            torch.cuda.empty_cache()
        # ---- and the prompt prefill that precedes the cycles: 4096 tokens, 1024 rows per launch ------------------
        from paper_2505_15380_amd import bench_prefill
        r = bench_prefill.measure(argparse.Namespace(workload="half_b_k4", tokens=4096, rows=1024, iters=3), weights=tw)
        rec["prefill"] = {k: r[k] for k in ("tokens", "rows_per_launch", "prefill_ms", "tokens_per_s", "forward_path",
                                            "gemm_TFLOPs_between_events", "gemm_frac_of_bf16_mfma_peak")}
        rec["prefill"]["per_operator_us_per_launch"] = {k: v["us_per_launch"] for k, v in r["per_operator"].items()}
        torch.cuda.empty_cache()

    # ---- CPU oracle on a bounded sample of the same workload -------------------------------------------
    if not args.no_cpu_baseline:
        rec["cpu_baseline"] = cpu_baseline(tshape, tw, dshape, dw, prefix, K, args.beta, wl)
    print(json.dumps(rec))


def cpu_baseline(tshape, tw, dshape, dw, prefix, K, beta, wl):
    """The fp64 oracle as it stands: whole SSD cycles (K draft steps + verification) at prefix 1024.  The caches
    are filled with seeded random keys/values instead of an oracle prefill (timing does not depend on them)."""
    import numpy as np
    from oracle import decoder as OD
    from oracle import ssd as OS
    rng = np.random.default_rng(7)
    t, d = OD.Model(tshape, tw), OD.Model(dshape, dw)
    L = len(prefix) - 1
    cycles = 128
    tc, dc = OD.Cache(tshape, L + (cycles + 20) * (K + 1) + 8), OD.Cache(dshape, L + (cycles + 20) * (K + 1) + 8)
    for c in (tc, dc):
        c.k[:, :L] = rng.standard_normal(c.k[:, :L].shape) * 0.5
        c.v[:, :L] = rng.standard_normal(c.v[:, :L].shape) * 0.5
        c.length = L
    cfg = OS.sample_cfg(beta=beta, temperature=wl["temperature"], top_k=wl["top_k"], seed=wl["seeds"]["rng"])
    dcfg = OS.sample_cfg(temperature=wl["temperature"], top_k=wl["top_k"], seed=wl["seeds"]["rng"] + 1)
    OS.ssd_generate(t, d, tc.copy(), dc.copy(), int(prefix[-1]), K, cfg, dcfg, 1)      # warm-up cycle
    t0 = time.perf_counter()
    toks, ns = OS.ssd_generate(t, d, tc, dc, int(prefix[-1]), K, cfg, dcfg, 10 ** 9, max_cycles=cycles)
    dt = time.perf_counter() - t0
    emitted = sum(n + 1 for n in ns)
    one = None
    try:
        import threadpoolctl
        threads = max([p["num_threads"] for p in threadpoolctl.threadpool_info()] or [1])
        with threadpoolctl.threadpool_limits(limits=1):     # the same oracle on one thread, a shorter sample
            t1 = time.perf_counter()
            _, ns1 = OS.ssd_generate(t, d, tc, dc, int(prefix[-1]), K, cfg, dcfg, 10 ** 9, max_cycles=16)
            dt1 = time.perf_counter() - t1
        one = {"value": round(sum(n + 1 for n in ns1) / dt1, 3), "cycles": len(ns1), "seconds": round(dt1, 2)}
    except Exception:
        threads = os.cpu_count()
    return {"value": round(emitted / dt, 3), "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": f"{len(ns)} SSD cycles (K={K} draft steps + one verification each) at prefix {L}, fp64 numpy, "
                      f"caches filled with random keys/values", "seconds": round(dt, 2), "single_thread": one}


if __name__ == "__main__":
    main()
