"""Tolerance / draft-length sweep of whole SSD cycles on one GPU (the trade-offs of Sec. 4.3 with Table 3 - the
tolerance factor - and of Sec. 4.4 with Fig. 3 - the draft length - in throughput terms only: no audio is produced here, so the quality columns of the paper have no counterpart).

    python -m paper_2505_15380_amd.sweep [--cycles N] [--prefix P] [--head-scale S] [--top-k k] [--independent-draft]

Target = the 0.5B-shaped synthetic model; draft = the layer-inheritance construction of Sec. 2.3 applied to it
(lower 2 + upper 2 layers, shared embeddings and head, no fine-tuning: there is no data here).  With weights drawn
from N(0, 0.02) the output distributions are almost flat and every draft is accepted for a trivial reason, so the
shared head is scaled (default x5: logit standard deviation about 3) to give target and draft distinct, peaked
distributions.  Prints one JSON line per (beta, K) and a markdown table; `speedup` is emitted tokens/s over the same
GPU's plain autoregressive decoding of the same target.  `--independent-draft --head-scale 1 --prefix 4096 --top-k 25`
is the long-prefix configuration as its table states it (unrelated draft and target: with top-k on both the two kept
sets are almost disjoint, so about one token per cycle is emitted and the table shows cost, not speed-up)."""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--cycles", type=int, default=60)
    ap.add_argument("--prefix", type=int, default=1024)
    ap.add_argument("--head-scale", type=float, default=5.0)
    ap.add_argument("--betas", type=str, default="0,0.2,0.4")
    ap.add_argument("--ks", type=str, default="2,4,8,12")
    ap.add_argument("--top-k", type=int, default=0)
    ap.add_argument("--independent-draft", action="store_true", help="the workload's own 4-layer draft (independent weights)")
    args = ap.parse_args()

    import numpy as np
    import torch
    import paper_2505_15380_amd as ssd
    import synth_inputs as si

    wl = si.workload("half_b_k4")
    tshape = si.model_shape(wl["target"])
    tw = si.make_weights(tshape, wl["seeds"]["target"])
    tw["head"] = (tw["head"] * args.head_scale).astype(np.float32)
    if args.independent_draft:
        dshape = si.model_shape(wl["draft"])
        dw = si.make_weights(dshape, wl["seeds"]["draft"])
    else:
        dshape, dw = si.correlated_draft_weights(tshape, tw, 4, n_lower=2)
    prefix = si.make_prefix(tshape, args.prefix // 4, args.prefix - args.prefix // 4, wl["seeds"]["prefix"])
    L0, pend = len(prefix) - 1, int(prefix[-1])
    betas = [float(b) for b in args.betas.split(",")]
    Ks = [int(k) for k in args.ks.split(",")]
    cycles = args.cycles
    max_pos = len(prefix) + (cycles + 12) * (max(Ks) + 1) + 64
    dev_prefix = torch.from_numpy(prefix).cuda()

    rows = []
    ar_tps = None
    for K in Ks:
        for beta in betas:
            cfg = ssd.sample_config(beta=beta, temperature=1.0, top_k=args.top_k, seed=wl["seeds"]["rng"])
            dcfg = ssd.sample_config(temperature=1.0, top_k=args.top_k, seed=wl["seeds"]["rng"] + 1)
            sess = ssd.SSDSession(tshape, tw, dshape, dw, 1, K, max_pos, cfg, dcfg)
            sess.prefill(0, dev_prefix)
            n_log = torch.zeros((cycles + 10, 1), dtype=torch.int32, device="cuda")
            t_log = torch.zeros((cycles + 10, 1), dtype=torch.int32, device="cuda")
            for s in range(10):
                sess.cycle(s, out=dict(n_accepted=n_log[s], next_token=t_log[s], probs=None, logits=None))
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for s in range(10, 10 + cycles):
                sess.cycle(s, out=dict(n_accepted=n_log[s], next_token=t_log[s], probs=None, logits=None))
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            n_acc = n_log[10:].cpu().numpy().ravel()
            emitted = int((n_acc + 1).sum())
            if ar_tps is None:                       # the same target decoding one token per forward
                for s in range(10):
                    sess.ar_step(100_000 + s)
                torch.cuda.synchronize()
                t1 = time.perf_counter()
                for s in range(100):
                    sess.ar_step(200_000 + s)
                torch.cuda.synchronize()
                ar_tps = 100 / (time.perf_counter() - t1)
            # the verification alone at the nominal prefix (cache rolled back before each call, rollback subtracted)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            stream = torch.cuda.current_stream()

            def timed(fn, iters=30):
                torch.cuda.synchronize()
                e0.record(stream)
                for i in range(iters):
                    fn(i)
                e1.record(stream)
                e1.synchronize()
                return e0.elapsed_time(e1) / iters

            def rb(i):
                ssd.ssd_kv_rollback(sess.kv, 0, L0, pend)

            def ver(i):
                rb(i)
                ssd.ssd_verify(sess.target, sess.kv, 1, sess.x, sess.pd, K, cfg, 50_000 + i,
                               out=dict(n_accepted=sess.n_acc, next_token=sess.next, probs=None, logits=None))
            ver(0)
            verify_us = (timed(ver) - timed(rb)) * 1e3
            rec = {"beta": beta, "K": K, "verify_us": round(verify_us, 1), "mean_accepted": round(float(n_acc.mean()), 3),
                   "acceptance_rate": round(float(n_acc.mean()) / K, 3), "emitted_per_cycle": round(emitted / cycles, 3),
                   "cycle_ms": round(dt / cycles * 1e3, 3), "tokens_per_s": round(emitted / dt, 1),
                   "ar_tokens_per_s": round(ar_tps, 1), "speedup": round(emitted / dt / ar_tps, 3)}
            rows.append(rec)
            print(json.dumps(rec), flush=True)
            del sess
            torch.cuda.empty_cache()
    print("\n| K | beta | verify us | accepted / K | emitted per cycle | cycle ms | tokens/s | speedup vs AR |")
    print("|---|---|---|---|---|---|---|---|")
    for r in rows:
        print(f"| {r['K']} | {r['beta']} | {r['verify_us']:.0f} | {r['acceptance_rate']:.2f} | {r['emitted_per_cycle']:.2f} | {r['cycle_ms']:.2f} | "
              f"{r['tokens_per_s']:.0f} | {r['speedup']:.2f} |")


if __name__ == "__main__":
    main()
