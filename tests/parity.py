"""Teacher-forced parity of the HIP path against the CPU oracle (used by the GPU tests and the smoke check).

Protocol per verification step, same seeded inputs on both sides:
  P1  logits and probabilities of the K+1 rows: max-abs difference within tolerance;
  P2  decisions: the oracle's canonical acceptance fed the GPU's own fp32 probabilities, the same draft rows
      and the same Philox uniforms must give the same n_accepted and emitted token, bit for bit;
  P3  cache: length, pending token, block table and free stack equal the allocator model; key/value
      contents of committed positions within tolerance of the oracle's.
The oracle then advances with the (identical) decision, so both sides stay in lockstep."""
import numpy as np
import torch

import paper_2505_15380_amd as ssd
import synth_inputs as si
from oracle import decoder as OD
from oracle import ssd as OS
from oracle.kv_alloc import PagedAllocator


class Pair:
    """One model on both sides with one sequence slot set."""

    def __init__(self, shape_name, seed, max_positions, max_seqs=1, max_rows=16, n_blocks=None, block_tokens=16,
                 pending_cap=1, weights=None, shape=None, store=None):
        self.shape = shape or si.model_shape(shape_name)
        self.w = weights if weights is not None else si.make_weights(self.shape, seed)
        self.omodel = OD.Model(self.shape, self.w)
        self.gmodel = ssd.Model(self.shape, ssd.upload_weights(self.shape, self.w), max_positions)
        mbps = -(-max_positions // block_tokens)
        if n_blocks is None:
            n_blocks = max_seqs * mbps
        self.kv = ssd.KVCache(self.gmodel, max_seqs, max_rows, n_blocks, block_tokens, mbps, pending_cap)
        self.alloc = PagedAllocator(n_blocks, block_tokens, max_seqs, mbps)
        self.ocache = [OD.Cache(self.shape, max_positions, store=store) for _ in range(max_seqs)]   # store: see oracle.decoder.Cache
        self.pending = [None] * max_seqs
        self.max_rows = max_rows

    def prefill(self, seq, tokens):
        tokens = np.asarray(tokens, dtype=np.int32)
        ssd.ssd_prefill(self.gmodel, self.kv, seq, torch.from_numpy(tokens).cuda())
        self.ocache[seq].length = 0
        OD.prefill(self.omodel, self.ocache[seq], tokens[:-1])
        self.pending[seq] = int(tokens[-1])
        # allocator model: reset, then one reservation per chunk of max_rows rows
        self.alloc.set_length(seq, 0)
        n = len(tokens) - 1
        for i in range(0, n, self.max_rows):
            r = min(self.max_rows, n - i)
            self.alloc.reserve(seq, r)
            self.alloc.set_length(seq, self.alloc.length[seq] + r)

    def check_state(self, seq, atol_kv, layers=None):
        st = self.kv.state(seq)
        oc = self.ocache[seq]
        assert st["len"] == oc.length == self.alloc.length[seq], (st, oc.length, self.alloc.length[seq])
        assert st["n_owned"] == self.alloc.owned[seq]
        assert st["table"] == self.alloc.table[seq][:st["n_owned"]], "block table differs from the allocator model"
        if self.kv.pending_cap == 1:
            assert st["pending"] == [self.pending[seq]]
        worst = 0.0
        for l in (layers if layers is not None else range(self.shape["n_layers"])):
            k, v = self.kv.gather(seq, l, oc.length)
            worst = max(worst, np.abs(k - oc.k[l, :oc.length]).max(), np.abs(v - oc.v[l, :oc.length]).max())
        assert worst <= atol_kv, f"cache contents differ by {worst}"
        return worst

    def check_free_stack(self):
        free, err = self.kv.free_stack()
        assert err == 0
        assert free == self.alloc.free, "free stack differs from the allocator model"


def draw_drafts(rng, V, K, pt_hint=None, alpha=2.0):
    """Synthetic draft rows pd [K,V] (fp32) and tokens x_i ~ pd_i."""
    pd = si.make_probs(rng, K, V, alpha) if K else np.zeros((0, V), np.float32)
    x = [int(rng.choice(V, p=pd[i].astype(np.float64) / pd[i].astype(np.float64).sum())) for i in range(K)]
    return np.asarray(x, dtype=np.int32), pd


def verify_parity_step(pair, cfg_dict, K, step, rng, atol_logits, atol_probs, seqs=(0,), check=True):
    """One teacher-forced verification on sequences `seqs` (must be 0..B-1).  Returns per-seq results."""
    B = len(seqs)
    V = pair.shape["vocab"]
    xs, pds = [], []
    for b in seqs:
        x, pd = draw_drafts(rng, V, K)
        xs.append(x)
        pds.append(pd)
    cfg = ssd.sample_config(**cfg_dict)
    dt = torch.from_numpy(np.stack(xs)).cuda() if K else None
    dp = torch.from_numpy(np.stack(pds)).cuda() if K else None
    lens = [pair.ocache[b].length for b in seqs]
    out = ssd.ssd_verify(pair.gmodel, pair.kv, B, dt, dp, K, cfg, step, prefix_len=lens, want_probs=True,
                         want_logits=True)
    torch.cuda.synchronize()
    g_logits = out["logits"].cpu().numpy()
    g_probs = out["probs"].cpu().numpy()
    g_n = out["n_accepted"].cpu().numpy()
    g_next = out["next_token"].cpu().numpy()
    res = []
    for i, b in enumerate(seqs):                       # ascending, as the allocator contract says
        pair.alloc.reserve(b, K + 1)
    for i, b in enumerate(seqs):
        r, u = OS.verify_uniforms(cfg_dict.get("seed", 0), b, step, K)
        o = OS.verify_step(pair.omodel, pair.ocache[b], pair.pending[b], xs[i], pds[i], OS.sample_cfg(**cfg_dict), r, u,
                           pt32=g_probs[i])
        dl = float(np.abs(g_logits[i] - o["logits"]).max())
        if cfg_dict.get("top_k", 0) or cfg_dict.get("greedy", False):
            # the kept set / arg-max is decided in the kernel's own precision: compare the warp on its logits
            from oracle.warp import warp_probs
            ref = warp_probs(g_logits[i].astype(np.float64), cfg_dict.get("temperature", 1.0),
                             cfg_dict.get("top_k", 0), cfg_dict.get("greedy", False))
        else:
            ref = o["pt"]
        dp_ = float(np.abs(g_probs[i] - ref).max())
        if check:
            assert dl <= atol_logits, f"step {step} seq {b}: logits differ by {dl}"
            assert dp_ <= atol_probs, f"step {step} seq {b}: probabilities differ by {dp_}"
            assert (int(g_n[i]), int(g_next[i])) == (o["n"], o["next"]), \
                f"step {step} seq {b}: decision ({g_n[i]}, {g_next[i]}) != oracle ({o['n']}, {o['next']})"
        pair.pending[b] = o["next"]
        pair.alloc.set_length(b, pair.ocache[b].length)
        res.append(dict(n=o["n"], next=o["next"], dlogits=dl, dprobs=dp_, fallback=o["fallback"]))
    return res


def run_verify_parity(workload, steps, K, beta, atol_logits, atol_probs, temperature=1.0, top_k=0, greedy=False,
                      n_prefix=None, verbose=False, atol_kv=None, store=None):
    wl = si.workload(workload)
    shape = si.model_shape(wl["target"])
    n_text, n_speech = wl["prefix"]
    if n_prefix is not None:
        n_text, n_speech = 0, n_prefix
    toks = si.make_prefix(shape, n_text, n_speech, wl["seeds"]["prefix"])
    Ks = list(K) if isinstance(K, (list, tuple)) else [K] * steps          # a draft length per step
    assert len(Ks) == steps
    max_pos = len(toks) + sum(k + 1 for k in Ks) + 32
    pair = Pair(wl["target"], wl["seeds"]["target"], max_pos, max_rows=16, store=store)
    pair.prefill(0, toks)
    atol_kv = atol_kv if atol_kv is not None else atol_logits
    pair.check_state(0, atol_kv)
    pair.check_free_stack()
    rng = np.random.default_rng(wl["seeds"]["rng"])
    cfg = dict(beta=beta, temperature=temperature, top_k=top_k, greedy=greedy, seed=wl["seeds"]["rng"])
    worst_l = worst_p = 0.0
    ns = []
    for s in range(steps):
        (r,) = verify_parity_step(pair, cfg, Ks[s], s, rng, atol_logits, atol_probs)
        worst_l, worst_p = max(worst_l, r["dlogits"]), max(worst_p, r["dprobs"])
        ns.append(r["n"])
        pair.check_state(0, atol_kv, layers=[0, shape["n_layers"] - 1])
        pair.check_free_stack()
    if verbose:
        print(f"{workload}: {steps} steps K={Ks} beta={beta}: max|dlogits|={worst_l:.3g} max|dprobs|={worst_p:.3g} "
              f"accepted={ns}")
    return dict(dlogits=worst_l, dprobs=worst_p, accepted=ns, path=pair.kv.last_forward_path())
