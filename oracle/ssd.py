"""One SSD cycle and the generation loops of Alg. 1 on top of the fp64 decoder (test oracle)."""
import numpy as np
from .decoder import forward_rows
from .warp import warp_probs
from .accept import accept_canonical, sample_canonical
from .philox import uniform24


def sample_cfg(beta=0.0, temperature=1.0, top_k=0, greedy=False, seed=0):
    return dict(beta=beta, temperature=temperature, top_k=top_k, greedy=greedy, seed=seed)


DRAFT_SLOT0 = 16   # first slot of the draft's draws: past every slot a verification can use (K <= 15)


def verify_uniforms(seed, seq, step, K):
    """r_1..r_K (slots 0..K-1) and the sampling uniform (slot K) of one verify step."""
    return [uniform24(seed, seq, step, i) for i in range(K)], uniform24(seed, seq, step, K)


def draft_uniform(seed, seq, step, i):
    """The uniform that draws x_{i+1} ~ pd_{i+1} (Eq. 3).  Eq. 5 needs r_i independent of the draw of x_i
    (Alg. 1 draws r ~ U[0,1] afresh), so the draft's draws have slots of their own: a caller may give both
    models one seed."""
    return uniform24(seed, seq, step, DRAFT_SLOT0 + i)


def verify_step(model, cache, pending, x, pd, cfg, r, u, pt32=None):
    """Target verification (Eq. 4-6, Alg. 1 loop body after drafting).
    cache.length = L cached positions, `pending` is the last emitted token (position L, not yet cached).
    Returns dict(logits [K+1,V] f64, pt [K+1,V] f64, n, next, fallback); on return cache.length = L+1+n.
    `pt32`, when given, replaces the oracle's own probabilities in the decision (decision parity with
    externally computed fp32 probabilities)."""
    K = len(x)
    logits = forward_rows(model, cache, [int(pending)] + [int(t) for t in x])
    pt = warp_probs(logits, cfg["temperature"], cfg["top_k"], cfg["greedy"])
    use = pt.astype(np.float32) if pt32 is None else np.asarray(pt32, dtype=np.float32)
    n, nxt, fb = accept_canonical(use, np.asarray(pd, dtype=np.float32).reshape(K, -1) if K else
                                  np.zeros((0, use.shape[1]), np.float32), list(x), r, u, cfg["beta"])
    cache.length += 1 + n
    return dict(logits=logits, pt=pt, n=n, next=nxt, fallback=fb)


def draft_step(model, cache, pending_tokens, cfg, u):
    """One autoregressive draft step (Eq. 2-3): feed the 1 or 2 pending tokens, return
    (token drawn from the warped draft distribution, that distribution as fp32 row)."""
    logits = forward_rows(model, cache, [int(t) for t in pending_tokens])
    cache.length += len(pending_tokens)
    pd = warp_probs(logits[-1:], cfg["temperature"], cfg["top_k"], cfg["greedy"])[0].astype(np.float32)
    return sample_canonical(pd, u), pd


def ar_generate(model, cache, pending, cfg, n_tokens, seq=0, step0=0):
    """Plain autoregressive decoding with the same sampler: a verify step with K = 0 per token."""
    out = []
    for s in range(n_tokens):
        _, u = verify_uniforms(cfg["seed"], seq, step0 + s, 0)
        res = verify_step(model, cache, pending, [], np.zeros((0, model.shape["vocab"]), np.float32), cfg, [], u)
        pending = res["next"]
        out.append(pending)
    return out


def ssd_generate(target, draft, tcache, dcache, pending, K, cfg, dcfg, n_tokens, seq=0, max_cycles=None):
    """Alg. 1: repeat {draft K tokens, verify in parallel, accept / resample / bonus} until n_tokens are
    emitted (L_acc grows by n+1 per cycle; the last cycle's surplus is cut).  Both caches hold the same
    prefix on entry.  Returns (tokens, list of n_accepted per cycle)."""
    out, ns = [], []
    dpend = [pending]
    step = 0
    while len(out) < n_tokens and (max_cycles is None or step < max_cycles):
        xs, pds = [], []
        for i in range(K):
            tok, pd = draft_step(draft, dcache, dpend, dcfg, draft_uniform(dcfg["seed"], seq, step, i))
            xs.append(tok)
            pds.append(pd)
            dpend = [tok]
        r, u = verify_uniforms(cfg["seed"], seq, step, K)
        L = tcache.length
        res = verify_step(target, tcache, pending, xs, np.stack(pds) if K else None, cfg, r, u)
        n, pending = res["n"], res["next"]
        out += xs[:n] + [pending]
        ns.append(n)
        if K > 0 and n < K:
            dcache.length = L + 1 + n          # keep p, x_1..x_n; drop the rejected draft positions
            dpend = [pending]
        elif K > 0:
            dpend = [xs[-1], pending]          # x_K was sampled but never fed to the draft
        step += 1
    return out[:n_tokens], ns
