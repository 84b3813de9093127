"""Logit warping and softmax (test oracle).  The paper states no sampling hyper-parameters; the
distributions q^s and p^d of Alg. 1 are taken to be the post-warp ones: temperature, then top-k
(ties at the k-th value broken by lower index, exactly k survive), then softmax.  Greedy mode is the
T -> 0 limit: a one-hot row at the arg-max (lowest index among equals)."""
import numpy as np


def warp_probs(logits, temperature=1.0, top_k=0, greedy=False):
    """logits [R, V] -> probabilities [R, V], same floating type as given (fp64 in the oracle)."""
    z = np.asarray(logits, dtype=np.float64)
    R, V = z.shape
    out = np.zeros((R, V))
    for r in range(R):
        row = z[r]
        if greedy:
            out[r, int(np.argmax(row))] = 1.0          # np.argmax returns the first maximum
            continue
        row = row / temperature
        keep = np.ones(V, dtype=bool)
        if 0 < top_k < V:
            order = sorted(range(V), key=lambda j: (-row[j], j))
            keep[:] = False
            keep[order[:top_k]] = True
        m = row[keep].max()
        e = np.where(keep, np.exp(row - m), 0.0)
        out[r] = e / e.sum()
    return out
