"""Plain reference of the graph-aware size model (test infrastructure: only tests may import it).

Frame of the paper's appendix A: |D_h| is a sum of independent per-vertex indicators.  The inclusion
probabilities come from the graph: with q_u = P(u in D_h) and r_u the chance that a given neighbor of u is
among u's picks at hop h, P(v not in D_{h+1}) = (1 - q_v) * prod over edges u -> v of (1 - q_u r_u).
Written with dense loops over a scipy CSR matrix in fp64; no blocking, no fixed point.
"""
import numpy as np
import scipy.sparse as sp


def graph_model(offsets, indices, fanouts, batch, with_replacement=False, seed_prob=None):
    off = np.asarray(offsets, dtype=np.int64)
    idx = np.asarray(indices, dtype=np.int64)
    n = len(off) - 1
    deg = np.diff(off).astype(np.float64)
    adj = sp.csr_matrix((np.ones(len(idx)), idx, off), shape=(n, n))
    q = np.full(n, batch / n) if seed_prob is None else np.clip(np.asarray(seed_prob, dtype=np.float64), 0.0, 1.0)
    mean, sigma = [float(batch)], [0.0]
    for F in fanouts:
        safe = np.maximum(deg, 1.0)
        if with_replacement:
            r = np.where(deg > 0, 1.0 - (1.0 - 1.0 / safe) ** F, 0.0)
        else:
            r = np.where(deg > 0, np.minimum(F, deg) / safe, 0.0)
        x = np.minimum(q * r, 1.0 - 1e-9)  # a certain hit would be log(0)
        stay_out = np.exp(-(adj.T @ (-np.log1p(-x))))
        q = 1.0 - (1.0 - q) * stay_out
        mean.append(float(q.sum()))
        sigma.append(float(np.sqrt((q * (1.0 - q)).sum())))
    return mean, sigma
