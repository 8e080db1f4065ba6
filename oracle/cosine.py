"""Oracle of the outer-gradient cosine similarity (TEST INFRASTRUCTURE ONLY).

Appendix, paragraph on the cosine similarity of the outer gradients: for one
set of parameters (a transformer layer, the embedding, a fragment, all
fragments but the embedding) the similarity between the outer gradients of
every pair of replicas.  Written out as the textbook definition:

    Delta_m   = g - float(w_m)             one fp32 subtraction, Algorithm 2's outer gradient
    G[a][b]   = sum_i Delta_a[i] * Delta_b[i]                 (Gram matrix, in fp64)
    cos[a][b] = G[a][b] / (sqrt(G[a][a]) * sqrt(G[b][b]))

Readings where the paper is silent: a replica whose outer gradient is entirely
zero has similarity 0 with everything (itself included); the single curve the
figures draw is taken to be the mean of cos[a][b] over the pairs a < b (0 when
there is only one replica); the similarity of a union of parameter sets comes
from the sum of their Gram matrices, which is the same definition applied to
the concatenated vectors.
"""
from __future__ import annotations

import numpy as np


def outer_grads(g: np.ndarray, w_bits) -> np.ndarray:
    """[M, n] fp32 outer gradients from the fp32 global copy and the replicas' bf16 bit patterns."""
    assert g.dtype == np.float32
    rows = []
    for w in w_bits:
        assert w.dtype == np.uint16 and w.shape == g.shape
        wf = (w.astype(np.uint32) << 16).view(np.float32)       # bf16 -> fp32 is exact
        rows.append(g - wf)                                      # one fp32 rounding
    return np.stack(rows) if rows else np.zeros((0, g.size), np.float32)


def gram(g: np.ndarray, w_bits) -> np.ndarray:
    """M x M Gram matrix of the outer gradients, accumulated in fp64."""
    d = outer_grads(g, w_bits).astype(np.float64)                # products of fp32 values are exact in fp64
    return d @ d.T


def cosine_from_gram(G: np.ndarray):
    """(cos[M][M], mean over the pairs a < b) from a Gram matrix."""
    M = G.shape[0]
    norm = np.sqrt(np.diag(G))
    cos = np.zeros((M, M), np.float64)
    for a in range(M):
        for b in range(M):
            den = norm[a] * norm[b]
            cos[a, b] = G[a, b] / den if den > 0 else 0.0
    pairs = [cos[a, b] for a in range(M) for b in range(a + 1, M)]
    mean = float(np.sum(np.array(pairs, np.float64)) / len(pairs)) if pairs else 0.0
    return cos, mean


def outer_grad_cosine(g: np.ndarray, w_bits):
    """(G, cos, mean) of one set of parameters."""
    G = gram(g, w_bits)
    cos, mean = cosine_from_gram(G)
    return G, cos, mean


def combine(grams):
    """(G, cos, mean) of the union of several parameter sets, given their Gram matrices."""
    G = np.zeros_like(np.asarray(grams[0], np.float64))
    for x in grams:
        G = G + np.asarray(x, np.float64)
    cos, mean = cosine_from_gram(G)
    return G, cos, mean
