"""Dense brute-force attention in numpy fp64, for tiny inputs only.

TEST INFRASTRUCTURE.  Independent of kvq_oracle.c's attention loops: it takes K and V
already gathered into dense arrays and evaluates softmax(q K^T * sm_scale) V with
whole-array numpy operations.  Follows the textbook definition of attention that the
paper's decode phase (Section 2) relies on.
"""
import numpy as np


def dense_attention(q, K, V, sm_scale):
    """q [R, D], K [n, D], V [n, D] float64 -> (out [R, D], weights [R, n])."""
    q = np.asarray(q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    z = (q @ K.T) * sm_scale
    z = z - z.max(axis=1, keepdims=True)
    w = np.exp(z)
    w = w / w.sum(axis=1, keepdims=True)
    return w @ V, w


def lse_merge(parts):
    """Merge per-chunk (max logit m [R], sum of exp l [R], unnormalised acc [R, D]) triples
    into the normalised output: the log-sum-exp rule a split evaluation has to use."""
    M = np.max(np.stack([m for m, _, _ in parts]), axis=0)
    num = sum(np.exp(m - M)[:, None] * acc for m, _, acc in parts)
    den = sum(np.exp(m - M) * l for m, l, _ in parts)
    return num / den[:, None]


def chunk_partial(q, K, V, sm_scale):
    """(m, l, acc) of one chunk of positions, in fp64."""
    z = (np.asarray(q, np.float64) @ np.asarray(K, np.float64).T) * sm_scale
    m = z.max(axis=1)
    p = np.exp(z - m[:, None])
    return m, p.sum(axis=1), p @ np.asarray(V, np.float64)
