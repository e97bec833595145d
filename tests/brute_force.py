"""Dense NumPy attention on UNPAGED, contiguous K/V: the second, independent
implementation the C oracle is pinned against on tiny inputs.

Deliberately different in every way that could hide a shared mistake:
the full score matrix is materialised, visibility is an explicit boolean mask
matrix, weights are exp(score) WITHOUT max-subtraction, heads are expanded by
np.repeat, and nothing is paged.
"""
import numpy as np


def dense_attention(q, k, v, prefix, scale):
    """q [N, Hq, D], k/v [L, Hkv, D] with L = prefix + N (float64) -> [N, Hq, D].

    Row i may look at key j iff j <= prefix + i.
    """
    q = np.asarray(q, np.float64)
    k = np.asarray(k, np.float64)
    v = np.asarray(v, np.float64)
    n, hq, d = q.shape
    l, hkv, _ = k.shape
    assert l == prefix + n and hq % hkv == 0
    g = hq // hkv
    kx = np.repeat(k, g, axis=1)            # head h <- kv head h // g
    vx = np.repeat(v, g, axis=1)
    scores = np.einsum("ihd,jhd->hij", q, kx) * scale
    visible = np.zeros((n, l), dtype=bool)
    for i in range(n):
        for j in range(l):
            visible[i, j] = j <= prefix + i
    w = np.where(visible[None], np.exp(scores), 0.0)
    w = w / w.sum(axis=2, keepdims=True)
    return np.einsum("hij,jhd->ihd", w, vx)
