"""Decode attention over the compressed cache, fp64.  Test infrastructure only.

Eq. 2 of the paper (A = Softmax(Q K^T), O = A V; A is 1 x N, O is 1 x d) with
the 1/sqrt(d) factor of Eq. 6 (appendix A).  The rows are the cache's
original-precision rows followed by the dequantized rows; Sec. 2.4 / Eq. 3:
any joint permutation of the rows of K and V gives the same O, which is what
allows the two regions to be stored one after the other.
"""
import numpy as np


def softmax_attention(q, K, V, scale=None):
    """q [g][d], K [n][d], V [n][d] (any float type) -> O [g][d] fp64.

    Plain definition: logits = scale * K q, p = softmax(logits), O = p^T V.
    The maximum logit is subtracted before exponentiation (no change in value).
    """
    q = np.asarray(q, np.float64)
    K = np.asarray(K, np.float64)
    V = np.asarray(V, np.float64)
    d = q.shape[-1]
    if scale is None or scale <= 0:
        scale = 1.0 / np.sqrt(float(d))
    logits = scale * (q @ K.T)                       # [g][n]
    logits = logits - logits.max(axis=-1, keepdims=True)
    p = np.exp(logits)
    p = p / p.sum(axis=-1, keepdims=True)
    return p @ V


def decode_attention(cache, q_heads, scale=None):
    """One decode step for one kv head: q_heads [g][d] are the query heads that
    share this kv head (grouped-query attention: query head h reads kv head
    h // (Hq/Hkv)).  Output [g][d] fp64, not rounded to T."""
    K, V = cache.rows_fp64()
    return softmax_attention(q_heads, K, V, scale)
