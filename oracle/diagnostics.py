"""Attention-distribution error of four ways to shrink the cache (a synthetic
analogue of the paper's Table 2, Sec. 2.3).  Test infrastructure only.

For one query the exact attention distribution over L tokens (Eq. 2's A with
Eq. 6's 1/sqrt(d)) is compared with the distribution the same query sees when

  log-quant     the positions Algorithm 1 retains keep their keys, every other key is
                replaced by its dequantized 2-bit (or 4-bit) value, groups of G tokens
                per channel in the order of eviction (the paper's method);
  recent-quant  the newest n_fp positions keep their keys (n_fp = size of the set
                Algorithm 1 retains, i.e. the same memory), the older ones are
                quantized in groups of G consecutive positions (the window-based
                selection of the paper's comparison method, Sec. 2.2 / Fig. 3);
  log-evict     only the positions Algorithm 1 retains exist;
  recent-evict  only the newest n_fp positions exist.

The error is the L1 distance sum_n |A_exact[n] - A_method[n]| per head (an evicted
token has probability 0 in A_method), between 0 and 2.  The paper sums it over a
model's heads, layers and a dataset's samples, so its absolute numbers (432.5 ...
1612.6) are not comparable; what carries over is the ordering and the ratio between
quantization and eviction.
"""
import numpy as np

from . import quantizer
from . import selection


def attention_distribution(q, K, scale=None, live=None):
    """q [g][d], K [n][d] -> softmax(scale * q K^T) [g][n] fp64; positions where
    `live` is False get probability 0 and take no part in the normalisation."""
    q = np.asarray(q, np.float64)
    K = np.asarray(K, np.float64)
    if scale is None or scale <= 0:
        scale = 1.0 / np.sqrt(float(q.shape[-1]))
    logits = scale * (q @ K.T)
    if live is not None:
        logits = np.where(np.asarray(live, bool)[None, :], logits, -np.inf)
    logits = logits - logits.max(axis=-1, keepdims=True)
    p = np.exp(logits)
    return p / p.sum(axis=-1, keepdims=True)


def l1_error(p_exact, p_method):
    """Per head: sum over tokens of |difference|."""
    return np.abs(np.asarray(p_exact) - np.asarray(p_method)).sum(axis=-1)


def log_quant_keys(K, W, G, dtype, bits=2):
    """Keys as the compressed cache holds them after L appends, back in position
    order.  Returns (K_hat [L][d] fp64, retained positions)."""
    K = np.asarray(K, np.float32)
    A, Q = selection.stream_eager(K.shape[0], W)
    K_hat = K.astype(np.float64).copy()
    for e in range(len(Q) // W):                    # one filtering event at a time, eviction order
        ev = Q[e * W:(e + 1) * W]
        codes, s, z = quantizer.quantize_keys(K[ev], G, dtype, bits)
        K_hat[ev] = quantizer.dequantize_keys(codes, s, z, G)
    return K_hat, A


def recent_quant_keys(K, n_fp, G, dtype, bits=2):
    """The newest n_fp keys exact, the older ones quantized in runs of G positions
    (the last run shorter when G does not divide their number)."""
    K = np.asarray(K, np.float32)
    n_old = K.shape[0] - n_fp
    K_hat = K.astype(np.float64).copy()
    for lo in range(0, n_old, G):
        hi = min(lo + G, n_old)
        codes, s, z = quantizer.quantize_keys(K[lo:hi], hi - lo, dtype, bits)
        K_hat[lo:hi] = quantizer.dequantize_keys(codes, s, z, hi - lo)
    return K_hat


def attention_errors(q, K, W, G, dtype, bits=2, scale=None):
    """The four L1 errors for one kv head: q [g][d], K [L][d] -> dict name -> [g]."""
    L = np.asarray(K).shape[0]
    exact = attention_distribution(q, K, scale)
    K_log, A = log_quant_keys(K, W, G, dtype, bits)
    n_fp = len(A)
    log_live = np.zeros(L, bool)
    log_live[A] = True
    recent_live = np.arange(L) >= L - n_fp
    return {
        "log_quant": l1_error(exact, attention_distribution(q, K_log, scale)),
        "recent_quant": l1_error(exact, attention_distribution(q, recent_quant_keys(K, n_fp, G, dtype, bits), scale)),
        "log_evict": l1_error(exact, attention_distribution(q, K, scale, log_live)),
        "recent_evict": l1_error(exact, attention_distribution(q, K, scale, recent_live)),
    }
