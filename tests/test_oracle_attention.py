"""Pins for oracle/attention.py (Eq. 2 with Eq. 6's 1/sqrt(d); Eq. 3 permutation invariance)."""
import numpy as np
import scipy.special

from oracle import attention
from oracle.cache import SliceCache
from paper_2503_19950_amd import inputs


def _rand(n, d, g=4, seed=0):
    rng = np.random.default_rng(seed)
    return rng.standard_normal((g, d)), rng.standard_normal((n, d)), rng.standard_normal((n, d))


def test_equals_library_softmax_attention():
    q, K, V = _rand(300, 64)
    want = scipy.special.softmax((q @ K.T) / 8.0, axis=-1) @ V      # 1/sqrt(64)
    assert np.abs(attention.softmax_attention(q, K, V) - want).max() < 1e-13
    want = scipy.special.softmax((q @ K.T) * 0.3, axis=-1) @ V
    assert np.abs(attention.softmax_attention(q, K, V, 0.3) - want).max() < 1e-13


def test_elementwise_definition_tiny():
    # written out term by term for one query, three tokens
    q = np.array([[1.0, 2.0]])
    K = np.array([[0.5, -1.0], [2.0, 0.0], [0.0, 1.0]])
    V = np.array([[1.0, 0.0], [0.0, 1.0], [2.0, 2.0]])
    s = np.array([0.5 - 2.0, 2.0, 2.0]) / np.sqrt(2.0)
    w = np.exp(s) / np.exp(s).sum()
    want = w[0] * V[0] + w[1] * V[1] + w[2] * V[2]
    assert np.allclose(attention.softmax_attention(q, K, V)[0], want, atol=1e-15)


def test_permutation_invariance():
    q, K, V = _rand(513, 128, seed=1)
    P = np.random.default_rng(2).permutation(513)
    a = attention.softmax_attention(q, K, V)
    b = attention.softmax_attention(q, K[P], V[P])
    assert np.abs(a - b).max() < 1e-12


def test_special_cases():
    q, K, V = _rand(50, 32, seed=3)
    assert np.allclose(attention.softmax_attention(q, K[:1], V[:1]), np.broadcast_to(V[0], (4, 32)))
    same = np.broadcast_to(K[0], K.shape)
    assert np.allclose(attention.softmax_attention(q, same, V), np.broadcast_to(V.mean(0), (4, 32)))
    # adding the same vector's projection to all logits: K + c*u with q.u = const shift -> no change
    a = attention.softmax_attention(q[:1], K, V)
    u = q[0] / (q[0] @ q[0])
    b = attention.softmax_attention(q[:1], K + 7.0 * u, V)
    assert np.abs(a - b).max() < 1e-12


def test_split_and_merge_equals_unsplit():
    q, K, V = _rand(400, 64, seed=4)
    sc = 1.0 / 8.0
    full = attention.softmax_attention(q, K, V)
    parts = []
    for lo, hi in ((0, 37), (37, 256), (256, 400)):
        s = sc * (q @ K[lo:hi].T)
        m = s.max(-1)
        p = np.exp(s - m[:, None])
        parts.append((m, p.sum(-1), p @ V[lo:hi]))
    M = np.max([p[0] for p in parts], 0)
    l = sum(np.exp(p[0] - M) * p[1] for p in parts)
    o = sum(np.exp(p[0] - M)[:, None] * p[2] for p in parts)
    assert np.abs(o / l[:, None] - full).max() < 1e-13


def test_all_fp_budget_is_exact_attention():
    """With a window so large that nothing is ever evicted the cache's decode
    attention is plain softmax attention over the original rows."""
    W, G, d = 64, 32, 128
    K, V = inputs.slice_kv(1, 0, 0, 0, 150)
    c = SliceCache(W, G, d, "f16")
    c.append_block(K, V)
    assert c.n_q == 0 and c.n_fp == 150
    q = inputs.queries(1)[0, :4]
    want = scipy.special.softmax((q.astype(np.float64) @ K.T.astype(np.float64)) / np.sqrt(128.0), -1) @ V
    assert np.abs(attention.decode_attention(c, q) - want).max() < 1e-13


def test_quantized_cache_attention_is_close_to_exact_and_order_free():
    W, G, d = 32, 32, 128
    K, V = inputs.slice_kv(1, 0, 1, 0, 512)
    c = SliceCache(W, G, d, "f16")
    c.append_block(K, V)
    assert c.n_fp + c.n_q == 512 and c.n_q > 0
    q = inputs.queries(1)[0, 4:8]
    out = attention.decode_attention(c, q)
    exact = attention.softmax_attention(q, K, V)
    assert 1e-4 < np.abs(out - exact).max() < 3.0            # 2-bit noise on N(0,1) rows is coarse
    Kr, Vr = c.rows_fp64()
    P = np.random.default_rng(5).permutation(Kr.shape[0])
    assert np.abs(attention.softmax_attention(q, Kr[P], Vr[P]) - out).max() < 1e-12
