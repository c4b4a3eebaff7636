"""Pins for oracle/diagnostics.py: the synthetic analogue of the paper's Table 2 (Sec. 2.3;
L1 distance between the exact attention distribution and the one seen after quantizing
or evicting the tokens a selection rule does not keep)."""
import numpy as np
import scipy.special

from oracle import diagnostics as D
from oracle import selection
from oracle.cache import SliceCache
from paper_2503_19950_amd import inputs


def _slice(h, L, spiky=True, cfg=3):
    wl = dict(inputs.WORKLOADS[cfg])
    gh = wl["Hq"] // wl["Hkv"]
    if spiky:
        K, V, _ = inputs.slice_kv_spiky(cfg, 0, h, L, wl)
        q = inputs.queries_spiky(cfg, 0, wl)[0, h * gh:(h + 1) * gh]
    else:
        K, V = inputs.slice_kv(cfg, 0, h, 0, L, wl)
        q = inputs.queries(cfg, 0, wl)[0, h * gh:(h + 1) * gh]
    return wl, q, K, V


def test_distribution_is_library_softmax_and_masks():
    rng = np.random.default_rng(0)
    q, K = rng.standard_normal((3, 32)), rng.standard_normal((200, 32))
    want = scipy.special.softmax(q @ K.T / np.sqrt(32.0), axis=-1)
    assert np.abs(D.attention_distribution(q, K) - want).max() < 1e-14
    live = rng.random(200) < 0.3
    got = D.attention_distribution(q, K, live=live)
    assert (got[:, ~live] == 0).all()
    # restriction of the exact distribution to the live set, renormalised
    assert np.abs(got[:, live] - want[:, live] / want[:, live].sum(-1, keepdims=True)).max() < 1e-14


def test_eviction_error_closed_form():
    # evicting a set of tokens moves exactly their mass: L1 = 2 * (exact mass of the evicted tokens)
    wl, q, K, _ = _slice(1, 3000)
    W = 64
    A, _ = selection.stream_eager(3000, W)
    exact = D.attention_distribution(q, K)
    e = D.attention_errors(q, K, W, 64, wl["dtype"])
    keep = np.zeros(3000, bool)
    keep[A] = True
    assert np.allclose(e["log_evict"], 2.0 * exact[:, ~keep].sum(-1), atol=1e-12)
    assert np.allclose(e["recent_evict"], 2.0 * exact[:, :3000 - len(A)].sum(-1), atol=1e-12)


def test_log_quant_keys_are_the_cache_oracles_rows():
    # the diagnostic's keys, put back in storage order, are what the streaming cache oracle holds
    wl, q, K, V = _slice(2, 1500)
    W, G = 64, 32
    c = SliceCache(W, G, wl["d"], wl["dtype"])
    c.append_block(K, V)
    K_hat, A = D.log_quant_keys(K, W, G, wl["dtype"])
    assert A == c.pos_fp
    K_rows, _ = c.rows_fp64()
    assert np.array_equal(K_hat[c.pos_fp + c.pos_q], K_rows)


def test_no_error_when_everything_is_retained():
    wl, q, K, _ = _slice(0, 300)
    e = D.attention_errors(q, K, 128, 64, wl["dtype"])          # 300 < 3W: nothing leaves
    assert all((v == 0).all() for v in e.values())


def test_recent_quant_touches_only_old_tokens_and_respects_groups():
    wl, q, K, _ = _slice(3, 1000)
    K_hat = D.recent_quant_keys(K, 200, 64, wl["dtype"])
    assert np.array_equal(K_hat[800:], K[800:].astype(np.float64))
    # each run of 64 positions (the last one 32 long) has at most 4 levels per channel
    for lo in range(0, 800, 64):
        run = K_hat[lo:min(lo + 64, 800)]
        assert max(len(np.unique(run[:, c])) for c in range(run.shape[1])) <= 4
        assert np.abs(run - K[lo:lo + run.shape[0]]).max() <= 0.5 * (K[lo:lo + run.shape[0]].max(0) - K[lo:lo + run.shape[0]].min(0)).max() / 3 + 2e-2


def test_bounds_and_more_bits_help():
    wl, q, K, _ = _slice(4, 4096)
    W = wl["F"] // 2
    e2 = D.attention_errors(q, K, W, wl["G"], wl["dtype"], bits=2)
    e4 = D.attention_errors(q, K, W, wl["G"], wl["dtype"], bits=4)
    for e in (e2, e4):
        assert all(((v >= 0) & (v <= 2 + 1e-12)).all() for v in e.values())
    assert (e4["log_quant"] < e2["log_quant"]).all()
    assert np.array_equal(e4["log_evict"], e2["log_evict"])


def test_table2_ordering_on_the_spiky_generator():
    """Workload 3's generator with attention spikes at log-uniform distances, L = 8192:
    the order of the paper's Table 2 (log-quant < recent-quant < log-evict < recent-evict,
    eviction at least twice the error of quantization under the same selection)."""
    L, tot = 8192, {}
    for h in range(8):
        wl, q, K, _ = _slice(h, L)
        for k, v in D.attention_errors(q, K, wl["F"] // 2, wl["G"], wl["dtype"]).items():
            tot[k] = tot.get(k, 0.0) + float(v.sum())
    assert tot["log_quant"] < tot["recent_quant"] < tot["log_evict"] < tot["recent_evict"]
    assert tot["log_evict"] > 2 * tot["log_quant"] and tot["recent_evict"] > 2 * tot["recent_quant"]
