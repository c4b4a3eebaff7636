"""Pins for oracle/cache.py: Algorithm 1 applied to rows, evicted rows quantized once."""
import numpy as np
import pytest

from oracle import selection
from oracle.cache import SliceCache
from paper_2503_19950_amd import inputs


@pytest.mark.parametrize("W,G,n", [(32, 32, 97), (32, 32, 96), (64, 32, 512), (64, 64, 777)])
def test_positions_follow_algorithm_1(W, G, n):
    d = 64
    rng = np.random.default_rng(0)
    K = inputs.to_T(rng.standard_normal((n, d)), "f16")
    V = inputs.to_T(rng.standard_normal((n, d)), "f16")
    a = SliceCache(W, G, d, "f16")
    a.append_block(K, V)
    b = SliceCache(W, G, d, "f16")
    for t in range(n):
        b.append(K[t], V[t])
    A, Qp = selection.stream_eager(n, W)
    for c in (a, b):
        assert c.pos_fp == A and c.pos_q == Qp
        assert c.n_fp + c.n_q == n and c.n_q == W * c.events
        # fp rows are the original rows at the kept positions, untouched
        assert np.array_equal(c.K_fp, K[A]) and np.array_equal(c.V_fp, V[A])
    for name in ("K_codes", "V_codes", "K_scale", "K_zero", "V_scale", "V_zero"):
        assert np.array_equal(getattr(a, name), getattr(b, name))


def test_every_token_is_kept_or_quantized_within_half_a_step():
    W, G, d, n = 32, 32, 128, 400
    K, V = inputs.slice_kv(3, 0, 2, 0, n)        # outlier channels and sink rows, bf16
    c = SliceCache(W, G, d, "bf16")
    c.append_block(K, V)
    Kh, Vh = c.rows_fp64()
    pos = np.array(c.pos_fp + c.pos_q)
    assert sorted(pos.tolist()) == list(range(n))
    nf = c.n_fp
    assert np.array_equal(Kh[:nf], K[pos[:nf]]) and np.array_equal(Vh[:nf], V[pos[:nf]])
    ks = c.K_scale.astype(np.float64)[np.arange(c.n_q) // G]            # [n_q][d]
    vs = c.V_scale.astype(np.float64)[:, np.arange(d) // G]
    # bf16 scales can round down by up to 2^-9 relative: the top bin then overshoots slightly
    assert (np.abs(Kh[nf:] - K[pos[nf:]]) <= ks * (0.5 + 3 * 2.0 ** -8)).all()
    assert (np.abs(Vh[nf:] - V[pos[nf:]]) <= vs * (0.5 + 3 * 2.0 ** -8)).all()


@pytest.mark.parametrize("cfg,n_fp,n_q,events", [(1, 128, 384, 6), (2, 256, 7936, 62),
                                                  (3, 512, 130560, 510), (4, 256, 3840, 30),
                                                  (5, 512, 32256, 168)])
def test_workload_states(cfg, n_fp, n_q, events):
    wl = inputs.WORKLOADS[cfg]
    W = wl["F"] // 2
    A, Qp = selection.stream_eager(wl["L"], W)
    assert (len(A), len(Qp), len(Qp) // W) == (n_fp, n_q, events)
    assert W % wl["G"] == 0


def test_compression_ratio_formula():
    """Eq. 4/5: 16 L / (2 (L - R) + 16 R) when scales and zero-points are not counted."""
    for cfg in (1, 2, 3):
        wl = inputs.WORKLOADS[cfg]
        A, Qp = selection.stream_eager(wl["L"], wl["F"] // 2)
        L, R = wl["L"], len(A)
        bits = 16 * len(A) + 2 * len(Qp)           # per channel, metadata ignored
        assert abs(16 * L / bits - 16 * L / (2 * (L - R) + 16 * R)) < 1e-12
