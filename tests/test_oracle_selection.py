"""Pins for oracle/selection.py (Algorithm 1, Sec. 2.5 of the paper)."""
import os

import pytest

from oracle import selection

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "alg1_traces.txt")


def _read_traces():
    rows = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        W, n, A, Q = [f.strip() for f in line.split(";")]
        rows.append((int(W), int(n), [int(x) for x in A.split()], [int(x) for x in Q.split()]))
    return rows


@pytest.mark.parametrize("W,n,A,Q", _read_traces())
def test_hand_traces(W, n, A, Q):
    a, q = selection.stream_lazy(n, W)
    assert a == A and q == Q


def _brute_force(n, W, eager):
    """Independent formulation: every token carries its current logical index.
    At a filtering step a token with index i < 2W survives iff i is even and
    moves to i/2; a token with i >= 2W moves to i - W."""
    idx = {}          # position -> logical index (only for tokens still kept)
    removed = []

    def event():
        gone = sorted((i, p) for p, i in idx.items() if i < 2 * W and i % 2 == 1)
        for _, p in gone:
            removed.append(p)
            del idx[p]
        for p in list(idx):
            i = idx[p]
            idx[p] = i // 2 if i < 2 * W else i - W

    for t in range(n):
        if not eager and len(idx) == 3 * W:
            event()
        idx[t] = len(idx)
        if eager and len(idx) == 3 * W:
            event()
    kept = [p for p, _ in sorted(idx.items(), key=lambda kv: kv[1])]
    return kept, removed


@pytest.mark.parametrize("W", [1, 2, 3, 4, 5, 6, 7, 8])
def test_brute_force_enumeration(W):
    for n in range(0, 40 * W + 1, max(1, W // 2)):
        assert selection.stream_lazy(n, W) == _brute_force(n, W, eager=False)
        assert selection.stream_eager(n, W) == _brute_force(n, W, eager=True)


@pytest.mark.parametrize("W", [1, 2, 3, 5, 42, 64, 128, 192])
def test_closed_forms(W):
    for n in list(range(0, 6 * W + 2)) + [9 * W, 12 * W - 1, 12 * W]:
        A, Q = selection.stream_lazy(n, W)
        want = n if n <= 3 * W else 2 * W + 1 + ((n - 1) % W)
        assert len(A) == want
        events = 0 if n <= 3 * W else (n - 2 * W - 1) // W
        assert len(Q) == W * events
        assert len(A) + len(Q) == n and sorted(A + Q) == list(range(n))
        assert A == sorted(A)
        assert A[-min(n, W):] == list(range(n - min(n, W), n))     # newest W always kept
        if n:
            assert A[0] == 0                                       # position 0 is never removed
        Ae, Qe = selection.stream_eager(n, W)
        assert len(Ae) == (n if n < 3 * W else 2 * W + (n % W))
        assert len(Ae) + len(Qe) == n


def test_length_stays_between_2W_and_3W():
    # Sec. 2.5: the retained length fluctuates between 2W and 3W
    W = 7
    for n in range(3 * W, 20 * W):
        A, _ = selection.stream_lazy(n, W)
        assert 2 * W <= len(A) <= 3 * W


def test_paper_window_for_R128():
    # Sec. 3.1 / 3.2.3: W = floor(R/3); R = 128 gives 3W = 126 original-precision tokens
    W = 128 // 3
    assert W == 42 and 3 * W == 126
    A, _ = selection.stream_lazy(3 * W, W)
    assert len(A) == 126
    for n in (1000, 1700):
        A, _ = selection.stream_lazy(n, W)
        assert len(A) <= 126


@pytest.mark.parametrize("W", [2, 3, 5, 8])
def test_eager_is_lazy_shifted_by_one_append(W):
    for n in range(0, 12 * W):
        Ae, Qe = selection.stream_eager(n, W)
        Al, Ql = selection.stream_lazy(n, W)
        if n < 3 * W or n % W != 0:
            assert (Ae, Qe) == (Al, Ql)
        else:
            Al1, Ql1 = selection.stream_lazy(n + 1, W)
            assert Ae == Al1[:-1] and Qe == Ql1


@pytest.mark.parametrize("m", [1, 2, 3, 6, 8])
def test_steady_state_is_log_sparse(m):
    """For W = 2^m, after enough events the kept set is position 0 plus blocks of
    W, W/2, ..., 1 positions with strides 1, 2, ..., 2^m going back in time
    (the log2-sparse picture of Sec. 2.2 / 2.5)."""
    W = 2 ** m
    for c in range(m + 3, m + 6):          # c = index (1-based) of the last event
        n = (c + 2) * W                    # eager: event c fires at n = (c+2) W
        A, _ = selection.stream_eager(n, W)
        want = {0}
        for i in range(m + 1):
            base = (c + 1 - i) * W
            want |= {base + o for o in range(0, W, 2 ** i)}
        assert set(A) == want and len(A) == 2 * W


def test_compress_event_rejects_partial_list():
    with pytest.raises(ValueError):
        selection.compress_event(list(range(5)), 2)
