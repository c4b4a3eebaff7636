"""Algorithm 1 of the paper (Sec. 2.5): which tokens stay at original precision.

Test infrastructure only (see oracle/__init__.py).

The list ``A`` holds absolute token positions in logical order.  Slices are
read as Python half-open, 0-based slices: ``A[0:2W:2]`` keeps the even logical
indices below 2W, ``A[2W:3W]`` keeps the newest window.  The tokens dropped
from ``A`` (odd logical indices below 2W) are not discarded: Fig. 6's caption
and Sec. 2.3 say they are quantized, so every routine here also returns them,
in the order they leave ``A``.
"""


def append_token(A, a_new, W):
    """One call of AppendToken(A, a*, W), Algorithm 1, as printed (lazy form):
    the length test happens before the new token is appended.

    Returns (A_updated, evicted) where ``evicted`` is the list of entries
    removed from A by this call (empty unless the list was full).
    """
    if len(A) < 3 * W:
        return A + [a_new], []
    evicted = A[1:2 * W:2]
    A = A[0:2 * W:2] + A[2 * W:3 * W]
    return A + [a_new], evicted


def stream_lazy(n, W):
    """State after n calls of Algorithm 1 on positions 0..n-1.

    Returns (A, Q): A = positions kept at original precision (logical order),
    Q = positions handed to the quantizer, in the order they were handed over.
    """
    A, Q = [], []
    for t in range(n):
        A, ev = append_token(A, t, W)
        Q += ev
    return A, Q


def compress_event(A, W):
    """The filtering step of Algorithm 1 on a full list (len(A) == 3W).

    Returns (kept, evicted).  Sec. 2.5: the first two windows (2W entries) are
    thinned to every second entry, the newest window is kept whole.
    """
    if len(A) != 3 * W:
        raise ValueError("compress_event needs a full list of 3W entries")
    return A[0:2 * W:2] + A[2 * W:3 * W], A[1:2 * W:2]


def stream_eager(n, W):
    """Same retention rule, but the filtering step runs as soon as an append
    makes the list 3W long (a reading: the workloads say compression is
    triggered when the window fills).  The sequence of retained sets is the one
    Algorithm 1 produces; only the moment of filtering moves by one append.
    """
    A, Q = [], []
    for t in range(n):
        A = A + [t]
        if len(A) == 3 * W:
            A, ev = compress_event(A, W)
            Q += ev
    return A, Q
