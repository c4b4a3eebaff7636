"""Group quantizer of the evicted tokens (2 bits; 4 bits as the paper's higher-
precision variant).  Test infrastructure only.

The paper fixes the bit width (INT2 in the main experiments, 4-bit in Sec. 3.2.1 /
Table 3), the group size G and the axis for keys ("Key-per-channel", Sec. 2.5; G and
INT2 in Sec. 3.1) but prints no formula.  The reading used everywhere in this
repository, for one group of values x_i held in the cache type T (fp16 or bf16) and
b bits, with n = 2^b - 1 steps (3 or 15):

    zero  z = min_i x_i                      (an element of T; a minimum or maximum
                                              equal to zero is taken as +0.0)
    scale s = round_to_T( (f32(max) - f32(min)) / n )   one fp32 subtract, one
            correctly rounded fp32 divide, one round-to-nearest-even to T
    code_i = sum_{k=0}^{n-1} [d_i >= (k + 0.5) s],  d_i = x_i - z in fp64
             (round-half-up of d_i / s clamped to 0..n, written without a
             division); all codes are 0 when s == 0
    dequantized value  z + code_i * s        (fp64)

The scale is the one place evaluated in fp32 on purpose: it is a stored
parameter that has to be reproducible bit for bit.

Grouping.  Keys: statistics run along the token axis, one group per channel
per run of G tokens in the order the tokens were evicted; the runs restart at
every filtering event (its W tokens are quantized together, Sec. 2.5), the last
run of an event shorter when G does not divide W (a reading: the paper's
W = floor(R/3) with G = 64, Sec. 3.1 / appendix D, needs one).  Values: statistics
run along the channel axis, one group per token per run of G channels, the last
run shorter when G does not divide d (a reading: the paper is silent on values).
"""
import numpy as np


def round_to_T(x, dtype):
    """Round fp32 values to the nearest value of T (ties to even); result is
    returned as fp32 holding exactly representable values."""
    x = np.asarray(x, dtype=np.float32)
    if dtype == "f16":
        return x.astype(np.float16).astype(np.float32)
    if dtype == "bf16":
        bits = x.view(np.uint32).astype(np.uint64)
        lsb = (bits >> np.uint64(16)) & np.uint64(1)
        bits = (bits + np.uint64(0x7FFF) + lsb) & np.uint64(0xFFFF0000)
        return bits.astype(np.uint32).view(np.float32).reshape(x.shape)
    raise ValueError("dtype must be 'f16' or 'bf16'")


def quantize_groups(x, dtype, bits=2):
    """Quantize every group along the LAST axis of x to `bits` bits.

    x : array [..., n] of values exactly representable in T.
    Returns (codes uint8 [..., n], scale fp32 [...], zero fp32 [...]); scale and
    zero hold values of T.
    """
    if bits not in (2, 4):
        raise ValueError("bits must be 2 or 4")
    steps = (1 << bits) - 1
    x32 = np.asarray(x, dtype=np.float32)
    mn = x32.min(axis=-1)
    mx = x32.max(axis=-1)
    mn = np.where(mn == 0, np.float32(0.0), mn).astype(np.float32)  # -0.0 -> +0.0
    mx = np.where(mx == 0, np.float32(0.0), mx).astype(np.float32)  # (min/max do not order signed zeros)
    diff = (mx.astype(np.float32) - mn).astype(np.float32)          # fp32 subtract
    s = round_to_T((diff / np.float32(steps)).astype(np.float32), dtype)
    d = x32.astype(np.float64) - mn.astype(np.float64)[..., None]   # fp64 subtract
    s64 = s.astype(np.float64)[..., None]
    codes = np.zeros(d.shape, dtype=np.uint8)
    for k in range(steps):
        codes += (d >= (k + 0.5) * s64).astype(np.uint8)    # (k + 0.5) * s is exact in fp64
    codes = np.where(s64 == 0, np.uint8(0), codes).astype(np.uint8)
    return codes, s, mn


def key_group_bounds(W, G):
    """Token runs of one compress event: [(0,G), (G,2G), ..., (kG, W)]."""
    return [(lo, min(lo + G, W)) for lo in range(0, W, G)]


def quantize_keys(K_ev, G, dtype, bits=2):
    """Keys of one compress event, [W][d] in eviction order.

    Returns codes [W][d] uint8, scale [ceil(W/G)][d], zero [ceil(W/G)][d]."""
    W, d = K_ev.shape
    K_ev = np.asarray(K_ev, dtype=np.float32)
    bounds = key_group_bounds(W, G)
    codes = np.zeros((W, d), dtype=np.uint8)
    s = np.zeros((len(bounds), d), dtype=np.float32)
    z = np.zeros((len(bounds), d), dtype=np.float32)
    for j, (lo, hi) in enumerate(bounds):
        c, sj, zj = quantize_groups(K_ev[lo:hi].T, dtype, bits)      # [d][hi-lo]: one group per channel
        codes[lo:hi] = c.T
        s[j] = sj
        z[j] = zj
    return codes, s, z


def value_group_bounds(d, G):
    """Channel runs of a value row: [(0,G), (G,2G), ..., (kG, d)]."""
    return [(lo, min(lo + G, d)) for lo in range(0, d, G)]


def quantize_values(V_ev, G, dtype, bits=2):
    """Values of one compress event, [W][d].

    Returns codes [W][d] uint8, scale [W][ceil(d/G)], zero [W][ceil(d/G)]."""
    W, d = V_ev.shape
    bounds = value_group_bounds(d, G)
    codes = np.zeros((W, d), dtype=np.uint8)
    s = np.zeros((W, len(bounds)), dtype=np.float32)
    z = np.zeros((W, len(bounds)), dtype=np.float32)
    for j, (lo, hi) in enumerate(bounds):
        c, sj, zj = quantize_groups(np.asarray(V_ev, dtype=np.float32)[:, lo:hi], dtype, bits)
        codes[:, lo:hi] = c
        s[:, j] = sj
        z[:, j] = zj
    return codes, s, z


def dequantize_keys(codes, scale, zero, G, W=None):
    """x_hat[t][c] = zero[g(t)][c] + codes[t][c] * scale[g(t)][c], fp64.  The rows are
    whole compress events of W tokens one after the other (W=None: one event), each
    with ceil(W/G) groups: g(t) = (t // W) * ceil(W/G) + (t % W) // G."""
    n, d = codes.shape
    W = W or max(n, 1)
    t = np.arange(n)
    grp = (t // W) * (-(-W // G)) + (t % W) // G
    return zero.astype(np.float64)[grp] + codes.astype(np.float64) * scale.astype(np.float64)[grp]


def dequantize_values(codes, scale, zero, G):
    """x_hat[t][c] = zero[t][c//G] + codes[t][c] * scale[t][c//G], fp64."""
    n, d = codes.shape
    grp = np.arange(d) // G
    return zero.astype(np.float64)[:, grp] + codes.astype(np.float64) * scale.astype(np.float64)[:, grp]
