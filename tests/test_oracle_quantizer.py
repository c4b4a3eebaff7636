"""Pins for oracle/quantizer.py: 2-bit asymmetric min/max group quantizer
(INT2, group size G: Sec. 3.1; keys per channel: Sec. 2.5; formula is a reading)."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import quantizer as Q


def _f16(vals):
    return np.array(vals, dtype=np.float16).astype(np.float32)


def _bf16(x):
    return Q.round_to_T(np.asarray(x, np.float32), "bf16")


def test_round_to_T_known_values():
    # bf16: 8 significant bits.  1 + 2^-8 is a tie -> even (1.0); 1 + 3*2^-8 ties up to 1 + 2^-6
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 2.0 ** -7, 1.0 + 3 * 2.0 ** -8, 3.14159274], np.float32)
    want = np.array([1.0, 1.0, 1.0 + 2.0 ** -7, 1.0 + 2.0 ** -6, 3.140625], np.float32)
    assert np.array_equal(Q.round_to_T(x, "bf16"), want)
    # fp16: 11 significant bits: 1 + 2^-11 ties to 1.0, 2049 -> 2048, 2051 -> 2052
    x = np.array([1.0 + 2.0 ** -11, 2049.0, 2051.0, 0.1], np.float32)
    want = np.array([1.0, 2048.0, 2052.0, 0.0999755859375], np.float32)
    assert np.array_equal(Q.round_to_T(x, "f16"), want)


def test_tie_vectors_round_half_up():
    # s = 1.5 exactly, values on the grid z + k*s
    c, s, z = Q.quantize_groups(_f16([0, 4.5, 3, 1.5]), "f16")
    assert s == 1.5 and z == 0 and c.tolist() == [0, 3, 2, 1]
    # s = 1: every interior value is an exact tie; half-up gives 1,2,3 (half-even would give 0,2,2)
    c, s, z = Q.quantize_groups(_f16([0, 3, 0.5, 1.5, 2.5]), "f16")
    assert s == 1.0 and c.tolist() == [0, 3, 1, 2, 3]


def test_exact_grid_reconstructs_exactly():
    z, s = -2.5, 0.75
    x = _f16([z, z + s, z + 2 * s, z + 3 * s, z + s, z])
    c, ss, zz = Q.quantize_groups(x, "f16")
    assert ss == s and zz == z and c.tolist() == [0, 1, 2, 3, 1, 0]
    assert np.array_equal(zz + c * np.float64(ss), x.astype(np.float64))


def test_constant_group_and_signed_zero():
    c, s, z = Q.quantize_groups(_f16([1.25] * 8), "f16")
    assert s == 0 and z == 1.25 and not c.any()
    c, s, z = Q.quantize_groups(np.array([-0.0, 0.0, -0.0], np.float32), "f16")
    assert s == 0 and not np.signbit(z) and not c.any()
    c, s, z = Q.quantize_groups(np.array([-0.0, 3.0], np.float32), "f16")
    assert not np.signbit(z) and s == 1.0 and c.tolist() == [0, 3]


def _exact_reference(xs, dtype, bits=2):
    """Brute force in exact rational arithmetic, the scale taken from the
    definition (correctly rounded fp32 quotient, then nearest-even to T)."""
    steps = (1 << bits) - 1
    fx = [Fraction(float(v)) for v in xs]
    mn, mx = min(fx), max(fx)
    # fp32 subtract: correctly rounded value of the exact difference
    diff = _round_fraction_to_f32(mx - mn)
    quo = _round_fraction_to_f32(Fraction(float(diff)) / steps)
    s = Fraction(float(Q.round_to_T(np.float32(quo), dtype)))
    codes = []
    for v in fx:
        dlt = v - mn
        codes.append(0 if s == 0 else sum(int(dlt >= (2 * k + 1) * s / 2) for k in range(steps)))
    return codes, s, mn


def _round_fraction_to_f32(fr):
    """Nearest fp32 to an exact rational, ties to even, by exact comparison."""
    x = np.float32(float(fr))
    lo = np.nextafter(x, np.float32(-np.inf), dtype=np.float32)
    hi = np.nextafter(x, np.float32(np.inf), dtype=np.float32)
    cands = [(abs(Fraction(float(c)) - fr), int(np.float32(c).view(np.uint32)) & 1, c)
             for c in (x, lo, hi)]
    return min(cands, key=lambda t: (t[0], t[1]))[2]


@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_against_exact_rational_arithmetic(dtype, bits):
    rng = np.random.default_rng(7 + bits)
    for trial in range(300):
        n = int(rng.integers(2, 9 if bits == 2 else 40))
        scale = 10.0 ** rng.uniform(-3, 2)
        x = Q.round_to_T((rng.standard_normal(n) * scale).astype(np.float32), dtype)
        if trial % 5 == 0:      # grids with many exact ties
            x = Q.round_to_T((rng.integers(0, 7 if bits == 2 else 31, n) * 0.5).astype(np.float32), dtype)
        codes, s, z = Q.quantize_groups(x, dtype, bits)
        rc, rs, rz = _exact_reference(x, dtype, bits)
        assert Fraction(float(s)) == rs and Fraction(float(z)) == rz
        assert codes.tolist() == rc


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_invariants(dtype):
    rng = np.random.default_rng(11)
    x = Q.round_to_T(rng.standard_normal((500, 32)).astype(np.float32) * 3, dtype)
    x[:, 5] *= 10
    codes, s, z = Q.quantize_groups(x, dtype)
    assert codes.min() == 0 and codes.max() == 3
    rows = np.arange(x.shape[0])
    assert (codes[rows, x.argmin(1)] == 0).all() and (codes[rows, x.argmax(1)] == 3).all()
    order = np.argsort(x, axis=1, kind="stable")
    assert (np.diff(np.take_along_axis(codes.astype(int), order, 1), axis=1) >= 0).all()   # monotone
    xhat = z.astype(np.float64)[:, None] + codes * s.astype(np.float64)[:, None]
    err = np.abs(xhat - x)
    rng_ = (x.max(1) - x.min(1)).astype(np.float64)
    bound = np.maximum(s / 2.0, rng_ - 3.0 * s)       # top bin may exceed s/2 when s was rounded down
    assert (err <= bound[:, None] + 1e-300).all()
    # with a scale that was not rounded down the bound is exactly s/2
    ok = 3.0 * s.astype(np.float64) >= rng_
    assert (err[ok] <= (s[ok] / 2.0)[:, None]).all()


def test_key_and_value_grouping_axes():
    rng = np.random.default_rng(3)
    W, d, G = 64, 96, 32
    K = Q.round_to_T(rng.standard_normal((W, d)).astype(np.float32), "f16")
    kc, ks, kz = Q.quantize_keys(K, G, "f16")
    assert kc.shape == (W, d) and ks.shape == (W // G, d)
    # keys: statistics along tokens, per channel, per run of G tokens
    for g in range(W // G):
        for c in (0, 17, 95):
            col = K[g * G:(g + 1) * G, c]
            assert kz[g, c] == col.min()
            c1, s1, _ = Q.quantize_groups(col, "f16")
            assert ks[g, c] == s1 and (kc[g * G:(g + 1) * G, c] == c1).all()
    # values: statistics along channels, per token; ragged tail when G does not divide d
    G = 64
    vc, vs, vz = Q.quantize_values(K, G, "f16")
    assert vs.shape == (W, 2) and Q.value_group_bounds(d, G) == [(0, 64), (64, 96)]
    for t in (0, 13, 63):
        assert vz[t, 0] == K[t, :64].min() and vz[t, 1] == K[t, 64:].min()
        c1, s1, _ = Q.quantize_groups(K[t, 64:], "f16")
        assert vs[t, 1] == s1 and (vc[t, 64:] == c1).all()
    # dequantization addresses the same groups
    Kh = Q.dequantize_keys(kc, ks, kz, 32)
    assert np.abs(Kh - K).max() <= (ks.max() / 2) * 1.0001 + 1e-3
    Vh = Q.dequantize_values(vc, vs, vz, G)
    t, c = 5, 70
    assert Vh[t, c] == vz[t, 1].astype(np.float64) + vc[t, c] * vs[t, 1].astype(np.float64)
    t, c = 40, 3
    assert Kh[t, c] == kz[1, c].astype(np.float64) + kc[t, c] * ks[1, c].astype(np.float64)


def test_short_last_key_group_of_an_event():
    """W = 85 (the paper's floor(256/3)), G = 64: runs of 64 and 21 tokens, each with its
    own statistics; two events one after the other are addressed per event."""
    rng = np.random.default_rng(7)
    W, d, G = 85, 64, 64
    assert Q.key_group_bounds(W, G) == [(0, 64), (64, 85)] and Q.key_group_bounds(42, 64) == [(0, 42)]
    K = Q.round_to_T(rng.standard_normal((2 * W, d)).astype(np.float32), "bf16")
    parts = [Q.quantize_keys(K[e * W:(e + 1) * W], G, "bf16") for e in range(2)]
    for e, (kc, ks, kz) in enumerate(parts):
        assert kc.shape == (W, d) and ks.shape == (2, d) and kz.shape == (2, d)
        for j, (lo, hi) in enumerate(((0, 64), (64, 85))):
            for c in (0, 31, 63):
                col = K[e * W + lo:e * W + hi, c]
                c1, s1, z1 = Q.quantize_groups(col, "bf16")
                assert kz[j, c] == col.min() == z1 and ks[j, c] == s1
                assert (kc[lo:hi, c] == c1).all()
    codes = np.concatenate([p[0] for p in parts])
    scale = np.concatenate([p[1] for p in parts])
    zero = np.concatenate([p[2] for p in parts])
    Kh = Q.dequantize_keys(codes, scale, zero, G, W)
    for t, grp in ((0, 0), (63, 0), (64, 1), (84, 1), (85, 2), (85 + 64, 3), (169, 3)):
        want = zero[grp].astype(np.float64) + codes[t] * scale[grp].astype(np.float64)
        assert np.array_equal(Kh[t], want)
    # every dequantized value within half a step of the original (scale not rounded down)
    t = np.arange(2 * W)
    s_t = scale[(t // W) * 2 + (t % W) // G].astype(np.float64)
    assert (np.abs(Kh - K) <= s_t / 2 * 1.01 + 1e-6).all()
    # a group that divides evenly gives what the run-by-run form gives
    kc, ks, kz = Q.quantize_keys(K[:128], 64, "bf16")
    c1, s1, z1 = Q.quantize_keys(K[64:128], 64, "bf16")
    assert np.array_equal(kc[64:], c1) and np.array_equal(ks[1:], s1) and np.array_equal(kz[1:], z1)


# ---- 4-bit variant (Sec. 3.2.1, Table 3: the same method at higher precision) ----

def test_four_bit_tie_vectors_and_exact_grid():
    # 16 values on a grid of step 0.5: s = 7.5 / 15 = 0.5 exactly, every value is its own level
    x = _f16([k * 0.5 for k in range(16)])
    c, s, z = Q.quantize_groups(x, "f16", bits=4)
    assert s == 0.5 and z == 0 and c.tolist() == list(range(16))
    assert np.array_equal(z + c * np.float64(s), x.astype(np.float64))
    # s = 1 (range 15): the half-integers are exact ties and go up (half-even would send 0.5 -> 0, 2.5 -> 2)
    c, s, z = Q.quantize_groups(_f16([0, 15, 0.5, 1.5, 2.5, 13.5, 14.5]), "f16", bits=4)
    assert s == 1.0 and c.tolist() == [0, 15, 1, 2, 3, 14, 15]
    # a value just below a tie stays down
    c, s, z = Q.quantize_groups(_f16([0, 15, 2.498046875]), "f16", bits=4)
    assert c.tolist() == [0, 15, 2]


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_four_bit_invariants(dtype):
    rng = np.random.default_rng(13)
    x = Q.round_to_T(rng.standard_normal((400, 64)).astype(np.float32) * 3, dtype)
    x[:, 9] *= 10
    codes, s, z = Q.quantize_groups(x, dtype, bits=4)
    assert codes.min() == 0 and codes.max() == 15
    rows = np.arange(x.shape[0])
    assert (codes[rows, x.argmin(1)] == 0).all() and (codes[rows, x.argmax(1)] == 15).all()
    order = np.argsort(x, axis=1, kind="stable")
    assert (np.diff(np.take_along_axis(codes.astype(int), order, 1), axis=1) >= 0).all()
    xhat = z.astype(np.float64)[:, None] + codes * s.astype(np.float64)[:, None]
    err = np.abs(xhat - x)
    rng_ = (x.max(1) - x.min(1)).astype(np.float64)
    assert (err <= np.maximum(s / 2.0, rng_ - 15.0 * s)[:, None] + 1e-300).all()
    # five times finer than 2 bits on the same data
    c2, s2, _ = Q.quantize_groups(x, dtype, bits=2)
    ratio = s2.astype(np.float64) / s.astype(np.float64)
    assert (np.abs(ratio - 5.0) < 0.05).all()
    with pytest.raises(ValueError):
        Q.quantize_groups(x, dtype, bits=3)
