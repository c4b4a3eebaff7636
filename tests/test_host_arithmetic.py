"""Host checks (no GPU) of arithmetic identities that the quantizing kernels use in place of
the textbook operation.  Each is a claim about IEEE arithmetic, checked here with the C
library's correctly rounded operations; that the kernels produce the oracle's scales bit
for bit is what the GPU parity tests show."""
import os
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.mark.parametrize("stride", [61])
def test_fp32_quotient_by_three_operations(tmp_path, stride):
    """scale = fp32((max - min) / STEPS) (quantizer of Sec. 2.5 / Sec. 3.1 as read here: 3 steps
    for 2 bits, 15 for 4) is formed on the GPU by a multiplication and two fused
    multiply-adds; on a 1-in-61 sample of all non-negative finite fp32 numerators (every
    exponent, 70 million values per divisor) it equals the correctly rounded quotient.
    (`div_three_ops 1` runs the exhaustive check in under a minute.)"""
    exe = tmp_path / "div_three_ops"
    subprocess.run(["gcc", "-O2", "-ffp-contract=off", "-o", str(exe), os.path.join(HERE, "host", "div_three_ops.c"), "-lm"],
                   check=True)
    r = subprocess.run([str(exe), str(stride)], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "mismatches 0" in r.stdout


# ---- 2-bit codes from order-preserving 16-bit keys -------------------------------------------
# A numpy restatement of the arithmetic of the quantizing kernels' 2-bit path (not their code:
# the kernels are HIP), checked against the oracle's quantizer, which takes the definition
# literally (exact differences, three threshold compares).  It covers what random GPU inputs
# rarely hold: subnormals of T, signed zeros, all-negative groups, exact ties, flat groups.
import numpy as np

from oracle import quantizer


def _bits_of(x32, dtype):
    if dtype == "f16":
        return x32.astype(np.float16).view(np.uint16).astype(np.uint32)
    return (x32.view(np.uint32) >> 16).astype(np.uint32)


def _value_of(bits, dtype):
    bits = np.asarray(bits, dtype=np.uint32)
    if dtype == "f16":
        return bits.astype(np.uint16).view(np.float16).astype(np.float32)
    return (bits << 16).astype(np.uint32).view(np.float32)


def _key(bits):
    bits = np.asarray(bits, dtype=np.uint32)
    return np.where(bits & 0x8000, ~bits & 0xFFFF, bits | 0x8000).astype(np.uint32)


def _threshold_key(z, s, k_plus_half, dtype):
    """key(smallest value of T >= z + (k + 1/2) s) - 1, by the kernel's steps: fp64 sum, fp32
    rounding plus the side it fell on, nearest T, at most one key upwards, zero taken as -0."""
    t = np.float64(z) + np.float64(k_plus_half) * np.float64(s)
    f = np.float32(t)
    up = np.float64(f) < t
    h_bits = _bits_of(quantizer.round_to_T(np.array([f], np.float32), dtype), dtype)   # nearest, ties to even
    hb = _value_of(h_bits, dtype)[0]
    key = int(_key(h_bits)[0]) + int(hb < f or (hb == f and up))
    if key == 0x8000:
        key = 0x7FFF
    return 0xFFFF if s == 0 else key - 1


def _codes_by_keys(x32, dtype):
    keys = _key(_bits_of(x32, dtype))
    inv = lambda k: np.where(k & 0x8000, k ^ 0x8000, ~k & 0xFFFF)
    mn = _value_of(inv(keys.min()), dtype)
    mx = _value_of(inv(keys.max()), dtype)
    mn = np.float32(0.0) if mn == 0 else np.float32(mn)
    mx = np.float32(0.0) if mx == 0 else np.float32(mx)
    s = quantizer.round_to_T(np.array([(mx - mn) / np.float32(3)], np.float32), dtype)[0]
    th = [_threshold_key(mn, s, k + 0.5, dtype) for k in range(3)]
    return sum((keys > t).astype(np.uint8) for t in th), s, mn


def _groups(rng, dtype):
    tiny = 2.0 ** -24 if dtype == "f16" else 2.0 ** -133
    for _ in range(300):
        n = int(rng.integers(2, 40))
        kind = rng.integers(0, 7)
        scale = 2.0 ** rng.integers(-20, 14) if dtype == "f16" else 2.0 ** rng.integers(-100, 14)
        if kind == 0:
            x = rng.standard_normal(n) * scale
        elif kind == 1:
            x = -np.abs(rng.standard_normal(n)) * scale - scale          # all negative
        elif kind == 2:
            x = rng.integers(-6, 7, n) * tiny                            # subnormals and zeros of T
        elif kind == 3:
            x = np.where(rng.random(n) < 0.5, 0.0, -0.0) + (rng.random(n) < 0.2) * tiny
        elif kind == 4:
            x = np.full(n, rng.standard_normal() * scale)                # flat
        elif kind == 5:
            x = rng.integers(0, 13, n) * scale / 4 - rng.integers(0, 9) * scale   # exact ties on a grid
        else:
            x = rng.standard_normal(n) * scale + 1000 * scale            # small range on a large offset
        if dtype == "f16":
            x = np.clip(x, -60000.0, 60000.0)                            # the contract: finite values of T
        yield quantizer.round_to_T(x.astype(np.float32), dtype)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_two_bit_codes_from_sixteen_bit_keys(dtype):
    rng = np.random.default_rng([2503_19950, 77, dtype == "bf16"])
    seen_codes = set()
    for x in _groups(rng, dtype):
        want_codes, want_s, want_z = quantizer.quantize_groups(x[None, :], dtype)
        got_codes, got_s, got_z = _codes_by_keys(x, dtype)
        assert got_s == want_s[0] and got_z == want_z[0] and np.signbit(got_z) == np.signbit(want_z[0])
        assert np.array_equal(got_codes, want_codes[0]), (x, got_codes, want_codes[0])
        seen_codes.update(got_codes.tolist())
    assert seen_codes == {0, 1, 2, 3}
