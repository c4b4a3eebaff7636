"""Pins for oracle/layout.py: the documented index functions are bijections onto
their buffers and agree with hand-evaluated positions."""
import numpy as np
import pytest

from oracle import layout


@pytest.mark.parametrize("d", [64, 96, 128])
def test_fp_index_functions_are_bijections(d):
    cap = 96
    t = np.arange(cap)[:, None]
    c = np.arange(d)[None, :]
    for fn in (layout.k_fp_index, layout.v_fp_index):
        idx = np.broadcast_to(fn(t, c, d), (cap, d)).ravel()
        assert sorted(idx.tolist()) == list(range(cap * d))


@pytest.mark.parametrize("d", [64, 96, 128])
def test_code_positions_are_a_bijection_onto_bit_pairs(d):
    n = 128
    t = np.arange(n)[:, None]
    c = np.arange(d)[None, :]
    for fn in (layout.k_code_word_bit, layout.v_code_word_bit):
        w, b = fn(t, c, d)
        assert (b % 2 == 0).all() and b.max() == 30
        key = (np.broadcast_to(w, (n, d)) * 16 + np.broadcast_to(b, (n, d)) // 2).ravel()
        assert sorted(key.tolist()) == list(range(n * d))      # every 2-bit field used once


@pytest.mark.parametrize("d,G", [(128, 32), (128, 64), (96, 64), (64, 128)])
def test_v_meta_bijection(d, G):
    n = 96
    ngc = -(-d // G)
    idx = set()
    for t in range(n):
        for c in range(0, d, G):
            idx.add(int(layout.v_meta_index(t, c, d, G)))
    assert idx == set(range(n * ngc))


def test_hand_evaluated_positions():
    # kperm: 32 slots -> (lane group, element): x = 21 -> 8*((21%16)//4) + 4*(21//16) + 21%4 = 8+4+1
    assert int(layout.kperm(21)) == 13 and sorted(layout.kperm(np.arange(32)).tolist()) == list(range(32))
    d = 128
    # key code of slot 53 (block 1, x = 21, upper 16-row tile, row 5), channel 77 (chunk 2, octet 1, i 5)
    w, b = layout.k_code_word_bit(53, 77, d)
    o = 1 * 4 + 2
    assert int(w) == (1 * 64 + 16 * 1 + 5) * 4 + o // 2 and int(b) == 8 * (o % 2) + 2 * 2 + 16 * 1
    # value code of slot 53 (k = 13: lane group 1, element 5), channel 77 (tile 4, column 13)
    w, b = layout.v_code_word_bit(53, 77, d)
    assert int(w) == (1 * 64 + 16 * 1 + 13) * 4 + 2 and int(b) == 8 * 0 + 2 * 2 + 16 * 1
    assert int(layout.k_fp_index(53, 77, d)) == (((3 * 4 + 2) * 64) + 16 * 1 + 5) * 8 + 5
    assert int(layout.v_fp_index(53, 77, d)) == (((1 * 8 + 4) * 64) + 16 * 1 + 13) * 8 + 5
    assert int(layout.k_meta_index(53, 77, d, 32)) == 1 * 128 + 77
    assert int(layout.v_meta_index(53, 77, d, 32)) == ((1 * 4 + 2) * 32) + 13


@pytest.mark.parametrize("d", [96, 128])
def test_pack_unpack_roundtrip(d):
    rng = np.random.default_rng(0)
    codes = rng.integers(0, 4, (160, d)).astype(np.uint8)
    for which in ("k", "v"):
        words = layout.pack_codes(codes, which)
        assert words.shape == (160 // 32 * 64 * (d // 32),)
        assert np.array_equal(layout.unpack_codes(words, which, 160, d), codes)
    rows = rng.standard_normal((96, d)).astype(np.float32)
    for which in ("k", "v"):
        assert np.array_equal(layout.gather_fp(layout.scatter_fp(rows, which, 96), which, 96, d), rows)
    meta = rng.standard_normal((64, -(-d // 64))).astype(np.float32)
    assert np.array_equal(layout.gather_v_meta(layout.scatter_v_meta(meta, d, 64), 64, d, 64), meta)


# ---- 4-bit codes: one word per (lane, operand) ----

@pytest.mark.parametrize("d", [64, 96, 128])
def test_four_bit_code_positions_are_a_bijection_onto_nibbles(d):
    n = 128
    t = np.arange(n)[:, None]
    c = np.arange(d)[None, :]
    for fn in (layout.k_code_word_bit, layout.v_code_word_bit):
        w, b = fn(t, c, d, 4)
        assert (b % 4 == 0).all() and b.max() == 28
        key = (np.broadcast_to(w, (n, d)) * 8 + np.broadcast_to(b, (n, d)) // 4).ravel()
        assert sorted(key.tolist()) == list(range(n * d))      # every nibble used once


def test_four_bit_hand_evaluated_positions_and_roundtrip():
    d = 128
    # key code of slot 53 (block 1, upper 16-row tile, row 5), channel 77 (chunk 2, octet 1, element 5)
    w, b = layout.k_code_word_bit(53, 77, d, 4)
    assert int(w) == (1 * 64 + 16 * 1 + 5) * 8 + (1 * 4 + 2) and int(b) == 4 * 2 + 16 * 1
    # value code of slot 53 (k = 13: lane group 1, element 5), channel 77 (tile 4, column 13)
    w, b = layout.v_code_word_bit(53, 77, d, 4)
    assert int(w) == (1 * 64 + 16 * 1 + 13) * 8 + 4 and int(b) == 4 * 2 + 16 * 1
    rng = np.random.default_rng(1)
    codes = rng.integers(0, 16, (96, d)).astype(np.uint8)
    for which in ("k", "v"):
        words = layout.pack_codes(codes, which, bits=4)
        assert words.shape == (96 // 32 * 64 * (d // 32) * 2,)
        assert np.array_equal(layout.unpack_codes(words, which, 96, d, bits=4), codes)


def test_slot_mapping_with_short_key_groups():
    """Window 42, group 64 (the paper's floor(128/3)): every filtering event takes 64 slots,
    the first 42 hold its tokens in eviction order; window 85: 128 slots, 85 live."""
    assert layout.slots_per_event(42, 64) == 64 and layout.slots_per_event(85, 64) == 128 and layout.slots_per_event(64, 64) == 64
    assert layout.slots_per_event(96, 32) == 96 and layout.slots_per_event(1, 32) == 32
    s = layout.token_slots(3 * 42, 42, 64)
    assert s[:42].tolist() == list(range(42)) and s[42] == 64 and s[83] == 105 and s[84] == 128
    assert np.array_equal(layout.token_slots(200, 50, 25), np.arange(200))     # G divides W: identity
    rows = np.arange(2 * 85 * 3).reshape(170, 3)
    out = layout.to_slots(rows, 85, 64, fill=-1)
    assert out.shape == (256, 3)
    assert np.array_equal(out[:85], rows[:85]) and (out[85:128] == -1).all()
    assert np.array_equal(out[128:213], rows[85:]) and (out[213:] == -1).all()
