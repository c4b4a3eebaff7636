"""CPU-side checks of the C ABI: the library loads, exports every declared symbol,
and rejects bad arguments before touching the GPU."""
import ctypes as C
import os
import re

import pytest

from paper_2503_19950_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "logquant.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(logquant_\w+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    syms = _declared_symbols()
    assert set(syms) == set(B.EXPORTS)
    lib = C.CDLL(B.LIB_PATH)
    for s in syms:
        assert getattr(lib, s) is not None


def _cfg(**kw):
    a = dict(B=1, Hq=32, Hkv=8, d=128, fp_budget=128, group=32, dtype="f16", q_capacity=1024)
    a.update(kw)
    return B.make_config(**a)


def test_sizes_match_the_documented_layouts():
    s = B.logquant_sizes(_cfg())
    bh, cap, d, qc = 8, 192, 128, 1024
    assert s.k_fp == s.v_fp == bh * cap * d * 2
    assert s.k_codes == s.v_codes == bh * qc * d // 4
    assert s.k_meta == bh * (qc // 32) * d * 2 and s.v_meta == bh * qc * 4 * 2
    assert s.pos_fp == cap * 4 and s.pos_q == qc * 4
    assert s.workspace == B.logquant_workspace_bytes(_cfg()) > 0
    s4 = B.logquant_sizes(_cfg(bits=4))
    assert s4.k_codes == s4.v_codes == bh * qc * d // 2 and s4.k_meta == s.k_meta and s4.k_fp == s.k_fp
    s = B.logquant_sizes(_cfg(d=96, group=64, Hq=8, Hkv=8, fp_budget=384, q_capacity=384 * 2))
    assert s.v_meta == 8 * 768 * 2 * 2        # ceil(96/64) = 2 channel groups
    # the paper's W = floor(128/3) = 42 with G = 64: the fp buffers hold 3W = 126 rows rounded up to
    # whole 32-row tiles; every filtering event takes 64 quantized slots (one short key group)
    s = B.logquant_sizes(_cfg(fp_budget=84, group=64, q_capacity=640))
    assert s.k_fp == 8 * 128 * 128 * 2 and s.pos_fp == 128 * 4
    assert s.k_meta == 8 * (640 // 64) * 128 * 2 and s.k_codes == 8 * 640 * 128 // 4
    # W = 85 (floor(256/3)): 128 slots per event
    assert B._lib.logquant_sizes(C.byref(_cfg(fp_budget=170, group=64, q_capacity=128 * 5)), C.byref(B.lq_sizes())) == B.LQ_OK
    assert B._lib.logquant_sizes(C.byref(_cfg(fp_budget=170, group=64, q_capacity=85 * 64)), C.byref(B.lq_sizes())) == B.LQ_ERR_SHAPE


@pytest.mark.parametrize("kw,status", [
    (dict(bits=3), B.LQ_ERR_UNSUPPORTED),
    (dict(bits=8), B.LQ_ERR_UNSUPPORTED),
    (dict(d=80), B.LQ_ERR_UNSUPPORTED),
    (dict(group=16), B.LQ_ERR_UNSUPPORTED),
    (dict(fp_budget=170, group=64, q_capacity=192), B.LQ_ERR_SHAPE),   # W = 85, G = 64: an event takes 128 slots
    (dict(B=4096, Hq=16, Hkv=8), B.LQ_ERR_UNSUPPORTED),       # more (row, head) pairs than a launch has grid rows
    (dict(Hq=30), B.LQ_ERR_SHAPE),
    (dict(B=0), B.LQ_ERR_SHAPE),
    (dict(q_capacity=1000), B.LQ_ERR_SHAPE),
    (dict(fp_budget=127), B.LQ_ERR_SHAPE),
])
def test_bad_configs_are_rejected(kw, status):
    cfg = _cfg(**kw)
    out = B.lq_sizes()
    assert B._lib.logquant_sizes(C.byref(cfg), C.byref(out)) == status
    assert B.logquant_workspace_bytes(cfg) == 0
    cache = B.lq_cache()
    assert B.logquant_compress(cfg, cache) == status
    plan = B.lq_plan()
    assert B._lib.logquant_decode_plan(C.byref(cfg), 1, 0, C.byref(plan)) == status


def test_null_and_state_errors_without_a_gpu():
    cfg = _cfg()
    cache = B.lq_cache()                       # all pointers null
    assert B.logquant_compress(None, cache) == B.LQ_ERR_NULL
    assert B.logquant_compress(cfg, None) == B.LQ_ERR_NULL
    assert B.logquant_compress(cfg, cache) == B.LQ_ERR_NULL
    assert B.logquant_append(cfg, cache, None, None, 1) == B.LQ_ERR_NULL
    assert B.logquant_decode_attn(cfg, cache, None, 0.0, None, None) == B.LQ_ERR_NULL
    # fake non-null pointers: the state checks run before anything is enqueued
    for name, _ in B.lq_cache._fields_[3:10]:
        setattr(cache, name, 4096)
    for i in range(2):
        cache.k_fp[i] = cache.v_fp[i] = cache.pos_fp[i] = 4096
    cache.n_fp, cache.n_q = 10, 0
    assert B.logquant_compress(cfg, cache) == B.LQ_ERR_STATE            # window not full
    assert B.logquant_append(cfg, cache, 4096, 4096, 183) == B.LQ_ERR_CAPACITY
    assert B.logquant_append(cfg, cache, 4096, 4096, 0) == B.LQ_ERR_SHAPE
    cache.n_fp, cache.n_q = 192, 1024
    assert B.logquant_compress(cfg, cache) == B.LQ_ERR_CAPACITY         # quantized region full
    cache.n_fp, cache.n_q = 0, 0
    assert B.logquant_decode_attn(cfg, cache, 4096, 0.0, 4096, 4096) == B.LQ_ERR_STATE   # empty cache
    cache.n_q = 10
    assert B.logquant_compress(cfg, cache) == B.LQ_ERR_STATE            # n_q not a multiple of W
    assert cache.n_fp == 0 and cache.cur == 0                           # nothing was modified


def test_prefill_argument_and_state_errors_without_a_gpu():
    cfg = _cfg()                                # W = 64, q_capacity 1024
    cache = B.lq_cache()
    assert B.logquant_prefill(cfg, cache, 4096, 4096, 10) == B.LQ_ERR_NULL     # null cache buffers
    assert B.logquant_prefill(cfg, cache, None, 4096, 10) == B.LQ_ERR_NULL
    for name, _ in B.lq_cache._fields_[3:10]:
        setattr(cache, name, 4096)
    for i in range(2):
        cache.k_fp[i] = cache.v_fp[i] = cache.pos_fp[i] = 4096
    assert B.logquant_prefill(cfg, cache, 4096, 4096, 0) == B.LQ_ERR_SHAPE
    # 18 events fit 1024 + ... : L = 3W + 15W = 18W -> 16 events -> 1024 slots; one more window does not fit
    assert B.logquant_prefill(cfg, cache, 4096, 4096, 19 * 64) == B.LQ_ERR_CAPACITY
    cache.n_fp = 5
    assert B.logquant_prefill(cfg, cache, 4096, 4096, 10) == B.LQ_ERR_STATE    # cache not empty
    assert (cache.n_fp, cache.n_q, cache.cur) == (5, 0, 0)


@pytest.mark.parametrize("W", [1, 2, 3, 5, 8, 42, 64, 96, 128, 192, 256])
def test_prefill_positions_match_algorithm_1(W):
    """The closed form the prefill kernel places rows by (host entry point) against the
    literal list simulation of Algorithm 1 in the oracle (Sec. 2.5)."""
    from oracle import selection
    import random
    rnd = random.Random(W)
    Ls = list(range(0, 14 * W + 2)) if W <= 8 else \
        [0, 1, W, 2 * W, 3 * W - 1, 3 * W, 3 * W + 1, 4 * W - 1, 4 * W, 5 * W + 7, 12 * W, 40 * W + 3] + \
        [rnd.randrange(1, 70 * W) for _ in range(12)]
    for L in Ls:
        st, a, q = B.logquant_prefill_positions(W, L)
        A, Q = selection.stream_eager(L, W)
        assert st == B.LQ_OK and a == A and q == Q, (W, L)
    assert B.logquant_prefill_positions(0, 5)[0] == B.LQ_ERR_SHAPE
    assert B.logquant_prefill_positions(4, -1)[0] == B.LQ_ERR_SHAPE


def test_plan_reports_the_algorithmic_bytes():
    # cfg 1: 128 fp rows and 384 quantized rows per slice, 8 slices:
    # 128*512 + 384*96 bytes each
    p = B.logquant_decode_plan(_cfg(), 128, 384)
    assert p.bytes_read == 8 * (128 * 512 + 384 * 96) == 819200
    cfg3 = _cfg(fp_budget=512, group=64, dtype="bf16", q_capacity=131072)
    assert B.logquant_decode_plan(cfg3, 512, 130560).bytes_read == 85655552
    cfg5 = _cfg(B=16, Hq=32, Hkv=32, d=96, fp_budget=384, group=64, dtype="bf16", q_capacity=32256 + 192 * 2)
    assert B.logquant_decode_plan(cfg5, 512, 32256).bytes_read == 1124597760
    assert p.blocks >= 1 and p.splits >= 1
    # 4-bit codes: d/2 bytes per slot for keys and for values
    assert B.logquant_decode_plan(_cfg(bits=4), 128, 384).bytes_read == 8 * (128 * 512 + 384 * (128 + 32))


def test_decode_step_errors_without_a_gpu():
    cfg = _cfg()                               # W = 64: capacity 192 fp rows
    cache = B.lq_cache()
    assert B.logquant_decode_step(cfg, cache, 4096, 4096, 4096, 0.0, 4096, 4096) == B.LQ_ERR_NULL
    for name, _ in B.lq_cache._fields_[3:10]:
        setattr(cache, name, 4096)
    for i in range(2):
        cache.k_fp[i] = cache.v_fp[i] = cache.pos_fp[i] = 4096
    assert B.logquant_decode_step(cfg, cache, None, 4096, 4096, 0.0, 4096, 4096) == B.LQ_ERR_NULL
    cache.n_fp = 191                           # the append would fill the window: separate calls needed
    assert B.logquant_decode_step(cfg, cache, 4096, 4096, 4096, 0.0, 4096, 4096) == B.LQ_ERR_STATE
    assert cache.n_fp == 191


def test_launch_plans_of_the_five_workloads():
    """Workgroup shape and split count the planner picks: every compute unit gets work,
    the chip is filled in one round, and the fp share gets at least one wavefront."""
    shapes = {
        1: (dict(), 128, 384),
        2: (dict(B=8, fp_budget=256, q_capacity=8192), 256, 7936),
        3: (dict(fp_budget=512, group=64, dtype="bf16", q_capacity=131072), 512, 130560),
        4: (dict(B=64, fp_budget=256, q_capacity=4352), 256, 3840),
        5: (dict(B=16, Hq=32, Hkv=32, d=96, fp_budget=384, group=64, dtype="bf16", q_capacity=32256 + 384), 512, 32256),
    }
    for w, (kw, n_fp, n_q) in shapes.items():
        p = B.logquant_decode_plan(_cfg(**kw), n_fp, n_q)
        assert p.waves_per_block in (4, 8, 12) and p.splits >= 1 and 1 <= p.fp_waves < p.splits * p.waves_per_block
        if w >= 2:
            assert 256 <= p.blocks <= 512, (w, p.blocks)
            assert p.blocks * p.waves_per_block <= 256 * 12
    p3 = B.logquant_decode_plan(_cfg(**shapes[3][0]), 512, 130560)
    assert (p3.waves_per_block, p3.splits) == (12, 32)
    p4 = B.logquant_decode_plan(_cfg(**shapes[4][0]), 256, 3840)
    assert (p4.waves_per_block, p4.splits) == (4, 1)
    # 4-bit codes are not built for 12-wavefront workgroups
    assert B.logquant_decode_plan(_cfg(bits=4, **shapes[3][0]), 512, 130560).waves_per_block == 8
    # the variant that skips padding slots (window not a multiple of the group size) exists for 8 and
    # 12 wavefronts (never 4): 12 when a wavefront gets six tiles or more and the launch fits the chip
    # in one round, else 8
    rag = _cfg(fp_budget=84, group=64, dtype="bf16", q_capacity=3200 * 64)
    assert B.logquant_decode_plan(rag, 100, 3118 * 64).waves_per_block == 12
    rag4 = _cfg(B=64, fp_budget=170, group=64, q_capacity=128 * 48)
    assert B.logquant_decode_plan(rag4, 200, 128 * 46).waves_per_block == 8      # 512 workgroups: two rounds
    assert B.logquant_decode_plan(rag4, 200, 128 * 8).waves_per_block == 8


def test_plan_counts_live_slots_only_and_state_checks_use_slots():
    # W = 42, G = 64: 64 slots per filtering event, 42 of them hold tokens; key scales and
    # zero-points exist once per 64 slots
    cfg = _cfg(fp_budget=84, group=64, q_capacity=640)
    p = B.logquant_decode_plan(cfg, 100, 5 * 64)
    assert p.bytes_read == 8 * (100 * 512 + 5 * 42 * (64 + 8) + 5 * 512)
    assert B._lib.logquant_decode_plan(C.byref(cfg), 100, 5 * 42, C.byref(B.lq_plan())) == B.LQ_ERR_STATE
    assert B._lib.logquant_decode_plan(C.byref(cfg), 127, 64, C.byref(B.lq_plan())) == B.LQ_ERR_STATE   # n_fp > 3W = 126


def test_status_strings():
    assert B.logquant_status_string(0) == "ok"
    assert "capacity" in B.logquant_status_string(B.LQ_ERR_CAPACITY)


def test_per_sequence_calls_check_their_arguments_without_a_gpu():
    cfg = _cfg(B=3, fp_budget=64, q_capacity=256)          # W = 32
    assert B.logquant_seq_state_bytes(cfg) == 3 * 32
    assert B.logquant_seq_state_bytes(_cfg(d=80)) == 0
    cs = B.lq_cache_seq()
    assert B.logquant_compress_seq(cfg, cs) == B.LQ_ERR_NULL
    assert B.logquant_append_seq(cfg, cs, 4096, 4096) == B.LQ_ERR_NULL
    for name, _ in B.lq_cache_seq._fields_[3:10]:
        setattr(cs, name, 4096)
    for i in range(2):
        cs.k_fp[i] = cs.v_fp[i] = cs.pos_fp[i] = 4096
    cs.seq_state = 4096
    cur, n_fp, n_q = (C.c_int32 * 3)(0, 1, 0), (C.c_int32 * 3)(10, 96, 50), (C.c_int32 * 3)(0, 64, 32)
    cs.cur, cs.n_fp, cs.n_q = (C.cast(x, C.POINTER(C.c_int32)) for x in (cur, n_fp, n_q))
    assert B.logquant_decode_step_seq(cfg, cs, 4096, 4096, 4096, 0.0, 4096, 4096) == B.LQ_ERR_STATE   # row 1 is full
    assert B.logquant_append_seq(cfg, cs, 4096, 4096) == B.LQ_ERR_CAPACITY
    assert B.logquant_prefill_seq(cfg, cs, 4096, 4096, [5, 5, 5], 8) == B.LQ_ERR_STATE                # rows not empty
    assert list(n_fp) == [10, 96, 50] and list(n_q) == [0, 64, 32] and list(cur) == [0, 1, 0]
    n_q[2] = 33                                                                                     # not a multiple of W
    assert B.logquant_compress_seq(cfg, cs) == B.LQ_ERR_STATE
    n_q[2] = 32
    n_q[1] = 256                                                                                    # no room for the event
    assert B.logquant_compress_seq(cfg, cs) == B.LQ_ERR_CAPACITY
    # plan: made for the longest row with the general kernel variant (8 wavefronts), bytes summed over the rows
    p = B.logquant_decode_plan_seq(cfg, [10, 96, 50], [0, 64, 32])
    assert p.waves_per_block == 8      # (12 for long rows, never 4)
    assert p.bytes_read == 8 * ((10 + 96 + 50) * 512 + (64 + 32) * 96)
    with pytest.raises(B.LogQuantError):
        B.logquant_decode_plan_seq(cfg, [0, 96, 50], [0, 64, 32])                                   # an empty row


def test_static_scratch_entry_point_rejects_configs_beyond_its_array():
    """logquant_decode_attn_static: argument errors and the size limit are reported before
    any HIP call (no GPU needed)."""
    cfg = B.make_config(1, 32, 8, 128, 512, 64, "bf16", 4096)
    assert B.logquant_decode_attn_static(None, None, None, 0.0, None) == B.LQ_ERR_NULL
    cache = B.lq_cache()
    assert B.logquant_decode_attn_static(cfg, cache, 1, 0.0, 1) == B.LQ_ERR_NULL      # null cache buffers
    big = B.make_config(128, 32, 8, 128, 256, 32, "f16", 4096)     # B * Hq = 4096 > 3640: counters beyond 4 MiB
    for name, _ in B.lq_cache._fields_[:10]:
        if name in ("k_fp", "v_fp", "pos_fp"):
            getattr(cache, name)[0] = 1
            getattr(cache, name)[1] = 1
        else:
            setattr(cache, name, 1)
    cache.n_fp, cache.n_q = 10, 0
    assert B.logquant_decode_attn_static(big, cache, 1, 0.0, 1) == B.LQ_ERR_CAPACITY
