"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the
same seeded inputs.  Integer results (positions, packed codes, scales, zero-points,
fp rows) must match bit for bit; attention outputs within 2e-3 (fp16) / 1e-2 (bf16)
max-abs of the oracle's fp64 result."""
import numpy as np
import pytest

from paper_2503_19950_amd import inputs
from tests import gpu_util as U

pytestmark = pytest.mark.gpu

SMALL = [
    # name, workload overrides, L
    ("cfg1", dict(inputs.WORKLOADS[1]), 512),
    ("mha_d96_g64_bf16_midwindow", U.make_wl(B=2, Hq=4, Hkv=4, d=96, G=64, F=128, dtype="bf16",
                                             dist="laplace"), 700),
    ("d64_gqa2_ragged", U.make_wl(B=2, Hq=4, Hkv=2, d=64, G=32, F=64), 333),
    ("d128_g64_bf16_sinks", U.make_wl(B=1, Hq=8, Hkv=2, d=128, G=64, F=128, dtype="bf16",
                                      sinks=4), 1000),
    ("d128_g64_bf16_large_values", U.make_wl(B=1, Hq=8, Hkv=2, d=128, G=64, F=128, dtype="bf16",
                                             v_outliers=True, sinks=4, sink_v=True), 1000),
    # bf16 caches whose scales lie below fp16's normal range (6.1e-5): the stored parameters are
    # fp16 values (rounded there), the codes were formed with the bf16 ones
    ("d128_g64_bf16_scales_fp16_subnormal", U.make_wl(B=1, Hq=8, Hkv=2, d=128, G=64, F=128, dtype="bf16",
                                                      gain=1e-6), 700),
    ("d96_g64_bf16_scales_around_fp16_min_normal", U.make_wl(B=1, Hq=4, Hkv=4, d=96, G=64, F=128, dtype="bf16",
                                                             gain=1e-5, dist="laplace"), 500),
    ("d128_g128_gqa8", U.make_wl(B=1, Hq=8, Hkv=1, d=128, G=128, F=256), 900),
    ("gqa3_odd_ratio", U.make_wl(B=1, Hq=6, Hkv=2, d=128, G=32, F=64), 200),
    ("all_fp_no_quantized_rows", U.make_wl(B=2, Hq=8, Hkv=2, d=128, G=32, F=128), 50),
    ("single_token", U.make_wl(B=1, Hq=4, Hkv=1, d=128, G=32, F=64), 1),
    ("exactly_at_event", U.make_wl(B=1, Hq=4, Hkv=1, d=128, G=32, F=64), 96),
    ("one_before_event", U.make_wl(B=1, Hq=4, Hkv=1, d=128, G=32, F=64), 95),
    # the 4-bit variant (Sec. 3.2.1, Table 3)
    ("bits4_cfg1", dict(inputs.WORKLOADS[1], bits=4), 512),
    ("bits4_d128_g64_bf16_sinks", U.make_wl(B=1, Hq=8, Hkv=2, d=128, G=64, F=128, dtype="bf16", sinks=4,
                                            bits=4), 1000),
    ("bits4_mha_d96_g64_bf16_midwindow", U.make_wl(B=2, Hq=4, Hkv=4, d=96, G=64, F=128, dtype="bf16",
                                                   dist="laplace", bits=4), 700),
    ("bits4_d64_gqa2_partial_tile", U.make_wl(B=2, Hq=4, Hkv=2, d=64, G=32, F=64, bits=4), 365),
    ("bits4_d128_g128_gqa8", U.make_wl(B=1, Hq=8, Hkv=1, d=128, G=128, F=256, bits=4), 900),
]


@pytest.mark.parametrize("name,wl,L", SMALL, ids=[s[0] for s in SMALL])
def test_small_cases_every_slice(name, wl, L):
    seed_id = 100 + [s[0] for s in SMALL].index(name)
    print("case", name, "L", L, flush=True)
    dc = U.build_gpu(wl, seed_id, L)
    ocs = {}
    for b in range(wl["B"]):
        for h in range(wl["Hkv"]):
            oc = U.build_oracle(wl, seed_id, L, b, h)
            U.check_state(dc, oc, wl, b, h)
            ocs[(b, h)] = oc
    q = inputs.queries(seed_id, 0, wl)
    U.check_attention(dc, ocs, wl, q)
    U.check_attention(dc, ocs, wl, q, scale=0.2)


def test_single_token_output_is_its_value_row():
    wl = U.make_wl(B=1, Hq=4, Hkv=1, d=128, G=32, F=64)
    dc = U.build_gpu(wl, 150, 1)
    _, V = inputs.slice_kv(150, 0, 0, 0, 1, wl)
    q = inputs.queries(150, 0, wl)
    out = dc.decode_attn(U.to_dev(q, "f16")).float().cpu().numpy()
    assert np.array_equal(out[0], np.broadcast_to(V[0], (4, 128)))


def test_slots_beyond_the_counts_do_not_matter():
    """Unused capacity filled with NaN bit patterns must not change any output."""
    wl = U.make_wl(B=1, Hq=8, Hkv=2, d=128, G=32, F=64)
    q = U.to_dev(inputs.queries(160, 0, wl), "f16")
    outs = []
    for poison in (False, True):
        dc = U.build_gpu(wl, 160, 237, q_capacity=1024, poison=poison)
        outs.append(dc.decode_attn(q).cpu().view(dtype=__import__("torch").int16).numpy())
    assert np.array_equal(outs[0], outs[1])


def test_decode_does_not_modify_the_cache_and_is_repeatable():
    import torch
    wl = U.make_wl(B=2, Hq=8, Hkv=2, d=128, G=32, F=64)
    dc = U.build_gpu(wl, 170, 400)
    before = [t.clone() for t in (dc.k_fp[dc.c.cur], dc.v_fp[dc.c.cur], dc.k_codes, dc.v_codes,
                                  dc.k_scale, dc.v_scale)]
    q = U.to_dev(inputs.queries(170, 0, wl), "f16")
    a = dc.decode_attn(q).clone()
    b = dc.decode_attn(q)
    torch.cuda.synchronize()
    assert torch.equal(a, b)
    after = (dc.k_fp[dc.c.cur], dc.v_fp[dc.c.cur], dc.k_codes, dc.v_codes, dc.k_scale, dc.v_scale)
    assert all(torch.equal(x, y) for x, y in zip(before, after))


def test_error_codes_with_live_device_buffers():
    from paper_2503_19950_amd import binding as B
    wl = U.make_wl(B=1, Hq=4, Hkv=1, d=128, G=32, F=64)
    dc = U.build_gpu(wl, 180, 40, q_capacity=64)
    assert B.logquant_compress(dc.cfg, dc.c) == B.LQ_ERR_STATE          # window not full
    K, V = inputs.batch_kv(180, 40, 200, wl)
    k, v = U.to_dev(K, "f16"), U.to_dev(V, "f16")
    assert B.logquant_append(dc.cfg, dc.c, k, v, 160) == B.LQ_ERR_CAPACITY   # 40 + 160 > 96
    assert dc.c.n_fp == 40
    dc.stream_in(k[:, :, :88], v[:, :, :88])          # two events fill q_capacity = 64
    assert (dc.c.n_fp, dc.c.n_q) == (64, 64)
    dc.append(k[:, :, 88:120].contiguous(), v[:, :, 88:120].contiguous())
    assert dc.c.n_fp == 96
    assert B.logquant_compress(dc.cfg, dc.c) == B.LQ_ERR_CAPACITY       # quantized region is full


@pytest.mark.parametrize("name,wl,L0,steps", [
    ("gqa4_f16", U.make_wl(B=2, Hq=8, Hkv=2, d=128, G=32, F=64), 130, 40),          # crosses events (W = 32)
    ("mha_d96_bf16", U.make_wl(B=2, Hq=4, Hkv=4, d=96, G=64, F=128, dtype="bf16"), 300, 20),
    ("gqa8_two_head_groups", U.make_wl(B=1, Hq=8, Hkv=1, d=128, G=32, F=64), 5, 70),
    ("from_empty_bits4", U.make_wl(B=1, Hq=4, Hkv=2, d=64, G=32, F=64, bits=4), 0, 40),
])
def test_fused_decode_step_equals_append_then_attend(name, wl, L0, steps):
    """logquant_decode_step against logquant_append + logquant_decode_attn on a twin cache:
    same outputs (to tolerance, and against the oracle) and bit-identical cache state
    after every step; at the step that fills the window both use the separate calls."""
    import torch
    seed_id = 400 + len(name)
    dt = wl["dtype"]
    K, V = inputs.batch_kv(seed_id, 0, L0 + steps, wl)
    Kd, Vd = U.to_dev(K, dt), U.to_dev(V, dt)
    qcap = 64 * ((L0 + steps) // 64 + 2)
    a, b = U.new_cache(wl, 0, q_capacity=qcap), U.new_cache(wl, 0, q_capacity=qcap)
    if L0:
        a.prefill(Kd[:, :, :L0].contiguous(), Vd[:, :, :L0].contiguous())
        b.prefill(Kd[:, :, :L0].contiguous(), Vd[:, :, :L0].contiguous())
    cap = 3 * (wl["F"] // 2)
    ocs = {(bb, h): U.build_oracle(wl, seed_id, L0, bb, h) for bb in range(wl["B"]) for h in range(wl["Hkv"])}
    gh = wl["Hq"] // wl["Hkv"]
    for j in range(steps):
        t = L0 + j
        kn, vn = Kd[:, :, t:t + 1].contiguous(), Vd[:, :, t:t + 1].contiguous()
        q_np = inputs.queries(seed_id, j, wl)
        q = U.to_dev(q_np, dt)
        b.append(kn, vn)
        if b.c.n_fp == cap:
            b.compress()
        out_b = b.decode_attn(q)
        if a.c.n_fp + 1 < cap:
            out_a = a.decode_step(kn, vn, q)
        else:
            a.append(kn, vn)
            a.compress()
            out_a = a.decode_attn(q)
        torch.cuda.synchronize()
        assert a.counts() == b.counts()
        assert (out_a.float() - out_b.float()).abs().max().item() <= 2 * 2.0 ** -U.MANT_BITS[dt] * max(1.0, out_b.float().abs().max().item())
        for (bb, h), oc in ocs.items():
            oc.append(K[bb, h, t], V[bb, h, t])
        if j % 13 == 0 or j == steps - 1:
            sa, sb = U.live_buffers(a, wl), U.live_buffers(b, wl)
            for key in sa:
                assert np.array_equal(sa[key], sb[key]), (key, j)
            from oracle import attention
            o = out_a.float().cpu().numpy()
            for (bb, h), oc in ocs.items():
                want = attention.decode_attention(oc, q_np[bb, h * gh:(h + 1) * gh], None)
                U.assert_outputs_close(o[bb, h * gh:(h + 1) * gh], want, dt, "step %d (b=%d,h=%d)" % (j, bb, h))


def test_repeated_calls_with_one_split_and_many_tiles_per_wavefront():
    """One workgroup per head group (no context split) with enough tiles per wavefront that
    a multi-split launch would draw tiles from the pool counters: every call must find the
    counters as the first one did.  (The shape is chosen so that the planner takes one
    split; forcing 12 wavefronts per workgroup through the environment is covered by the
    variant runs.)"""
    import torch
    wl = U.make_wl(B=16, Hq=16, Hkv=16, d=64, G=64, F=128)
    L = 64 * 64 + 128 + 11
    dc = U.build_gpu_prefill(wl, 190, L)
    from paper_2503_19950_amd import binding
    plan = binding.logquant_decode_plan(dc.cfg, dc.c.n_fp, dc.c.n_q)
    import os
    if os.environ.get("LOGQUANT_ATTN_WPB", "0") in ("0", "", "12") and not os.environ.get("LOGQUANT_ATTN_SPLITS"):
        assert plan.splits == 1        # (other forced shapes split the context; the calls are checked all the same)
    ocs = {(b, h): U.build_oracle(wl, 190, L, b, h) for (b, h) in [(0, 0), (7, 9), (15, 15)]}
    for rep in range(3):
        U.check_attention(dc, ocs, wl, inputs.queries(190, rep, wl))
