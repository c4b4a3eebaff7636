"""GPU parity of the per-sequence entry points (Algorithm 1 runs per sequence, Sec. 2.5:
in a batch of sequences of different lengths every row fills its window and runs its
filtering events at its own pace).  Every row is compared with an oracle cache of its own."""
import os

import numpy as np
import pytest

from oracle import attention
from oracle.cache import SliceCache
from paper_2503_19950_amd import inputs
from tests import gpu_util as U

pytestmark = pytest.mark.gpu


def _new(wl, Lmax, poison=False):
    from paper_2503_19950_amd import binding
    cfg = binding.make_config(wl["B"], wl["Hq"], wl["Hkv"], wl["d"], wl["F"], wl["G"], wl["dtype"],
                              U.q_capacity_for(wl, Lmax), wl.get("bits", 2))
    return binding.DeviceCacheSeq(cfg, poison=poison)


def _oracles(wl, K, V, lengths):
    ocs = {}
    for b in range(wl["B"]):
        for h in range(wl["Hkv"]):
            oc = SliceCache(wl["F"] // 2, wl["G"], wl["d"], wl["dtype"], wl.get("bits", 2))
            if lengths[b]:
                oc.append_block(K[b, h, :lengths[b]], V[b, h, :lengths[b]])
            ocs[(b, h)] = oc
    return ocs


def _check_outputs(out, ocs, wl, q, where):
    gh, dt = wl["Hq"] // wl["Hkv"], wl["dtype"]
    out = out.float().cpu().numpy()
    assert np.isfinite(out).all()
    for (b, h), oc in ocs.items():
        want = attention.decode_attention(oc, q[b, h * gh:(h + 1) * gh])
        U.assert_outputs_close(out[b, h * gh:(h + 1) * gh], want, dt, "%s (b=%d,h=%d)" % (where, b, h))


CASES = [
    # name, workload, prompt lengths (one per batch row), decode steps
    ("w32_f16", U.make_wl(B=4, Hq=8, Hkv=2, d=128, G=32, F=64), [1, 95, 96, 32 * 20 + 7], 70),
    ("w64_g64_bf16_d96", U.make_wl(B=3, Hq=4, Hkv=4, d=96, G=64, F=128, dtype="bf16", dist="laplace"),
     [700, 191, 64 * 9], 40),
    ("w42_g64_padding_slots", U.make_wl(B=3, Hq=8, Hkv=2, d=128, G=64, F=84, dtype="bf16"), [500, 125, 3], 50),
    ("bits4_one_row_empty_prompt", U.make_wl(B=3, Hq=4, Hkv=2, d=64, G=32, F=64, bits=4), [0, 333, 96], 35),
    # more rows than one hand-over launch carries (64)
    ("b70_d64", U.make_wl(B=70, Hq=2, Hkv=1, d=64, G=32, F=64),
     [int(x) for x in np.random.default_rng(70).integers(1, 400, size=70)], 34),
]


@pytest.mark.parametrize("name,wl,lengths,steps", CASES, ids=[c[0] for c in CASES])
def test_prefill_and_decode_with_per_sequence_lengths(name, wl, lengths, steps):
    import torch
    seed_id = 700 + [c[0] for c in CASES].index(name)
    print("case", name, lengths, flush=True)
    dt, W, B = wl["dtype"], wl["F"] // 2, wl["B"]
    Lmax = max(lengths)
    K, V = inputs.batch_kv(seed_id, 0, Lmax + steps, wl)
    Kd, Vd = U.to_dev(K, dt), U.to_dev(V, dt)
    dc = _new(wl, Lmax + steps, poison=True)
    dc.prefill_seq(Kd[:, :, :Lmax].contiguous(), Vd[:, :, :Lmax].contiguous(), lengths)
    ocs = _oracles(wl, K, V, lengths)
    for (b, h), oc in ocs.items():
        U.check_state(dc, oc, wl, b, h, counts=dc.view(b))
    if min(lengths) > 0:
        q = inputs.queries(seed_id, 999, wl)
        _check_outputs(dc.decode_attn_seq(U.to_dev(q, dt)), ocs, wl, q, "after prefill")
    # decode: row b's next token is its own position lengths[b] + s
    fused = separate = 0
    for s in range(steps):
        kn = torch.stack([Kd[b, :, lengths[b] + s:lengths[b] + s + 1] for b in range(B)]).contiguous()
        vn = torch.stack([Vd[b, :, lengths[b] + s:lengths[b] + s + 1] for b in range(B)]).contiguous()
        q = inputs.queries(seed_id, s, wl)
        if all(dc.n_fp[b] + 1 < 3 * W for b in range(B)):
            out = dc.decode_step_seq(kn, vn, U.to_dev(q, dt))
            fused += 1
        else:
            dc.append_seq(kn, vn)
            dc.compress_seq()
            out = dc.decode_attn_seq(U.to_dev(q, dt))
            separate += 1
        torch.cuda.synchronize()
        for (b, h), oc in ocs.items():
            oc.append(K[b, h, lengths[b] + s], V[b, h, lengths[b] + s])
        _check_outputs(out, ocs, wl, q, "step %d" % s)
    assert fused and separate
    for (b, h), oc in ocs.items():
        U.check_state(dc, oc, wl, b, h, counts=dc.view(b))


def test_rows_that_sit_out_are_untouched():
    """append_seq with an activity mask: only the active rows take a token."""
    import torch
    wl = U.make_wl(B=3, Hq=4, Hkv=2, d=128, G=32, F=64)
    lengths = [100, 40, 250]
    K, V = inputs.batch_kv(750, 0, 300, wl)
    Kd, Vd = U.to_dev(K, "f16"), U.to_dev(V, "f16")
    dc = _new(wl, 400)
    dc.prefill_seq(Kd[:, :, :250].contiguous(), Vd[:, :, :250].contiguous(), lengths)
    ocs = _oracles(wl, K, V, lengths)
    pos = list(lengths)
    for s, active in enumerate([[1, 0, 1], [0, 1, 0], [1, 1, 0], [0, 0, 0], [1, 1, 1]] * 6):
        kn = torch.stack([Kd[b, :, pos[b]:pos[b] + 1] for b in range(3)]).contiguous()
        vn = torch.stack([Vd[b, :, pos[b]:pos[b] + 1] for b in range(3)]).contiguous()
        dc.append_seq(kn, vn, active)
        dc.compress_seq()
        for b in range(3):
            if active[b]:
                for h in range(2):
                    ocs[(b, h)].append(K[b, h, pos[b]], V[b, h, pos[b]])
                pos[b] += 1
    q = inputs.queries(750, 0, wl)
    _check_outputs(dc.decode_attn_seq(U.to_dev(q, "f16")), ocs, wl, q, "after masked appends")
    for (b, h), oc in ocs.items():
        U.check_state(dc, oc, wl, b, h, counts=dc.view(b))


def test_equal_lengths_give_the_lock_step_result_bit_for_bit():
    import torch
    wl = U.make_wl(B=2, Hq=8, Hkv=2, d=128, G=32, F=64)
    L = 333
    K, V = inputs.batch_kv(760, 0, L, wl)
    Kd, Vd = U.to_dev(K, "f16"), U.to_dev(V, "f16")
    a = U.build_gpu_prefill(wl, 760, L, kv=(K, V))
    b = _new(wl, L)
    b.prefill_seq(Kd, Vd, [L, L])
    la, lb = U.live_buffers(a, wl), None
    b.c.cur, b.c.n_fp, b.c.n_q = b.view(0)
    lb = U.live_buffers(b, wl)
    for key in la:
        assert np.array_equal(la[key], lb[key]), key
    q = U.to_dev(inputs.queries(760, 0, wl), "f16")
    oa, ob = a.decode_attn(q), b.decode_attn_seq(q)
    torch.cuda.synchronize()
    if os.environ.get("LOGQUANT_ATTN_WPB") == "4":
        # a forced 4-wavefront shape applies to the lock-step launch only (the per-sequence kernel
        # is built for 8 and 12 wavefronts): the tiles are then summed in another order
        assert (oa.float() - ob.float()).abs().max().item() <= U.TOL["f16"] / 2
    else:
        assert torch.equal(oa, ob)


def test_compress_seq_of_many_full_rows_gives_the_lock_step_state_bit_for_bit():
    """240 slices whose windows fill at the same step: logquant_compress_seq then launches enough
    workgroups to let the quantizing ones move the kept rows as well (the route large lock-step
    batches take); the state must equal the one the lock-step calls reach, buffer by buffer."""
    wl = U.make_wl(B=30, Hq=8, Hkv=8, d=64, G=64, F=256, dtype="bf16")
    W = 128
    L = 4 * W
    K, V = inputs.batch_kv(780, 0, L, wl)
    Kd, Vd = U.to_dev(K, "bf16"), U.to_dev(V, "bf16")
    a = U.new_cache(wl, L)
    assert a.stream_in(Kd, Vd) == 2
    b = _new(wl, L)
    b.prefill_seq(Kd[:, :, :L - 1].contiguous(), Vd[:, :, :L - 1].contiguous(), [L - 1] * wl["B"])
    assert all(b.n_fp[i] == 3 * W - 1 for i in range(wl["B"]))
    b.append_seq(Kd[:, :, L - 1:].contiguous(), Vd[:, :, L - 1:].contiguous())
    b.compress_seq()
    assert all(b.view(i) == b.view(0) for i in range(wl["B"]))
    b.c.cur, b.c.n_fp, b.c.n_q = b.view(0)
    la, lb = U.live_buffers(a, wl), U.live_buffers(b, wl)
    for key in la:
        assert np.array_equal(la[key], lb[key]), key


def test_error_codes():
    from paper_2503_19950_amd import binding as B
    wl = U.make_wl(B=2, Hq=4, Hkv=2, d=128, G=32, F=64)
    K, V = inputs.batch_kv(770, 0, 200, wl)
    Kd, Vd = U.to_dev(K, "f16"), U.to_dev(V, "f16")
    dc = _new(wl, 200)
    q = U.to_dev(inputs.queries(770, 0, wl), "f16")
    out = q.clone()
    assert B.logquant_decode_attn_seq(dc.cfg, dc.cs, q, 0.0, out, dc.workspace) == B.LQ_ERR_STATE   # empty rows
    assert B.logquant_prefill_seq(dc.cfg, dc.cs, Kd, Vd, [10, 201], 200) == B.LQ_ERR_SHAPE
    assert B.logquant_prefill_seq(dc.cfg, dc.cs, Kd, Vd, [10, 95], 200) == B.LQ_OK
    assert (dc.n_fp[0], dc.n_fp[1], dc.n_q[1]) == (10, 95, 0)
    assert B.logquant_prefill_seq(dc.cfg, dc.cs, Kd, Vd, [10, 95], 200) == B.LQ_ERR_STATE           # not empty
    kn, vn = Kd[:, :, :1].contiguous(), Vd[:, :, :1].contiguous()
    assert B.logquant_decode_step_seq(dc.cfg, dc.cs, kn, vn, q, 0.0, out, dc.workspace) == B.LQ_ERR_STATE  # row 1 fills
    assert (dc.n_fp[0], dc.n_fp[1]) == (10, 95)
    assert B.logquant_append_seq(dc.cfg, dc.cs, kn, vn) == B.LQ_OK and dc.n_fp[1] == 96
    assert B.logquant_append_seq(dc.cfg, dc.cs, kn, vn) == B.LQ_ERR_CAPACITY and dc.n_fp[0] == 11
    assert B.logquant_compress_seq(dc.cfg, dc.cs) == B.LQ_OK
    assert (dc.cur[0], dc.cur[1], dc.n_fp[1], dc.n_q[1]) == (0, 1, 64, 32)
    assert B.logquant_compress_seq(dc.cfg, dc.cs) == B.LQ_OK            # nothing to do
    assert (dc.cur[1], dc.n_fp[1], dc.n_q[1]) == (1, 64, 32)
