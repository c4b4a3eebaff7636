"""GPU parity for windows that the group size does not divide (the paper's W = floor(R/3),
R = 128 / 192 / 256 with G = 64: Sec. 3.1, appendix D): the last key group of every
filtering event is short, the slots behind it are padding.  Streaming, bulk prefill,
decode attention and the fused decode step against the oracle; padding slots must hold
zeros and position -1 and must not take part in the softmax."""
import numpy as np
import pytest

from oracle import attention
from oracle.cache import SliceCache
from paper_2503_19950_amd import inputs
from tests import gpu_util as U

pytestmark = pytest.mark.gpu

CASES = [
    # name, workload, L
    ("w42_g64_bf16", U.make_wl(B=1, Hq=8, Hkv=2, d=128, G=64, F=84, dtype="bf16", sinks=4), 42 * 11 + 17),
    ("w85_g64_bf16", U.make_wl(B=2, Hq=8, Hkv=2, d=128, G=64, F=170, dtype="bf16"), 85 * 7 + 40),
    ("w85_g64_d96_bits4", U.make_wl(B=1, Hq=4, Hkv=4, d=96, G=64, F=170, dtype="f16", bits=4, dist="laplace"),
     85 * 5 + 84),
    ("w21_g32_d64", U.make_wl(B=2, Hq=4, Hkv=2, d=64, G=32, F=42), 21 * 30 + 5),
    ("w50_g128_tiles_of_padding_only", U.make_wl(B=1, Hq=8, Hkv=1, d=128, G=128, F=100), 50 * 9 + 3),
    ("w130_g128", U.make_wl(B=1, Hq=4, Hkv=2, d=128, G=128, F=260, dtype="bf16"), 130 * 5 + 77),
    ("w10_g32_gqa3", U.make_wl(B=1, Hq=6, Hkv=2, d=128, G=32, F=20), 10 * 25 + 3),
    ("w1_g32", U.make_wl(B=1, Hq=4, Hkv=1, d=128, G=32, F=2), 40),
    ("w42_g64_exactly_at_event", U.make_wl(B=1, Hq=4, Hkv=1, d=128, G=64, F=84), 126),
    ("w42_g64_one_before_event", U.make_wl(B=1, Hq=4, Hkv=1, d=128, G=64, F=84), 125),
]


@pytest.mark.parametrize("name,wl,L", CASES, ids=[c[0] for c in CASES])
def test_streaming_prefill_and_attention(name, wl, L):
    seed_id = 600 + [c[0] for c in CASES].index(name)
    print("case", name, "L", L, flush=True)
    streamed = U.build_gpu(wl, seed_id, L, poison=True)
    bulk = U.build_gpu_prefill(wl, seed_id, L, poison=True)
    a, b = U.live_buffers(streamed, wl), U.live_buffers(bulk, wl)
    for key in a:
        assert np.array_equal(a[key], b[key]), key
    ocs = {}
    for bb in range(wl["B"]):
        for h in range(wl["Hkv"]):
            oc = U.build_oracle(wl, seed_id, L, bb, h)
            U.check_state(streamed, oc, wl, bb, h)
            U.check_state(bulk, oc, wl, bb, h)
            ocs[(bb, h)] = oc
    q = inputs.queries(seed_id, 0, wl)
    U.check_attention(streamed, ocs, wl, q)
    U.check_attention(bulk, ocs, wl, q, scale=0.2)


@pytest.mark.parametrize("name,wl,L0,steps", [
    ("w42_g64_bf16", U.make_wl(B=2, Hq=8, Hkv=2, d=128, G=64, F=84, dtype="bf16"), 100, 75),   # events at 126, 168
    ("w21_g32_bits4_from_empty", U.make_wl(B=1, Hq=4, Hkv=2, d=64, G=32, F=42, bits=4), 0, 90),
])
def test_decode_steps_across_events(name, wl, L0, steps):
    """Prefill, then one token per step with logquant_decode_step (append + compress +
    attend at the step that fills the window): outputs and state against the oracle."""
    import torch
    seed_id = 650 + len(name)
    dt, W, gh = wl["dtype"], wl["F"] // 2, wl["Hq"] // wl["Hkv"]
    K, V = inputs.batch_kv(seed_id, 0, L0 + steps, wl)
    Kd, Vd = U.to_dev(K, dt), U.to_dev(V, dt)
    dc = U.new_cache(wl, L0 + steps)
    ocs = {}
    for b in range(wl["B"]):
        for h in range(wl["Hkv"]):
            ocs[(b, h)] = SliceCache(W, wl["G"], wl["d"], dt, wl.get("bits", 2))
            if L0:
                ocs[(b, h)].append_block(K[b, h, :L0], V[b, h, :L0])
    if L0:
        dc.prefill(Kd[:, :, :L0].contiguous(), Vd[:, :, :L0].contiguous())
    for s in range(steps):
        t = L0 + s
        q = inputs.queries(seed_id, s, wl)
        kn, vn = Kd[:, :, t:t + 1].contiguous(), Vd[:, :, t:t + 1].contiguous()
        if dc.c.n_fp + 1 < 3 * W:
            out = dc.decode_step(kn, vn, U.to_dev(q, dt))
        else:
            dc.stream_in(kn, vn)
            out = dc.decode_attn(U.to_dev(q, dt))
        torch.cuda.synchronize()
        out = out.float().cpu().numpy()
        for (b, h), oc in ocs.items():
            oc.append(K[b, h, t], V[b, h, t])
            want = attention.decode_attention(oc, q[b, h * gh:(h + 1) * gh])
            U.assert_outputs_close(out[b, h * gh:(h + 1) * gh], want, dt, "step %d (b=%d,h=%d)" % (s, b, h))
    for (b, h), oc in ocs.items():
        U.check_state(dc, oc, wl, b, h)
