"""Seeded sweep over configurations the hand-picked parity cases do not cover: every
head dimension, group size, cache type and code width the library accepts, odd
grouped-query ratios, batch sizes and context lengths around window boundaries, and
(the last 16 cases) windows of any length, which the group size does not divide.  Each
case builds its state with logquant_prefill, continues with fused decode steps, and is
compared with the oracle (state bit for bit, outputs to tolerance)."""
import numpy as np
import pytest

from paper_2503_19950_amd import inputs
from tests import gpu_util as U

pytestmark = pytest.mark.gpu


def _cases(seed=20250319):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(28):
        d = int(rng.choice([64, 96, 128]))
        G = int(rng.choice([32, 64, 128]))
        W = G * int(rng.choice([1, 1, 2, 3]))
        gh = int(rng.choice([1, 2, 3, 4, 6, 8]))
        Hkv = int(rng.choice([1, 2, 3]))
        B = int(rng.choice([1, 1, 2, 3]))
        bits = int(rng.choice([2, 2, 4]))
        dtype = str(rng.choice(["f16", "bf16"]))
        events = int(rng.integers(0, 7))
        L = 1 + int(rng.integers(0, 3 * W - 1)) if events == 0 else 3 * W + (events - 1) * W + int(rng.integers(0, W))
        wl = U.make_wl(B=B, Hq=gh * Hkv, Hkv=Hkv, d=d, G=G, F=2 * W, dtype=dtype, bits=bits,
                       dist=str(rng.choice(["normal", "laplace"])), sinks=int(rng.choice([0, 0, 4])))
        steps = int(rng.integers(1, 6))
        out.append(("%02d_d%d_g%d_w%d_gh%d_hkv%d_b%d_%s_bits%d_L%d" % (i, d, G, W, gh, Hkv, B, dtype, bits, L), wl, L, steps))
    # windows the group size does not divide (short last key group per filtering event, padding slots)
    rng = np.random.default_rng(seed + 1)
    for i in range(28, 44):
        d = int(rng.choice([64, 96, 128]))
        G = int(rng.choice([32, 64, 128]))
        W = int(rng.integers(1, 3 * G))
        if W % G == 0:
            W += 1
        gh = int(rng.choice([1, 2, 3, 4, 8]))
        Hkv = int(rng.choice([1, 2, 3]))
        B = int(rng.choice([1, 1, 2]))
        bits = int(rng.choice([2, 2, 4]))
        dtype = str(rng.choice(["f16", "bf16"]))
        events = int(rng.integers(0, 9))
        L = 1 + int(rng.integers(0, 3 * W - 1)) if events == 0 else 3 * W + (events - 1) * W + int(rng.integers(0, W))
        wl = U.make_wl(B=B, Hq=gh * Hkv, Hkv=Hkv, d=d, G=G, F=2 * W, dtype=dtype, bits=bits,
                       dist=str(rng.choice(["normal", "laplace"])), sinks=int(rng.choice([0, 0, 4])))
        steps = int(rng.integers(1, 6))
        out.append(("%02d_d%d_g%d_w%d_gh%d_hkv%d_b%d_%s_bits%d_L%d" % (i, d, G, W, gh, Hkv, B, dtype, bits, L), wl, L, steps))
    return out


# plus one case of another seed with large logits and few tokens sharing the weight, which exceeded the
# fp16 tolerance while q*s entered the matrix unit as two 11-bit pieces
# (its name keeps its own number: the data seed is derived from it)
# and one bf16 case of another seed in which one token carries the weight and outputs lie in [2, 4), where
# half an ulp of bf16 is 7.8e-3 of the 1e-2: it exceeded the tolerance (1.008e-2) while the head piece of the
# probabilities had all 11 bits and its product with the value scale was rounded to fp16
CASES = _cases() + [_cases(112)[2], _cases(17)[27]]


@pytest.mark.parametrize("name,wl,L,steps", CASES, ids=[c[0] for c in CASES])
def test_random_configuration(name, wl, L, steps):
    import torch
    from oracle import attention
    seed_id = 500 + int(name[:2])
    dt = wl["dtype"]
    W = wl["F"] // 2
    print("case", name, flush=True)
    K, V = inputs.batch_kv(seed_id, 0, L + steps, wl)
    dc = U.build_gpu_prefill(wl, seed_id, L, q_capacity=U.q_capacity_for(wl, L + steps), kv=(K[:, :, :L], V[:, :, :L]))
    slices = [(b, h) for b in range(wl["B"]) for h in range(wl["Hkv"])]
    ocs = {s: U.build_oracle(wl, seed_id, L, *s) for s in slices}
    for s, oc in ocs.items():
        U.check_state(dc, oc, wl, *s)
    U.check_attention(dc, ocs, wl, inputs.queries(seed_id, 99, wl))
    gh = wl["Hq"] // wl["Hkv"]
    Kd, Vd = U.to_dev(K, dt), U.to_dev(V, dt)
    for j in range(steps):
        t = L + j
        kn, vn = Kd[:, :, t:t + 1].contiguous(), Vd[:, :, t:t + 1].contiguous()
        q_np = inputs.queries(seed_id, j, wl)
        if dc.c.n_fp + 1 < 3 * W:
            out = dc.decode_step(kn, vn, U.to_dev(q_np, dt))
        else:
            dc.append(kn, vn)
            dc.compress()
            out = dc.decode_attn(U.to_dev(q_np, dt))
        torch.cuda.synchronize()
        o = out.float().cpu().numpy()
        for (b, h), oc in ocs.items():
            oc.append(K[b, h, t], V[b, h, t])
            want = attention.decode_attention(oc, q_np[b, h * gh:(h + 1) * gh], None)
            U.assert_outputs_close(o[b, h * gh:(h + 1) * gh], want, dt, "step %d (b=%d,h=%d)" % (j, b, h))
    for s, oc in ocs.items():
        U.check_state(dc, oc, wl, *s)
