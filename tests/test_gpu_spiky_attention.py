"""GPU parity on inputs with concentrated attention (the generator of the Table-2
analogue, Sec. 2.2 / 2.3 of the paper: a few positions at log-uniform distances carry
most of the probability mass, logits reach +-15).  Prefill + decode attention against
the oracle, 2-bit and 4-bit; also the output-level form of the diagnostic: the L1
distance of the compressed-cache output to the exact-attention output agrees between
the HIP path and the oracle."""
import numpy as np
import pytest

from oracle import attention
from oracle.cache import SliceCache
from paper_2503_19950_amd import inputs
from tests import gpu_util as U

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("cfg_id,L,bits", [(3, 8192, 2), (3, 8192 + 333, 4), (2, 4096, 2)],
                         ids=["cfg3_bf16_g64", "cfg3_bits4_ragged_tail", "cfg2_f16_g32"])
def test_spiky_inputs(cfg_id, L, bits):
    wl = dict(inputs.WORKLOADS[cfg_id], B=1, bits=bits)
    gh, dt = wl["Hq"] // wl["Hkv"], wl["dtype"]
    print("spiky", cfg_id, L, bits, flush=True)
    K = np.empty((1, wl["Hkv"], L, wl["d"]), np.float32)
    V = np.empty_like(K)
    for h in range(wl["Hkv"]):
        K[0, h], V[0, h], _ = inputs.slice_kv_spiky(cfg_id, 0, h, L, wl)
    q = inputs.queries_spiky(cfg_id, 0, wl)[:1]
    dc = U.build_gpu_prefill(wl, cfg_id, L, kv=(K, V))
    ocs = {}
    for h in range(wl["Hkv"]):
        oc = SliceCache(wl["F"] // 2, wl["G"], wl["d"], dt, bits)
        oc.append_block(K[0, h], V[0, h])
        U.check_state(dc, oc, wl, 0, h)
        ocs[(0, h)] = oc
    U.check_attention(dc, ocs, wl, q)

    # output-level diagnostic: distance to exact attention over the uncompressed rows
    import torch
    out = dc.decode_attn(U.to_dev(q, dt)).float().cpu().numpy()
    torch.cuda.synchronize()
    for h in range(wl["Hkv"]):
        qh = q[0, h * gh:(h + 1) * gh]
        exact = attention.softmax_attention(qh, K[0, h], V[0, h])
        o_want = attention.decode_attention(ocs[(0, h)], qh)
        want = np.abs(o_want - exact).sum(-1)
        got = np.abs(out[0, h * gh:(h + 1) * gh] - exact).sum(-1)
        # the two distances differ by at most the sum over channels of the output bound
        assert (np.abs(got - want) <= U.output_bound(o_want, dt)[0].sum(-1)).all()
