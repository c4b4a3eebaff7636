"""The decode-attention call recorded into a HIP graph: the library allocates nothing,
synchronises nothing and clears its counters inside the kernel, so a call with fixed
counts can be captured and replayed.  Every replay is checked against the eager result,
with eager work and synchronisations between the replays."""
import numpy as np
import pytest

from paper_2503_19950_amd import inputs
from tests import gpu_util as U

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,wl,L", [
    ("several_splits", U.make_wl(B=1, Hq=8, Hkv=2, d=128, G=64, F=128, dtype="bf16"), 64 * 40 + 17),
    ("one_split_per_group", U.make_wl(B=48, Hq=8, Hkv=8, d=128, G=32, F=64), 333),
])
def test_decode_attention_replays_from_a_graph(name, wl, L):
    import torch
    dt = wl["dtype"]
    dc = U.build_gpu_prefill(wl, 800, L)
    qs = [U.to_dev(inputs.queries(800, s, wl), dt) for s in range(4)]
    eager = [dc.decode_attn(q).clone() for q in qs]
    torch.cuda.synchronize()
    q_in = qs[0].clone()
    out = torch.empty_like(q_in)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        dc.decode_attn(q_in, out)                 # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        dc.decode_attn(q_in, out)
    for rep in range(3):
        for i, q in enumerate(qs):
            q_in.copy_(q)
            g.replay()
            torch.cuda.synchronize()
            assert torch.equal(out, eager[i]), (rep, i)
            # eager work between the replays, on the same cache and workspace
            again = dc.decode_attn(qs[(i + 1) % 4])
            torch.cuda.synchronize()
            assert torch.equal(again, eager[(i + 1) % 4])
