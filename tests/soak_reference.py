"""Child process of test_gpu_merge_soak.py: the same launches with ONE context split
(no cross-workgroup merge), results written to an .npy file.  The planner reads
LOGQUANT_ATTN_SPLITS once per process, hence the separate process.

usage: python -m tests.soak_reference <out.npy> <launches>"""
import sys

import numpy as np


def main():
    out_path, n = sys.argv[1], int(sys.argv[2])
    import torch
    from tests import test_gpu_merge_soak as S
    from paper_2503_19950_amd import binding
    caches, qs = S.build()
    plan = binding.logquant_decode_plan(caches[0].cfg, caches[0].c.n_fp, caches[0].c.n_q)
    assert plan.splits == 1, plan.splits
    outs = torch.empty((n,) + tuple(qs.shape[1:]), dtype=qs.dtype, device=qs.device)
    for i in range(n):
        caches[i % len(caches)].decode_attn(qs[i % qs.shape[0]], out=outs[i])
    torch.cuda.synchronize()
    np.save(out_path, outs.float().cpu().numpy())


if __name__ == "__main__":
    main()
