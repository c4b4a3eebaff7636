"""The launch planner picks the workgroup shape of the attention kernel (4, 8 or 12
wavefronts) from the workload; small test cases only ever get one of them.  Here a few
parity cases are run again in child processes with each shape forced (the planner's
environment overrides are read once per process)."""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CASES = "cfg1 or d64_gqa2_ragged or mha_d96_g64_bf16_midwindow or d128_g128_gqa8 or gqa3_odd_ratio or bits4_cfg1 or repeated_calls " \
        "or fused_decode_step"


@pytest.mark.parametrize("knob", ["LOGQUANT_ATTN_WPB=12", "LOGQUANT_ATTN_WPB=4", "LOGQUANT_ATTN_DYNAMIC=0"])
def test_parity_cases_with_forced_kernel_variant(knob):
    env = dict(os.environ)
    k, v = knob.split("=")
    env[k] = v
    # the second file: windows the group size does not divide (padding slots in the quantized region);
    # the third: per-sequence lengths
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_gpu_parity.py"),
                        os.path.join(ROOT, "tests", "test_gpu_ragged_window.py"),
                        os.path.join(ROOT, "tests", "test_gpu_per_sequence.py"), "-m", "gpu",
                        "-x", "-q", "-k", CASES + " or w42 or w85 or w50 or w1_g32 or per_sequence or sit_out", "--timeout", "300",
                        "--timeout-method", "thread"],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    print(r.stdout[-2000:])
    assert r.returncode == 0, r.stdout[-3000:] + r.stderr[-2000:]
