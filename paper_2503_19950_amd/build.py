"""Build the gfx950 shared library in-tree with hipcc (no torch extension machinery:
the library has a plain C ABI and is loaded with ctypes)."""
import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liblogquant.so")
# the plain vector-unit attention kernel: test and measurement aid, not part of the product library
CSRC_PLAIN = os.path.join(HERE, "csrc_plain")
LIB_PLAIN = os.path.join(HERE, "liblogquant_plain.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _hipcc(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
    # the host pass does not know the gfx9 feature name and says so once per function
    noise = "'-packed-fp32-ops' is not a recognized feature"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if err.strip():
        print(err, flush=True)
    if r.returncode:
        raise RuntimeError("hipcc failed (exit %d)" % r.returncode)


def build(verbose=False):
    """Compile every HIP source for gfx950 (always recompiles): csrc/ into liblogquant.so, the
    product; csrc_plain/ into liblogquant_plain.so, which tests and the benchmark's
    vector-unit measurement load on top of it."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    inc = ["-I", os.path.join(HERE, "..", "include")]
    _hipcc([hipcc, *HIPCC_FLAGS, *inc, "-o", LIB, *sources()], verbose)
    _hipcc([hipcc, *HIPCC_FLAGS, *inc, "-o", LIB_PLAIN, *sorted(glob.glob(os.path.join(CSRC_PLAIN, "*.hip"))),
            "-L", HERE, "-llogquant", "-Wl,-rpath,$ORIGIN"], verbose)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
