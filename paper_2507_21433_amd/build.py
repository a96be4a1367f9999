"""Build the C-ABI HIP library for gfx950 in-tree (``paper_2507_21433_amd/librc.so``) and, beside it, the
benchmark's MFMA-rate probe (``librc_probe.so``, a measurement aid that the search library does not contain)."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "librc.so")
PROBE_LIB = os.path.join(HERE, "librc_probe.so")
SOURCES = ["rc_norms.hip", "rc_match.hip", "rc_remap.hip", "rc_candidates.hip", "rc_pat.hip", "rc_pool.hip", "rc_evict.hip"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unused-const-variable",
    "-Wno-inline-asm",   # the m0 clobber of the direct-to-LDS loads is deliberate (m0 is set inside the same asm block)
]


def build(verbose=False):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    cmd += [os.path.join(CSRC, s) for s in SOURCES] + ["-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    probe = [hipcc] + FLAGS + [os.path.join(CSRC, "probe_mfma.hip"), "-o", PROBE_LIB]
    if verbose:
        print(" ".join(probe), flush=True)
    subprocess.check_call(probe)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
