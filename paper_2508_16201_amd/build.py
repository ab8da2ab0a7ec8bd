"""Build step: compile the HIP sources in ``csrc/`` into ``libspecvlm.so`` for
gfx950 with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libspecvlm.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed-fp32 VALU forms are kept off for every device function
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # MFMA results feed VALU code (softmax, exponentials): keep them in arch VGPRs
    # instead of AGPRs so no v_accvgpr_read copies are needed
    "-mllvm", "-amdgpu-mfma-vgpr-form=1",
    "-Wno-unused-command-line-argument",
]


def sources():
    return sorted(glob.glob(os.path.join(HERE, "csrc", "*.hip")))


# A second build for the CPU tests: the HOST code of the same sources (argument validation, launch
# planning, workspace sizing) under AddressSanitizer + UndefinedBehaviorSanitizer; device code unchanged.
LIB_HOSTSAN = os.path.join(HERE, "libspecvlm_hostsan.so")
HOSTSAN_FLAGS = ["-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                 "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-shared-libsan"]


def build(verbose: bool = False, host_sanitizers: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out_lib = LIB_HOSTSAN if host_sanitizers else LIB
    flags = [f if f != "-O3" else "-O1" for f in HIPCC_FLAGS] + HOSTSAN_FLAGS if host_sanitizers else HIPCC_FLAGS
    cmd = [hipcc, *flags, "-I", os.path.join(ROOT, "include"),
           "-I", os.path.join(HERE, "csrc"), "-o", out_lib, *sources()]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # the host pass warns that it does not know the packed-fp32 feature: harmless
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        sys.stderr.write(out + "\n")
        raise RuntimeError("hipcc failed")
    if verbose and out.strip():
        print(out)
    return out_lib


if __name__ == "__main__":
    print(build(verbose=True))
