"""Compile the HIP library for gfx950 into paper_2604_15180_amd/libentmax_attn.so."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libentmax_attn.so")
SOURCES = [os.path.join(CSRC, "api.hip")]
HEADERS = [os.path.join(CSRC, f) for f in ("tiles.hpp", "common.hpp", "fwd_kernels.hpp", "bwd_kernels.hpp")] + [
    os.path.join(os.path.dirname(HERE), "include", "entmax_attn.h")]


def build(force: bool = True, verbose: bool = False) -> str:
    if not force and os.path.exists(LIB):
        newest = max(os.path.getmtime(f) for f in SOURCES + HEADERS)
        if os.path.getmtime(LIB) >= newest:
            return LIB
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           # keep MFMA results in ordinary VGPRs: the AGPR form costs a v_accvgpr copy per
           # accumulator register each time the vector ALUs touch a score tile
           "-mllvm", "-amdgpu-mfma-vgpr-form=1",
           "-Wno-unused-command-line-argument"]
    if verbose:
        cmd += ["-Rpass-analysis=kernel-resource-usage"]
    cmd += ["-o", LIB] + SOURCES
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
