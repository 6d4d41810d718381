"""Compile the HIP library for gfx950 into paper_2604_15180_amd/libentmax_attn.so.

One translation unit per (input type, head dim) plus the host side; they compile in parallel
into paper_2604_15180_amd/_build/ and are linked into one shared library."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJDIR = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libentmax_attn.so")
UNITS = ["api", "decode", "inst_bf16_d64", "inst_bf16_d128", "inst_f32_d64", "inst_f32_d128"]
HEADERS = [os.path.join(CSRC, f) for f in
           ("tiles.hpp", "common.hpp", "fwd_kernels.hpp", "bwd_kernels.hpp", "launch.hpp", "ops.hpp")] + [
    os.path.join(os.path.dirname(HERE), "include", "entmax_attn.h"),
    os.path.join(os.path.dirname(HERE), "include", "entmax_attn_aids.h")]

BASE = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
        "-Wno-unused-command-line-argument"]
# 16-bit kernels keep MFMA results in ordinary VGPRs: the AGPR form costs a v_accvgpr copy per
# accumulator register each time the vector ALUs touch a score tile.  The fp32 kernels (twice the
# operand registers, not the throughput path) are left to the default register assignment.
VGPR_FORM = ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]


def _flags(unit: str):
    return VGPR_FORM if "bf16" in unit else []


def _compile(unit: str, verbose: bool) -> str:
    src = os.path.join(CSRC, unit + ".hip")
    obj = os.path.join(OBJDIR, unit + ".o")
    cmd = BASE + _flags(unit) + (["-Rpass-analysis=kernel-resource-usage"] if verbose else []) + ["-c", src, "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed on {unit}.hip:\n{res.stderr[-4000:]}")
    if verbose:
        sys.stderr.write(res.stderr)
    return obj


def build(force: bool = True, verbose: bool = False) -> str:
    sources = [os.path.join(CSRC, u + ".hip") for u in UNITS]
    if not force and os.path.exists(LIB):
        newest = max(os.path.getmtime(f) for f in sources + HEADERS)
        if os.path.getmtime(LIB) >= newest:
            return LIB
    os.makedirs(OBJDIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(len(UNITS), os.cpu_count() or 1)) as pool:
        objs = list(pool.map(lambda u: _compile(u, verbose), UNITS))
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
