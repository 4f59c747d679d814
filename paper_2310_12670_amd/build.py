"""Compile libreft.so for gfx950 with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import re
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libreft.so")
SOURCES = ["reft_api.hip", "reft_kernels.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-Wall",
         # Packed-FP32 instruction selection off for every kernel in the library.  The feature
         # belongs to the gfx950 device pass, where it takes effect (a float2 multiply-add compiles
         # to v_pk_fma_f32 without it and to two v_fma_f32 with it).  hipcc hands the same -Xclang
         # options to its x86 host pass, which does not know the feature and prints "not a recognized
         # feature for this target (ignoring feature)" once per function it compiles: harmless,
         # and filtered from the build's output below.
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # per-kernel register counts, checked below
         "-Rpass-analysis=kernel-resource-usage"]

HOST_PASS_NOTE = "'-packed-fp32-ops' is not a recognized feature for this target"

# The write-burst kernels run two 5-wave workgroups per compute unit, all resident at once.  Measured
# on gfx950: with more than 128 vector registers per lane only one such workgroup fits (four waves
# of two workgroups can land on one SIMD: 4 x 128 = its 512 registers), the second half of the
# grid then runs after the first, and the bursts lose their timing.
BURST_KERNELS = ("k_gather_burst", "k_xor_contig_burst")
BURST_MAX_VGPRS = 128


def check_burst_registers(compiler_output: str) -> dict:
    """VGPR count per burst-kernel instantiation from the compiler's resource remarks; raises if
    one exceeds the residency limit or if no such kernel was reported."""
    counts = {}
    name = None
    for line in compiler_output.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            name = m.group(1)
            continue
        m = re.search(r"\bVGPRs: (\d+)", line)
        if m and name and any(k in name for k in BURST_KERNELS):
            counts[name] = int(m.group(1))
    if not counts:
        raise RuntimeError("no register report for the burst kernels in the compiler output")
    over = {n: v for n, v in counts.items() if v > BURST_MAX_VGPRS}
    if over:
        raise RuntimeError("burst kernels over %d VGPRs (one workgroup per compute unit only): %s"
                           % (BURST_MAX_VGPRS, over))
    return counts


def build(verbose: bool = False) -> str:
    cmd = ["hipcc", *FLAGS, "-o", LIB, *[os.path.join(CSRC, s) for s in SOURCES]]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout)
    counts = check_burst_registers(res.stdout)
    if verbose:
        # the resource remarks and the source lines they quote are not worth showing
        print("\n".join(l for l in res.stdout.splitlines()
                        if "remark:" not in l and not re.match(r"\s*\d*\s*\|", l)
                        and HOST_PASS_NOTE not in l))
        print("burst kernels: %d instantiations, at most %d VGPRs" % (len(counts), max(counts.values())))
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
