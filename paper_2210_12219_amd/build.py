"""Build step: compile csrc/*.hip for gfx950 into paper_2210_12219_amd/libppo.so with hipcc."""
from __future__ import annotations

import glob
import os
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
LIB = os.path.join(PKG, "libppo.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    "-fno-fast-math", "-ffp-contract=off", "-fhip-fp32-correctly-rounded-divide-sqrt",
    # small dynamically indexed register arrays (DP chain prefixes) must stay in VGPRs, not scratch
    "-mllvm", "-amdgpu-promote-alloca-to-vector-vgpr-ratio=2",
    # packed-FP32 forms are never wanted here (the path is integer/min/max work)
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def sources():
    return sorted(glob.glob(os.path.join(PKG, "csrc", "*.hip")))


def build(verbose: bool = False) -> str:
    """Always recompiles; returns the path of the shared library."""
    tmp = LIB + f".tmp{os.getpid()}"
    cmd = [HIPCC, *FLAGS, "-I", os.path.join(ROOT, "include"), "-I", os.path.join(PKG, "csrc"), "-o", tmp, *sources()]
    if verbose:
        print(" ".join(cmd), flush=True)
    try:
        subprocess.check_call(cmd)
        check_paired_kernel(verbose)
        os.replace(tmp, LIB)
    finally:
        if os.path.exists(tmp):
            os.remove(tmp)
    return LIB


def check_paired_kernel(verbose: bool = False) -> None:
    """The paired enumeration kernel keeps values in fixed registers between inline-assembly blocks and jumps to
    offsets computed from instruction sizes: verify both on the code the toolchain emitted (csrc/check_pair_code.py)."""
    import sys
    import tempfile
    src = os.path.join(PKG, "csrc", "ppo_paired.hip")
    with tempfile.TemporaryDirectory() as d:
        asm, obj = os.path.join(d, "paired.s"), os.path.join(d, "paired.elf")
        device_flags = [f for f in FLAGS if f not in ("-fPIC", "-shared")]
        subprocess.check_call([HIPCC, *device_flags, "-I", os.path.join(ROOT, "include"), "-I", os.path.join(PKG, "csrc"),
                               "--cuda-device-only", "-S", "-o", asm, src])
        clang = os.path.join(os.path.dirname(os.path.realpath(HIPCC)), "..", "llvm", "bin", "clang")
        if not os.path.exists(clang):
            clang = "/opt/rocm/llvm/bin/clang"
        subprocess.check_call([clang, "-x", "assembler", "-target", "amdgcn-amd-amdhsa", "-mcpu=gfx950", "-c", asm, "-o", obj])
        subprocess.check_call([sys.executable, os.path.join(PKG, "csrc", "check_pair_code.py"), asm, obj])
    # and the tables that steer the jumps: the kernel's own table builder, compiled for the host, walked through a
    # model of the generated code (csrc/check_pair_program.py)
    subprocess.check_call([sys.executable, os.path.join(PKG, "csrc", "check_pair_program.py"), "200"])


if __name__ == "__main__":
    print(build(verbose=True))
