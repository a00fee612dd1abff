"""Builds libpbsa.so (HIP kernels + C ABI) in-tree for gfx950 with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libpbsa.so")
BUILD_DIR = os.path.join(ROOT, "_build")

# source file -> extra flags.  The coarse/update kernels implement arithmetic that is specified
# operation by operation, so they are compiled without contraction.
SOURCES = {
    "pbsa_api.hip": [],
    "pbsa_coarse.hip": ["-ffp-contract=off", "-fhip-fp32-correctly-rounded-divide-sqrt"],
    # the attention launch can carry the update's decisions (pbsa_plan_device.h): correctly rounded division for those
    "pbsa_attention.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1", "-fhip-fp32-correctly-rounded-divide-sqrt"],
    "pbsa_layout.hip": [],
    "pbsa_mass.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"],
    "pbsa_backward.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"],
}
COMMON = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden", "-Wall", "-Wno-unused-command-line-argument",
          # keep the compiler from forming packed-fp32 instructions
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-I", os.path.join(ROOT, "include"), "-I", CSRC]


# The attention, mass and backward kernels issue some matrix instructions as inline assembly with hand-placed wait
# states: the compiler these were checked with (every-element GPU tests of all <D, B> instances).  Another
# compiler may schedule around them differently: the build warns, and the GPU tests decide.
CHECKED_HIPCC = "7.2.26015"


def hipcc_version() -> str:
    out = subprocess.run(["hipcc", "--version"], check=True, capture_output=True, text=True).stdout
    for line in out.splitlines():
        if line.startswith("HIP version:"):
            return line.split(":", 1)[1].strip()
    return "unknown"


def _compile(name: str, flags, keep_asm: bool) -> str:
    obj = os.path.join(BUILD_DIR, name.replace(".hip", ".o"))
    cmd = ["hipcc", *COMMON, *flags, "-c", os.path.join(CSRC, name), "-o", obj]
    if keep_asm:
        cmd += ["-save-temps=obj"]
    subprocess.run(cmd, check=True, cwd=BUILD_DIR)
    return obj


def build(keep_asm: bool = False) -> str:
    os.makedirs(BUILD_DIR, exist_ok=True)
    ver = hipcc_version()
    if not ver.startswith(CHECKED_HIPCC):
        print(f"build.py: hipcc {ver} is not the checked {CHECKED_HIPCC}: run the GPU tests (pytest -m gpu) before "
              "trusting the inline-assembly kernels", file=sys.stderr)
    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        objs = list(ex.map(lambda kv: _compile(kv[0], kv[1], keep_asm), SOURCES.items()))
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], check=True)
    return LIB


if __name__ == "__main__":
    print(build(keep_asm="--asm" in sys.argv))
