"""Compile the HIP library for gfx950 into paper_2601_18383_amd/libdynts.so (in-tree)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "csrc", "dynts.hip")
LIB = os.path.join(HERE, "libdynts.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-mllvm", "-amdgpu-mfma-vgpr-form",   # MFMA results straight into arch VGPRs (no AGPR copies)
         "-Xarch_device", "-fno-honor-nans",   # device code only: no canonicalising v_max before every fmaxf
         "-Wall", "-Wno-unused-function"]


def sources():
    d = os.path.join(HERE, "csrc")
    return [os.path.join(d, f) for f in sorted(os.listdir(d))] + [os.path.join(HERE, "..", "include", "dynts.h")]


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(s) > t for s in sources())


def build(force: bool = True, extra=()) -> str:
    if not force and not is_stale():
        return LIB
    cmd = [HIPCC] + FLAGS + list(extra) + ["-o", LIB, SRC]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
