"""Builds tests/c_driver/abi_roundtrip: a caller of libadacomp's C ABI written in C++ with nothing
but the HIP runtime, checked against the CPU oracle, which is linked in (gcc, same options as the
oracle's own build).  Called from the repository's build entry point after libadacomp.so exists;
the GPU test only runs the result."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
EXE = os.path.join(HERE, "abi_roundtrip")


def build() -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    lib_dir = os.path.join(ROOT, "paper_1712_02679_amd")
    obj = os.path.join(HERE, "adacomp_oracle.o")
    subprocess.run(["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra", "-c",
                    "-o", obj, os.path.join(ROOT, "oracle", "adacomp_oracle.c")], check=True)
    res = subprocess.run([hipcc, "--offload-arch=gfx950", "-O2", "-std=c++17", "-Wall", "-Wextra",
                          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                          "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(ROOT, "oracle"),
                          "-x", "hip", os.path.join(HERE, "abi_roundtrip.cpp"), "-x", "none", obj,
                          "-o", EXE, "-L" + lib_dir, "-ladacomp", "-lm",
                          "-Wl,-rpath,$ORIGIN/../../paper_1712_02679_amd"],
                         capture_output=True, text=True)
    if res.returncode != 0:
        print(res.stdout)
        print(res.stderr)
        raise RuntimeError("building tests/c_driver/abi_roundtrip failed")
    os.remove(obj)
    return EXE


if __name__ == "__main__":
    print(build())
