"""Compile the HIP sources under csrc/ into lib/libw4a16.so for gfx950 (hipcc cross-compiles
without a GPU).  `python -m paper_2505_22179_amd.build` rebuilds unconditionally."""
from __future__ import annotations

import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIBDIR = os.path.join(HERE, "lib")
LIB = os.path.join(LIBDIR, "libw4a16.so")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")

# packed fp32 VALU instructions are switched off for every kernel in this library
HIPCC_FLAGS = ["-O3", "--offload-arch=gfx950", "-fPIC", "-std=c++17",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-mllvm", "-amdgpu-mfma-vgpr-form",   # MFMA results feed VALU scale folds: keep them in VGPRs
               "-Wall", "-Wno-unused-function", "-I" + INCLUDE]


def sources() -> list[str]:
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = sources() + glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(INCLUDE, "*.h"))
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = True, extra_flags: list[str] | None = None) -> str:
    if not force and not stale():
        return LIB
    os.makedirs(LIBDIR, exist_ok=True)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + (extra_flags or []) + ["-shared", "-o", LIB] + sources()
    proc = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(ln for ln in proc.stderr.splitlines() if noise not in ln)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if err.strip():
        print(err)
    return LIB


if __name__ == "__main__":
    print(build())
