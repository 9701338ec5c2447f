"""Builds libzi.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libzi.so")
SOURCES = ["zi_kernels.hip", "zi_api.hip", "zi_plan.hip", "zi_engine.hip", "zi_offload.hip", "zi_probe.hip"]

# -ffp-contract=off: the only fused multiply-adds are the ones the kernels write as fma.
# Packed fp32 instructions are switched off for the device code.
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off", "-fhip-fp32-correctly-rounded-divide-sqrt", "-fno-fast-math",
    "-fno-gpu-flush-denormals-to-zero",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def needs_build() -> bool:
    if not os.path.exists(LIB_PATH):
        return True
    t = os.path.getmtime(LIB_PATH)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + \
           [os.path.join(ROOT, "include", f) for f in ("zi.h", "zi_probe.h")]
    return any(os.path.getmtime(d) > t for d in deps)


# The host-CPU step is plain C++ with AVX2 / FMA / F16C intrinsics, built by the host compiler.
HOST_SOURCES = ["zi_cpu_step.cpp"]
HOST_FLAGS = ["-O3", "-std=c++17", "-fPIC", "-mavx2", "-mfma", "-mf16c", "-ffp-contract=off", "-fno-fast-math",
              "-Wall", "-Wextra", "-pthread"]


def build(force: bool = True, extra_flags=(), out: str | None = None) -> str:
    out = out or LIB_PATH
    if not force and out == LIB_PATH and not needs_build():
        return out
    objs = []
    for src in HOST_SOURCES:
        obj = os.path.join(HERE, "_" + os.path.splitext(src)[0] + ".o")
        subprocess.run(["g++", *HOST_FLAGS, "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-c", os.path.join(CSRC, src),
                        "-o", obj], check=True)
        objs.append(obj)
    cmd = [hipcc(), *HIPCC_FLAGS, *extra_flags, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           "-o", out, *[os.path.join(CSRC, s) for s in SOURCES], *["-Wl," + o for o in objs], "-pthread"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "packed-fp32-ops' is not a recognized feature"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if r.returncode != 0:
        sys.stderr.write(err + "\n")
        raise RuntimeError("hipcc failed: " + " ".join(cmd))
    if err.strip():
        sys.stderr.write(err + "\n")
    return out


if __name__ == "__main__":
    print(build(True))
