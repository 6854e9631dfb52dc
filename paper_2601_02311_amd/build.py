"""Compiles the HIP library for gfx950 into ``paper_2601_02311_amd/libps_step.so``.

hipcc cross-compiles without a GPU.  Flags that matter for the numerics:
contraction off (each operator in the kernels is one rounded binary32
operation), IEEE-accurate fp32 division and square root, denormals kept.
Packed-fp32 instructions are disabled for the device pass.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libps_step.so")
SOURCES = ["ps_cost.cpp", "ps_step.cpp", "ps_arena.cpp", "ps_kernels.hip"]
HEADERS = ["ps_internal.h", "ps_kernel_templates.h"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off", "-fno-fast-math",
    "-fhip-fp32-correctly-rounded-divide-sqrt", "-fno-gpu-flush-denormals-to-zero",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


BUILD_ID = os.path.join(HERE, "libps_step.build_id")   # what the library was built from


def source_id() -> str:
    """Hash of everything the library is compiled from (sources, headers, flags)."""
    import hashlib
    h = hashlib.sha256(" ".join(FLAGS[:-4]).encode())
    deps = [os.path.join(CSRC, f) for f in SOURCES + HEADERS]
    deps.append(os.path.join(ROOT, "include", "ps_step.h"))
    for d in deps:
        with open(d, "rb") as f:
            h.update(os.path.basename(d).encode() + b"\0" + f.read())
    return h.hexdigest()


def stale() -> bool:
    """True when there is no library, or when it was built from other sources than the
    ones on disk now (compared by content, not by time stamp)."""
    if not os.path.exists(LIB) or not os.path.exists(BUILD_ID):
        return True
    with open(BUILD_ID) as f:
        return f.read().strip() != source_id()


def build(verbose: bool = False) -> str:
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = [HIPCC, *FLAGS, "-x", "hip", *[os.path.join(CSRC, s) for s in SOURCES], "-o", tmp]
    if verbose:
        print(" ".join(cmd), file=sys.stderr)
    sid = source_id()
    subprocess.run(cmd, check=True)
    os.replace(tmp, LIB)
    with open(BUILD_ID + ".tmp.%d" % os.getpid(), "w") as f:
        f.write(sid + "\n")
    os.replace(BUILD_ID + ".tmp.%d" % os.getpid(), BUILD_ID)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
