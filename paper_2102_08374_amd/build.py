"""Compile the HIP library paper_2102_08374_amd/libintsgd.so for gfx950, in-tree."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libintsgd.so")
SOURCES = [os.path.join(CSRC, "intsgd_api.cpp"), os.path.join(CSRC, "intsgd_kernels.hip")]
HEADERS = [os.path.join(CSRC, "intsgd_internal.h"), os.path.join(ROOT, "include", "intsgd.h")]
SYMBOL_MAP = os.path.join(CSRC, "libintsgd.map")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # only the extern "C" entry points marked INTSGD_API are exported
    "-fvisibility=hidden", "-Wl,--version-script=" + SYMBOL_MAP,
    # IEEE arithmetic exactly as written: no contraction, fp32 denormals kept
    "-ffp-contract=off", "-fno-fast-math", "-fno-gpu-flush-denormals-to-zero",
    # packed fp32 instructions stay off on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(f) > t for f in SOURCES + HEADERS + [SYMBOL_MAP, os.path.abspath(__file__)])


def build(force: bool = True, extra_flags=()) -> str:
    if not force and not is_stale():
        return LIB
    tmp = LIB + ".tmp%d" % os.getpid()
    cmd = [HIPCC, *FLAGS, *extra_flags, "-x", "hip", *SOURCES, "-o", tmp]
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force=True, extra_flags=sys.argv[1:]))
