"""AddressSanitizer + UndefinedBehaviorSanitizer over the host code, on the CPU.

Builds the oracle (oracle/intsgd_oracle.cpp) and the library (csrc/intsgd_api.cpp's
validation, tiling and layout paths; the kernels are compiled as usual) with
-fsanitize=address,undefined -fno-sanitize-recover, then runs the oracle's pins and the
boundary checks through these builds in a child process.  Any report aborts the child.
GPU code is not sanitized (not available on the test machines).
"""
import glob
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLANG = "/opt/rocm/llvm/bin/clang++"
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all", "-shared-libasan", "-g"]


def _asan_runtime():
    hits = glob.glob("/opt/rocm/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
    return hits[0] if hits else None


@pytest.mark.timeout(900)
def test_pins_and_boundary_checks_under_asan_and_ubsan(tmp_path):
    rt = _asan_runtime()
    if rt is None or not os.path.exists(CLANG) or shutil.which(HIPCC) is None:
        pytest.skip("no clang sanitizer runtime / hipcc in this image")
    csrc = os.path.join(ROOT, "paper_2102_08374_amd", "csrc")
    oracle_lib = str(tmp_path / "liboracle_intsgd_san.so")
    subprocess.check_call([CLANG, "-O1", "-std=c++17", "-ffp-contract=off", "-fno-fast-math", *SAN,
                           "-shared", "-fPIC", os.path.join(ROOT, "oracle", "intsgd_oracle.cpp"),
                           "-o", oracle_lib])
    lib = str(tmp_path / "libintsgd.so")
    host_san = [f for flag in SAN for f in ("-Xarch_host", flag)]     # host pass only
    subprocess.check_call(
        [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fvisibility=hidden",
         "-Wl,--version-script=" + os.path.join(csrc, "libintsgd.map"),
         "-ffp-contract=off", "-fno-fast-math", "-fno-gpu-flush-denormals-to-zero",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", *host_san,
         "-I", os.path.join(ROOT, "include"), "-I", csrc, "-x", "hip",
         os.path.join(csrc, "intsgd_api.cpp"), os.path.join(csrc, "intsgd_kernels.hip"), "-o", lib],
        stderr=subprocess.DEVNULL)
    env = dict(os.environ)
    # the sanitizer runtime has to be loaded before the (uninstrumented) interpreter's libraries;
    # whatever the environment already preloads stays in place behind it
    env["LD_PRELOAD"] = rt + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["INTSGD_LIBRARY"] = lib
    env["INTSGD_ORACLE_LIBRARY"] = oracle_lib
    # not run in the child: the two checks that link or inspect the in-tree build itself
    cmd = [sys.executable, "-m", "pytest", "-q", "-x", "-p", "no:cacheprovider",
           os.path.join(ROOT, "tests", "test_oracle_pins.py"),
           os.path.join(ROOT, "tests", "test_boundary_host.py"),
           "-k", "not links and not exported"]
    out = subprocess.run(cmd, env=env, cwd=ROOT, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
    text = out.stdout.decode(errors="replace")
    assert out.returncode == 0, text[-4000:]
    assert " passed" in text and "runtime error" not in text and "AddressSanitizer" not in text, text[-4000:]
