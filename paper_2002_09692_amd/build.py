"""Builds libsaps.so (the HIP kernels and the C ABI of include/saps.h) for gfx950 with hipcc."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "csrc", "saps_api.hip")            # HIP kernels + round ABI
SRC_HOST = os.path.join(HERE, "csrc", "saps_select.cpp")     # host-only peer selection
DEPS = [SRC, SRC_HOST, os.path.join(HERE, "csrc", "saps_device.hpp"),
        os.path.join(os.path.dirname(HERE), "include", "saps.h"),
        os.path.join(os.path.dirname(HERE), "include", "saps_select.h")]
LIB = os.path.join(HERE, "libsaps.so")

HIPCC_FLAGS = [
    "-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-shared", "-Wall",
    # keep the compiler from forming packed fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def build(force: bool = True) -> str:
    """Compiles the library in-tree.  force=False skips the compile when the .so is newer than its sources."""
    if not force and os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(d) for d in DEPS):
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB + ".tmp.%d" % os.getpid()
    subprocess.run([hipcc, *HIPCC_FLAGS, SRC, SRC_HOST, "-o", tmp], check=True)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build())


NATIVE_TEST_SRC = os.path.join(os.path.dirname(HERE), "tests", "native", "abi_smoke.cpp")
NATIVE_TEST_BIN = os.path.join(os.path.dirname(HERE), "tests", "native", "abi_smoke.bin")


def build_native_test() -> str:
    """Compiles the stand-alone C++ user of the ABI (tests/native/abi_smoke.cpp) against the in-tree library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = NATIVE_TEST_BIN + ".tmp.%d" % os.getpid()
    subprocess.run([hipcc, "-O2", "--offload-arch=gfx950", "-std=c++17", NATIVE_TEST_SRC, "-L" + HERE, "-lsaps",
                    "-Wl,-rpath,$ORIGIN/../../paper_2002_09692_amd", "-o", tmp], check=True)
    os.replace(tmp, NATIVE_TEST_BIN)
    return NATIVE_TEST_BIN
