"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer — CPU only.

The oracle (oracle/saps_oracle.cpp) and the host-side peer selection (csrc/saps_select.cpp) are
rebuilt with -fsanitize=address,undefined and their CPU test suites are run against those builds in a
child process; any report (out-of-bounds access, signed overflow, misaligned load ...) aborts the child.
No GPU code is involved: the selector build contains no HIP code at all.
"""
import os
import subprocess
import sys
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g"]


def _asan_runtime():
    p = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not p or not os.path.isabs(p) or not os.path.exists(p):
        pytest.skip("no AddressSanitizer runtime for gcc in this image")
    return os.path.realpath(p)


def _child_env(asan, extra):
    env = dict(os.environ)
    # the sanitizer runtime has to be the first library of the (uninstrumented) interpreter; whatever is
    # already preloaded stays behind it
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"          # the interpreter itself never frees everything
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env.update(extra)
    return env


def test_oracle_pin_suite_under_asan_and_ubsan():
    asan = _asan_runtime()
    with tempfile.TemporaryDirectory() as tmp:
        lib = os.path.join(tmp, "liboracle_san.so")
        subprocess.run(["g++", "-O1", "-std=c++17", "-ffp-contract=off", "-mfma", "-shared", "-fPIC", *SAN,
                        os.path.join(ROOT, "oracle", "saps_oracle.cpp"), "-o", lib], check=True)
        env = _child_env(asan, {"SAPS_ORACLE_LIB": lib, "SAPS_ORACLE_MUTATION_RUN": "1"})
        files = ["test_oracle_mask.py", "test_oracle_round.py", "test_oracle_segments.py", "test_oracle_properties.py"]
        r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                            *[os.path.join(ROOT, "tests", f) for f in files]],
                           env=env, cwd=ROOT, capture_output=True, text=True, timeout=900)
        assert r.returncode == 0, f"exit {r.returncode}\n{r.stdout[-1500:]}\n{r.stderr[-3000:]}"
        assert "passed" in r.stdout


_SELECTOR_RUNNER = r"""
import ctypes, sys
import pytest
from paper_2002_09692_amd import binding
binding._lib = ctypes.CDLL(sys.argv[1])          # host-only build of the peer selection, instrumented
sys.exit(pytest.main(["-x", "-q", "-p", "no:cacheprovider", sys.argv[2]]))
"""


def test_peer_selection_suite_under_asan_and_ubsan():
    pytest.importorskip("torch")
    asan = _asan_runtime()
    with tempfile.TemporaryDirectory() as tmp:
        lib = os.path.join(tmp, "libselect_san.so")
        subprocess.run(["g++", "-O1", "-std=c++17", "-shared", "-fPIC", *SAN, "-I" + os.path.join(ROOT, "include"),
                        os.path.join(ROOT, "paper_2002_09692_amd", "csrc", "saps_select.cpp"), "-o", lib], check=True)
        r = subprocess.run([sys.executable, "-c", _SELECTOR_RUNNER, lib, os.path.join(ROOT, "tests", "test_selector.py")],
                           env=_child_env(asan, {}), cwd=ROOT, capture_output=True, text=True, timeout=900)
        assert r.returncode == 0, f"exit {r.returncode}\n{r.stdout[-1500:]}\n{r.stderr[-3000:]}"
        assert "passed" in r.stdout
