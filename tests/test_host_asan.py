"""Memory safety of the kernels' indexing: the CPU build of the library (every kernel lane by lane, "device"
buffers as exact-size heap blocks) driven through the C ABI under AddressSanitizer and UBSan.  An index that
leaves its buffer -- which on the GPU is silent at best and a fault at worst -- stops the driver."""
import os
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(HERE, "hostmath", "asan_driver.cpp")
EXE = os.path.join(HERE, "hostmath", "asan_driver")


def _newest_source():
    csrc = os.path.join(ROOT, "paper_2602_12630_amd", "csrc")
    files = [SRC, os.path.join(ROOT, "include", "tc.h")] + [os.path.join(csrc, f) for f in os.listdir(csrc)]
    return max(os.path.getmtime(f) for f in files)


def test_kernels_stay_inside_their_buffers():
    if not os.path.exists(EXE) or os.path.getmtime(EXE) < _newest_source():
        cmd = ["g++", "-O1", "-g", "-std=c++17", "-DTC_HOST_EMU", "-DTC_FB_C=8", "-D_GLIBCXX_ASSERTIONS",
               "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-static-libasan", "-Wno-unknown-pragmas",
               "-o", EXE, SRC]
        built = subprocess.run(cmd, capture_output=True, text=True)
        err = built.stderr.lower()
        if built.returncode != 0 and "cannot find" in err and ("asan" in err or "ubsan" in err or "sanitize" in err):
            pytest.skip("the sanitizer runtimes are not installed")
        assert built.returncode == 0, built.stderr[-4000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([EXE], capture_output=True, text=True, env=env, timeout=900)
    if "ASan runtime does not come first" in run.stderr:
        pytest.skip("a preloaded library keeps the sanitizer runtime from starting here")
    assert run.returncode == 0, (run.stdout + run.stderr)[-6000:]
    assert "asan driver: ok" in run.stdout
