"""Address- and undefined-behaviour-sanitizer builds of the native code that runs on the host alone:
the C oracle (oracle/moe_oracle.c) and the control plane (csrc/governor.cpp, csrc/scheduler.cpp),
each driven by a small program under tests/native/ over heap buffers of exactly the documented
sizes.  (The host side of csrc/api.hip needs a device for everything but argument checks, which
the GPU tests cover through canaries instead.)  No GPU is needed."""
import os
import subprocess
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1", OMP_NUM_THREADS="2")


def _run(cmd_build, exe):
    r = subprocess.run(cmd_build, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    r = subprocess.run([exe], capture_output=True, text=True, env=ENV, timeout=600)
    assert r.returncode == 0, (r.stdout[-1000:], r.stderr[-3000:])
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr and "LeakSanitizer" not in r.stderr, r.stderr[-3000:]
    return r.stdout


def test_c_oracle_is_clean_under_asan_and_ubsan():
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "oracle_driver")
        out = _run(["gcc", "-std=c11", "-fopenmp", "-ffp-contract=off"] + SAN +
                   [os.path.join(ROOT, "oracle", "moe_oracle.c"), os.path.join(ROOT, "tests", "native", "asan_oracle_driver.c"),
                    "-lm", "-o", exe], exe)
        assert "oracle driver: ok" in out


def test_control_plane_is_clean_under_asan_and_ubsan():
    csrc = os.path.join(ROOT, "paper_2511_14102_amd", "csrc")
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "sched_driver")
        out = _run(["g++", "-std=c++17", "-I", os.path.join(ROOT, "include")] + SAN +
                   [os.path.join(csrc, "governor.cpp"), os.path.join(csrc, "scheduler.cpp"),
                    os.path.join(ROOT, "tests", "native", "asan_sched_driver.cpp"), "-o", exe], exe)
        assert "control-plane driver: ok" in out
