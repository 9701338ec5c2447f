"""The library's host-only code under the compiler's sanitizers (CPU only, no GPU code involved).

tests/c/host_sanity.cpp exercises the host-CPU step, the chunk planner, the thread pool (memory and file
pieces), the parked stage threads and a model of the pinned ring's three-actor choreography; it is built
together with the host step and the oracle's C file, once with AddressSanitizer + UndefinedBehaviorSanitizer
and once with ThreadSanitizer, and must run clean."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2104_07857_amd", "csrc")


def _build_and_run(tmp_path, name, sanitize):
    if shutil.which("g++") is None or shutil.which("gcc") is None:
        pytest.skip("no host compiler")
    exe = str(tmp_path / name)
    oracle_o = str(tmp_path / (name + "_oracle.o"))
    common = ["-O1", "-g", "-fno-omit-frame-pointer", "-ffp-contract=off", "-fno-fast-math", "-mavx2", "-mfma", "-mf16c",
              "-fsanitize=" + sanitize]
    r = subprocess.run(["gcc", "-std=c11", *common, "-I", os.path.join(ROOT, "oracle"), "-c",
                        os.path.join(ROOT, "oracle", "zi_oracle.c"), "-o", oracle_o], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    r = subprocess.run(["g++", "-std=c++17", *common, "-Wall", "-Wextra", "-pthread",
                        "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-I", os.path.join(ROOT, "oracle"),
                        os.path.join(ROOT, "tests", "c", "host_sanity.cpp"), os.path.join(CSRC, "zi_cpu_step.cpp"),
                        oracle_o, "-o", exe, "-lm"], capture_output=True, text=True)
    if r.returncode != 0 and "cannot find -l" in r.stderr:
        pytest.skip("sanitizer runtime not installed: " + r.stderr.strip().splitlines()[-1])
    assert r.returncode == 0, r.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1",
               TSAN_OPTIONS="halt_on_error=1")
    run = subprocess.run([exe], capture_output=True, text=True, timeout=600, env=env)
    assert run.returncode == 0, f"{name} failed ({run.returncode}):\n{run.stdout}\n{run.stderr[-4000:]}"
    assert "host sanity ok" in run.stdout or "skipped" in run.stdout
    assert "ERROR: " not in run.stderr and "WARNING: ThreadSanitizer" not in run.stderr, run.stderr[-4000:]


def test_host_code_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    _build_and_run(tmp_path, "host_sanity_asan", "address,undefined")


def test_host_code_under_thread_sanitizer(tmp_path):
    _build_and_run(tmp_path, "host_sanity_tsan", "thread")
