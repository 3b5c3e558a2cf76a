"""Host-side sanitizer builds (CPU only).

The CPU oracle, and the C-ABI layer of the library compiled against a stand-in HIP runtime
(tests/hostbuild/hip/hip_runtime.h: device memory is host memory, kernel launches are logged and
checked but run nothing), are built with AddressSanitizer + UndefinedBehaviorSanitizer and, for
the oracle's worker threads, ThreadSanitizer, and run through short drivers.  A driver returns 0
only if every call behaved as documented; a sanitizer report aborts it with a non-zero status.
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HOSTBUILD = os.path.join(ROOT, "tests", "hostbuild")
CSRC = os.path.join(ROOT, "paper_2507_17346_amd", "csrc")
ASAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan"]
COMMON = ["g++", "-std=c++17", "-O1", "-g", "-ffp-contract=off", "-pthread"]
ENV = {**os.environ, "ASAN_OPTIONS": "detect_leaks=1:abort_on_error=0", "UBSAN_OPTIONS": "print_stacktrace=1",
       "LD_PRELOAD": ""}


def build_and_run(tmp_path, name, flags, sources):
    if shutil.which("g++") is None:
        pytest.skip("no host compiler")
    exe = str(tmp_path / name)
    subprocess.check_call([*COMMON, *flags, *sources, "-o", exe])
    run = subprocess.run([exe], env=ENV, capture_output=True, text=True, timeout=600)
    assert run.returncode == 0, run.stdout[-4000:] + run.stderr[-8000:]
    assert "ok" in run.stdout
    assert "runtime error" not in run.stderr and "Sanitizer" not in run.stderr, run.stderr[-8000:]


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    build_and_run(tmp_path, "oracle_asan", ASAN,
                  [os.path.join(ROOT, "oracle", "ddef_oracle.cpp"), os.path.join(HOSTBUILD, "oracle_driver.cpp")])


def test_oracle_threads_under_thread_sanitizer(tmp_path):
    build_and_run(tmp_path, "oracle_tsan", ["-fsanitize=thread"],
                  [os.path.join(ROOT, "oracle", "ddef_oracle.cpp"), os.path.join(HOSTBUILD, "oracle_driver.cpp")])


def test_c_abi_layer_and_deco_under_sanitizers_with_injected_failures(tmp_path):
    """State machine, argument checks, getter and setter sizes, DeCo / look-up table / timing model,
    and the lazy set-ups (prefetch stream and buffer, sample buffers, candidate and message rows)
    with each allocation, stream or event failing in turn: the failure is reported, nothing leaks,
    nothing is launched on a null buffer, and the next call recovers."""
    includes = ["-I", HOSTBUILD, "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    build_and_run(tmp_path, "api_asan", [*ASAN, *includes],
                  ["-x", "c++", os.path.join(CSRC, "ddef_api.hip"), os.path.join(CSRC, "ddef_deco.cpp"),
                   os.path.join(HOSTBUILD, "api_driver.cpp")])
