"""CPU sanitizer builds (no GPU): the oracle's C++ and the library's host-only layer under
AddressSanitizer + UndefinedBehaviorSanitizer, and the host-side update's thread pool and grain
queue under ThreadSanitizer.  Each harness under tests/pins/ is compiled here into a temporary
directory and run; a sanitizer report or a failed check makes it exit non-zero."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PINS = os.path.join(ROOT, "tests", "pins")
CSRC = os.path.join(ROOT, "paper_2406_08334_amd", "csrc")
CLANG = "/opt/rocm/llvm/bin/clang++"
HIPCC = "/opt/rocm/bin/hipcc"
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1",
           TSAN_OPTIONS="halt_on_error=1")


def build_and_run(cmd, exe, tmp_path, timeout=600):
    res = subprocess.run(cmd, capture_output=True, text=True, cwd=tmp_path)
    noise = "is not a recognized feature for this target"
    assert res.returncode == 0, "\n".join(l for l in (res.stdout + res.stderr).splitlines() if noise not in l)[-4000:]
    run = subprocess.run([exe], capture_output=True, text=True, cwd=tmp_path, env=ENV, timeout=timeout)
    assert run.returncode == 0, (run.stdout + run.stderr)[-4000:]
    return run.stdout


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_sanitize")
    out = build_and_run(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                         "-ffp-contract=off", "-pthread", os.path.join(PINS, "oracle_sanitize.cpp"), "-o", exe], exe, tmp_path)
    assert "all checks held" in out


@pytest.mark.skipif(not os.path.exists(CLANG), reason="needs the ROCm clang++")
def test_host_update_thread_pool_under_thread_sanitizer(tmp_path):
    exe = str(tmp_path / "host_update_tsan")
    # the x86 clones are resolved by an ifunc that runs before the sanitizer's runtime is up: plain loops here
    out = build_and_run([CLANG, "-std=c++17", "-O1", "-g", "-fsanitize=thread", "-DPT_HOST_NO_CLONES", "-ffp-contract=off",
                         "-pthread", "-I", CSRC, os.path.join(PINS, "host_update_tsan.cpp"), "-o", exe], exe, tmp_path)
    assert "equal the serial pass" in out


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="needs hipcc")
def test_library_host_layer_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    """The library's own sources, host side instrumented (device code is built as usual and never runs)."""
    exe = str(tmp_path / "host_layer_sanitize")
    srcs = [os.path.join(CSRC, f) for f in sorted(os.listdir(CSRC)) if f.endswith(".hip")]
    cmd = [HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-Xarch_host", "-fsanitize=address", "-Xarch_host",
           "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined", "-ffp-contract=off", "-Xclang",
           "-target-feature", "-Xclang", "-packed-fp32-ops", "-I", os.path.join(ROOT, "include"), "-I", CSRC] + srcs + \
          [os.path.join(PINS, "host_layer_sanitize.cpp"), "-o", exe]
    out = build_and_run(cmd, exe, tmp_path)
    assert "all checks held" in out
