"""Host code of the executor and the search under sanitizers.

AddressSanitizer + UndefinedBehaviorSanitizer:

tests/sanitize/driver.cpp walks the C ABI without a GPU (descriptor loading, plan validation, Matrix_P -> edges, plan
<-> text, the search on random lookup tables, the model residue, the error paths of calls that need a device); the
kernels are replaced by geometry-only stubs.  The sanitizers apply to host code only: device code is compiled as usual.

ThreadSanitizer: tests/sanitize/tsan_driver.cpp runs the per-tenant issue threads (generation counters on the sync events,
fork / join of every round, sibling streams, the checking mode, the static-workspace entry point) on a HIP runtime made of
host code (tests/sanitize/stub_hip.cpp), which also checks the rule the threads exist to keep: no hipStreamWaitEvent is
issued before the hipEventRecord it belongs to.
"""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "..", "paper_2304_11745_amd", "csrc")


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not on PATH")
def test_abi_walk_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "san_driver")
    cmd = ["hipcc", "--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Xarch_host", "-fsanitize=address,undefined", "-Xarch_host", "-fno-sanitize-recover=undefined",
           "-x", "hip", os.path.join(CSRC, "executor.cpp"), os.path.join(CSRC, "search.cpp"),
           os.path.join(HERE, "sanitize", "stub_kernels.cpp"), os.path.join(HERE, "sanitize", "driver.cpp"), "-o", exe]
    built = subprocess.run(cmd, capture_output=True, text=True, timeout=600)
    assert built.returncode == 0, built.stderr[-4000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    ran = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
    assert ran.returncode == 0, (ran.stdout + ran.stderr)[-6000:]
    assert "all checks held" in ran.stdout


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not on PATH")
def test_issue_threads_are_race_free_and_never_wait_before_the_record(tmp_path):
    exe = str(tmp_path / "tsan_driver")
    cmd = ["hipcc", "--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Xarch_host", "-fsanitize=thread",
           "-x", "hip", os.path.join(CSRC, "executor.cpp"), os.path.join(CSRC, "search.cpp"),
           os.path.join(HERE, "sanitize", "stub_kernels.cpp"), os.path.join(HERE, "sanitize", "stub_hip.cpp"),
           os.path.join(HERE, "sanitize", "tsan_driver.cpp"), "-o", exe]
    built = subprocess.run(cmd, capture_output=True, text=True, timeout=600)
    assert built.returncode == 0, built.stderr[-4000:]
    env = dict(os.environ, TSAN_OPTIONS="halt_on_error=1:exitcode=66")
    ran = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
    assert ran.returncode == 0, (ran.stdout + ran.stderr)[-6000:]
    assert "none before its record" in ran.stdout
