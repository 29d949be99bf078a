"""ThreadSanitizer over the host logic: pool.cpp, ctx.cpp and controller.cpp compiled for the CPU with
-fsanitize=thread and driven by tests/tsan_storm.cpp (two worker threads on one pool and one adjuster, a third
thread staging partitions).  No GPU code is built or run."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2504_19867_amd", "csrc")


def test_two_thread_storm_is_clean_under_thread_sanitizer(tmp_path):
    gxx = shutil.which("g++")
    if gxx is None or not os.path.isdir("/opt/rocm/include"):
        pytest.skip("needs g++ and the HIP headers")
    exe = str(tmp_path / "tsan_storm")
    cmd = [gxx, "-std=c++17", "-O1", "-g", "-fsanitize=thread", "-ffp-contract=off", "-D__HIP_PLATFORM_AMD__",
           "-I/opt/rocm/include", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           os.path.join(CSRC, "pool.cpp"), os.path.join(CSRC, "ctx.cpp"), os.path.join(CSRC, "controller.cpp"),
           os.path.join(ROOT, "tests", "tsan_storm.cpp"), "-o", exe, "-L/opt/rocm/lib", "-lamdhip64",
           "-Wl,-rpath,/opt/rocm/lib", "-lpthread"]
    build = subprocess.run(cmd, capture_output=True, text=True)
    if build.returncode != 0 and "tsan" in build.stderr.lower():
        pytest.skip("no ThreadSanitizer runtime for this compiler")
    assert build.returncode == 0, build.stderr[-2000:]
    env = dict(os.environ, TSAN_OPTIONS="halt_on_error=1 exitcode=66")
    run = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
    assert "ThreadSanitizer" not in run.stderr, run.stderr[-3000:]
    assert run.returncode == 0, (run.returncode, run.stdout[-500:], run.stderr[-2000:])
    assert "storm ok" in run.stdout
