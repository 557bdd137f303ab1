"""The host-side C++ of the library (planner, online sampler) under AddressSanitizer +
UndefinedBehaviorSanitizer and under ThreadSanitizer: random graphs and batches, 1 / 3 / 8
sampler threads, both schedules, malformed input.  CPU only; the GPU code is not involved."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(ROOT, "paper_2602_21597_amd", "csrc")


@pytest.mark.parametrize("flags", ["-fsanitize=address,undefined", "-fsanitize=thread"])
def test_planner_and_sampler_under_sanitizers(tmp_path, flags):
    if shutil.which("g++") is None:
        pytest.skip("no g++")
    exe = str(tmp_path / "driver")
    cmd = ["g++", "-std=c++17", "-O1", "-g", flags, "-fno-omit-frame-pointer", "-I" + os.path.join(ROOT, "include"),
           "-I" + CSRC, os.path.join(HERE, "host_sanitize_driver.cpp"), os.path.join(CSRC, "planner.cpp"),
           os.path.join(CSRC, "sampler.cpp"), "-lpthread", "-o", exe]
    built = subprocess.run(cmd, capture_output=True, text=True, timeout=300)
    if built.returncode != 0 and ("cannot find -l" in built.stderr or "No such file" in built.stderr):
        pytest.skip("sanitizer runtime library not installed: " + built.stderr.strip().splitlines()[-1])
    assert built.returncode == 0, built.stderr[-4000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1")
    out = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
    if out.returncode != 0 and ("runtime does not come first" in out.stderr or "unexpected memory mapping" in out.stderr):
        pytest.skip("the sanitizer runtime cannot start in this environment: " + out.stderr.strip().splitlines()[0])
    assert out.returncode == 0, out.stdout[-2000:] + out.stderr[-4000:]
    assert "ok" in out.stdout.splitlines()[-1]
    assert "malformed: rc -1" in out.stdout and "range: rc -3" in out.stdout
