"""The host side of the queue protocol on the CPU: csrc/gpuos_runtime.cpp is compiled unchanged
against a host thread that stands in for the device (tests/standin/device_standin.cpp: it speaks
the protocol and executes nothing) and driven by tests/standin/ring_protocol_test.cpp, once
plainly and once under ThreadSanitizer: many producers on rings of 2, 8 and 64 slots, back-pressure,
non-blocking mode, swaps under load, the kill switch, shutdown with tasks in flight."""
import os
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = [os.path.join(ROOT, "paper_2604_17861_amd", "csrc", "gpuos_runtime.cpp"),
       os.path.join(HERE, "standin", "device_standin.cpp"), os.path.join(HERE, "standin", "ring_protocol_test.cpp")]


@pytest.mark.parametrize("sanitizer", ["none", "thread"])
def test_host_protocol_against_a_device_stand_in(sanitizer, tmp_path):
    exe = str(tmp_path / ("ring_" + sanitizer))
    flags = ["-std=c++17", "-O1", "-g", "-pthread", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include"]
    if sanitizer == "thread":
        flags += ["-fsanitize=thread"]
    subprocess.run(["g++"] + flags + SRC + ["-o", exe], check=True, cwd=ROOT)
    env = dict(os.environ, TSAN_OPTIONS="halt_on_error=1 exitcode=66 second_deadlock_stack=1")
    r = subprocess.run([exe], capture_output=True, text=True, timeout=600, env=env)
    print(r.stdout[-3000:], r.stderr[-6000:])
    assert r.returncode == 0, "exit %d" % r.returncode
    assert "all ok" in r.stdout and "ThreadSanitizer" not in r.stderr
