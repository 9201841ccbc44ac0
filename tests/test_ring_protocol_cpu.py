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
CSRC = os.path.join(ROOT, "paper_2604_17861_amd", "csrc")
SRC = [os.path.join(CSRC, "gpuos_runtime.cpp"), os.path.join(CSRC, "gpuos_jit.cpp"),
       os.path.join(HERE, "standin", "device_standin.cpp"), os.path.join(HERE, "standin", "ring_protocol_test.cpp")]


@pytest.mark.parametrize("sanitizer", ["none", "thread"])
def test_host_protocol_against_a_device_stand_in(sanitizer, tmp_path):
    exe = str(tmp_path / ("ring_" + sanitizer))
    flags = ["-std=c++17", "-O1", "-g", "-pthread", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-DGPUOS_CSRC_DIR=" + CSRC]
    if sanitizer == "thread":
        flags += ["-fsanitize=thread"]
    subprocess.run(["g++"] + flags + SRC + ["-ldl", "-o", exe], check=True, cwd=ROOT)
    recorder, record = str(tmp_path / "libroctx_recorder.so"), str(tmp_path / "markers.txt")
    subprocess.run(["gcc", "-shared", "-fPIC", "-O1", os.path.join(HERE, "standin", "roctx_recorder.c"), "-o", recorder], check=True)
    env = dict(os.environ, TSAN_OPTIONS="halt_on_error=1 exitcode=66 second_deadlock_stack=1",
               GPUOS_ROCTX_LIBRARY=recorder, ROCTX_RECORD=record)
    # The plain run compiles the programs it defines with the real run-time compiler and then finds that the
    # stand-in cannot load code objects: the fall-back to interpreted programs.  Under the sanitizer the
    # compiler (a large library that was not built for it) stays out.
    if sanitizer == "thread":
        env["GPUOS_JIT"] = "0"
    r = subprocess.run([exe], capture_output=True, text=True, timeout=600, env=env)
    print(r.stdout[-3000:], r.stderr[-6000:])
    assert r.returncode == 0, "exit %d" % r.returncode
    assert "all ok" in r.stdout and "ThreadSanitizer" not in r.stderr
    # only the context created with cfg.markers = 1 wrote markers: ranges are balanced and name the calls
    lines = open(record).read().splitlines()
    print("\n".join(lines))
    assert sum(l.startswith("push") for l in lines) == sum(l.startswith("pop") for l in lines) == 4
    want = ["mark gpuos: worker launched, 12 workgroups, ring of 16 slots", "mark gpuos register: op 7 impl 1 version 1 from ticket 0",
            "push gpuos_submit 5 tasks", "push gpuos_wait ticket 4", "mark gpuos swap: op 7 impl 2 version 2 from ticket 5",
            "push gpuos_stop_worker", "mark gpuos: worker launched again at ticket 5", "push gpuos_wait all"]
    it = iter(lines)
    assert all(any(l == w for l in it) for w in want), lines
