"""Operators defined at run time as NATIVE code (paper Sections 1.2 and 4.1): the programs of a
context are compiled with the HIP run-time compiler into a second resident worker kernel and the
dispatcher routes their tasks to it.  Checked against the oracle like every operator, against the
interpreter bit for bit, under load (a new program retires the previous generation of the kernel
while tasks are in flight) and across stop / start of the worker."""
import numpy as np
import pytest

from paper_2604_17861_amd import runtime as R
from paper_2604_17861_amd import streams as S
import parity_cases as C

pytestmark = pytest.mark.gpu
# two workgroups per compute unit for the library's worker: the run-time kernel takes the third place and the
# fourth stays free (beside the default three, programs are interpreted: see the last test)
CFG = dict(idle_exit_ms=20000, wait_timeout_ms=20000, workgroups_per_cu=2)


def _run(stream, **cfg):
    from gpu_helpers import DevicePools, run_stream
    dp = DevicePools(stream)
    with R.Runtime(0, **CFG, **cfg) as rt:
        rt.register_table(stream.table, stream.programs)
        live = rt.native_info()
        t0 = run_stream(stream, rt, dp)
        comps = rt.completions(t0, len(stream))
        assert rt.worker_alive()
        rt.stop_worker()
        info = rt.native_info()
    assert np.all(comps["status"] == 0), comps["status"][comps["status"] != 0][:10]
    return dp.download(), live, info


def test_native_programs_match_the_oracle_and_the_interpreter():
    """The operator-program parity stream (six programs; contiguous, row / column broadcast,
    transposed, strided and mixed-dtype operands; several chunks) through the native path: every
    task of a program was executed by the run-time kernel, the results meet the oracle's bars
    (programs of exactly rounded instructions bit-exact) and equal the interpreter's bit for bit."""
    from gpu_helpers import compare_with_oracle
    s = C.operator_programs()
    print("operator programs, native:", len(s), "tasks,", len(s.programs), "programs", flush=True)
    got, live, info = _run(s)
    print(live, info, flush=True)
    assert live["native"] == 1 and live["programs"] == len(s.programs) and live["generation"] == 1, live
    assert live["compiled"] + live["cache_hits"] == 1          # one kernel for all six programs, built at the first bind
    fake = s.materialize([1 << 20] * len(s.pools))             # any aligned addresses: only the chunk counts are wanted
    units = sum(R.task_plan(fake, i, _stand_in(s, i))[1] for i in range(len(s)))
    assert info["units"] == units, (info, units)               # every work unit of every program task ran natively
    stats = compare_with_oracle(s, got)
    print(stats, flush=True)
    print("operator programs, interpreted", flush=True)
    want, live2, info2 = _run(s, jit_mode=2)
    assert live2["native"] == 0 and info2["units"] == 0 and "switched off" in info2["why"]
    for k, (g, w) in enumerate(zip(got, want)):
        assert np.array_equal(np.asarray(g).view(np.uint8), np.asarray(w).view(np.uint8)), "pool %d: native and interpreted differ" % k


def _stand_in(s, i):
    """A built-in of the same arity and kind plans like the program (same paths, same chunking)."""
    nin = s.programs[int(s.impl_for()[i])][1]
    return {1: S.IMPL["RELU"], 2: S.IMPL["DIV"], 3: S.IMPL["FMA"]}[nin]


def test_new_program_under_load_brings_up_the_next_generation():
    """The paper's injection flow with native code: tasks of two logical operators are in flight; a
    program is defined and swapped in for the first (the run-time kernel is compiled and launched
    while the worker runs), later a second program for the other operator: the kernel that holds
    one program drains and leaves, one that holds both takes over, and nothing stops.  Every task's
    result is the one of the version it recorded."""
    from gpu_helpers import DevicePools, compare_with_oracle
    s = S.config1(n_tasks=6000, numel=4096, seed=11)
    s.tasks["op_id"][1::2] = S.OP["MUL"]                       # odd tasks multiply
    dp = DevicePools(s)
    p1 = S.program(("ADD", 4, 0, 1), ("MUL", 0, 4, 4), ("IMM", 5, 0.5), ("SUB", 0, 0, 5))     # (x + y)^2 - 0.5
    p2 = S.program(("MUL", 4, 0, 1), ("ABS", 4, 4), ("SQRT", 0, 4))                           # sqrt|x y|
    with R.Runtime(0, **CFG) as rt:
        rt.register_table(s.table)
        rt.submit(dp.tasks, 0, 2000)
        i1 = rt.define_program(p1, 2)
        assert rt.native_info()["native"] == 0                 # defined, not bound: nothing compiled yet
        v1 = rt.swap_op(S.OP["ADD"], i1)                       # compiles and launches generation 1 under load
        n1 = rt.native_info()
        rt.submit(dp.tasks, 2000, 2000)
        i2 = rt.define_program(p2, 2)
        v2 = rt.swap_op(S.OP["MUL"], i2)                       # generation 1 drains and leaves, generation 2 holds both programs
        n2 = rt.native_info()
        rt.submit(dp.tasks, 4000, 2000)
        rt.wait()
        comps = rt.completions(0, 6000)
        assert rt.worker_alive()
        rt.stop_worker()
        n3 = rt.native_info()
    print(n1, n2, n3, flush=True)
    assert (i1, i2, v1, v2) == (S.PROGRAM_BASE, S.PROGRAM_BASE + 1, 2, 2)
    assert n1["native"] == 1 and n1["generation"] == 1 and n1["programs"] == 1
    assert n2["native"] == 1 and n2["generation"] == 2 and n2["programs"] == 2
    assert np.all(comps["status"] == 0)
    ver = comps["op_version"]
    add, mul = s.tasks["op_id"] == S.OP["ADD"], s.tasks["op_id"] == S.OP["MUL"]
    # (a task submitted before a swap and dequeued after it may record either version)
    assert np.all(ver[2000:][add[2000:]] == 2) and np.all(ver[4000:] == 2) and np.all(ver[:2000][mul[:2000]] == 1)
    assert set(np.unique(ver)) == {1, 2}
    assert n3["units"] == int((ver == 2).sum())                # exactly the tasks that recorded a program's version ran natively
    s.swaps = [(2000, S.OP["ADD"], i1), (4000, S.OP["MUL"], i2)]
    s.programs = {i1: (p1, 2), i2: (p2, 2)}
    stats = compare_with_oracle(s, dp.download(), versions=ver)
    assert stats["max_ulp"] == 0


def test_native_kernel_comes_back_after_stop_start_and_idle_exit():
    """Stop / start of the worker (handing the GPU over and taking it back) and the idle exit take
    the run-time kernel along: program tasks before, between and after are executed, natively again
    once it is back."""
    from gpu_helpers import DevicePools, compare_with_oracle
    import time
    s = S.config1(n_tasks=3000, numel=2048, seed=12)
    dp = DevicePools(s)
    p1 = S.program(("SUB", 4, 0, 1), ("MUL", 0, 4, 4))                                        # (x - y)^2
    with R.Runtime(0, **CFG) as warm:                          # compile once, so that the context with the short idle limit
        warm.register_table({S.OP["ADD"]: warm.define_program(p1, 2)})     # below finds the kernel in the process's cache
        assert warm.native_info()["compiled"] == 1
    with R.Runtime(0, idle_exit_ms=300, wait_timeout_ms=20000, workgroups_per_cu=2) as rt:
        i1 = rt.define_program(p1, 2)
        rt.register_table({S.OP["ADD"]: i1})
        assert rt.native_info()["native"] == 1
        rt.submit(dp.tasks, 0, 1000)
        rt.wait()
        rt.stop_worker()
        assert rt.native_info()["units"] == 1000
        rt.start_worker()
        assert rt.native_info()["native"] == 1
        rt.submit(dp.tasks, 1000, 1000)
        rt.wait()
        time.sleep(0.8)                                        # the worker leaves by itself ...
        assert not rt.worker_alive()
        rt.start_worker()                                      # ... and both kernels are launched again
        assert rt.native_info()["native"] == 1
        rt.submit(dp.tasks, 2000, 1000)
        rt.wait()
        comps = rt.completions(0, 3000)
        rt.stop_worker()
        info = rt.native_info()
    assert np.all(comps["status"] == 0) and info["units"] == 3000 and info["generation"] == 1 and info["cache_hits"] == 1, info
    s.table = {S.OP["ADD"]: i1}
    s.programs = {i1: (p1, 2)}
    stats = compare_with_oracle(s, dp.download())
    assert stats["max_ulp"] == 0


def test_beside_the_default_worker_programs_are_interpreted_unless_the_caller_fills_the_compute_units():
    """Four workgroups fit a compute unit.  With the default three of the library's worker a run-time
    kernel would leave no place for anybody else's kernels, so none is brought up and the reason is
    reported; naming jit_workgroups_per_cu takes the last place knowingly."""
    p1 = S.program(("SUB", 4, 0, 1), ("MUL", 0, 4, 4))
    with R.Runtime(0, idle_exit_ms=20000, wait_timeout_ms=20000) as rt:
        rt.register_table({S.OP["ADD"]: rt.define_program(p1, 2)})
        info = rt.native_info()
        assert info["native"] == 0 and info["compiled"] == 0 and "free" in info["why"], info
    with R.Runtime(0, idle_exit_ms=20000, wait_timeout_ms=20000, jit_workgroups_per_cu=1) as rt:
        rt.register_table({S.OP["ADD"]: rt.define_program(p1, 2)})
        info = rt.native_info()
        assert info["native"] == 1 and info["workgroups"] == int(R.device_info(0)["compute_units"]), info
