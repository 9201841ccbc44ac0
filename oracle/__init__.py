"""ctypes loader for the CPU oracle (TEST INFRASTRUCTURE ONLY).

Only tests/, the smoke check and the benchmark's cpu_baseline leg may import
this package; the product package never does.  The oracle is plain C++ built
with g++ (see build()); it takes the same task-descriptor arrays as the GPU
library, with HOST pointers in them.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "liboracle.so")

MODE_F64CORE = 0
MODE_F32LIBM = 1


def build(force=True):
    """Compile oracle.cpp into liboracle.so (host code only)."""
    src = os.path.join(_HERE, "oracle.cpp")
    if not force and os.path.exists(_SO) and os.path.getmtime(_SO) >= os.path.getmtime(src):
        return _SO
    cmd = ["g++", "-std=c++17", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
           "-Wall", "-Wextra", "-o", _SO, src]
    subprocess.run(cmd, check=True, cwd=_HERE)
    return _SO


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_SO):
            build()
        L = ctypes.CDLL(_SO)
        L.orc_validate.argtypes = [ctypes.c_void_p, ctypes.c_int]
        L.orc_validate.restype = ctypes.c_int
        L.orc_run_task.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int]
        L.orc_run_task.restype = ctypes.c_int
        L.orc_run_stream.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_int,
                                     ctypes.c_void_p]
        L.orc_run_stream.restype = ctypes.c_int64
        L.orc_sum_last_f64.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        L.orc_sum_last_f64.restype = ctypes.c_int
        L.orc_rowop_f64.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p]
        L.orc_rowop_f64.restype = ctypes.c_int
        L.orc_validate_program.argtypes = [ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint32]
        L.orc_validate_program.restype = ctypes.c_int
        L.orc_run_task_program.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint32, ctypes.c_int]
        L.orc_run_task_program.restype = ctypes.c_int
        L.orc_f16_to_f32.argtypes = [ctypes.c_uint16]
        L.orc_f16_to_f32.restype = ctypes.c_float
        L.orc_f32_to_f16.argtypes = [ctypes.c_float]
        L.orc_f32_to_f16.restype = ctypes.c_uint16
        L.orc_bf16_to_f32.argtypes = [ctypes.c_uint16]
        L.orc_bf16_to_f32.restype = ctypes.c_float
        L.orc_f32_to_bf16.argtypes = [ctypes.c_float]
        L.orc_f32_to_bf16.restype = ctypes.c_uint16
        L.orc_scalar_op.argtypes = [ctypes.c_int] + [ctypes.c_float] * 4 + [ctypes.c_int]
        L.orc_scalar_op.restype = ctypes.c_float
        L.orc_abi_layout.argtypes = [ctypes.c_void_p]
        L.orc_abi_layout.restype = None
        _lib = L
    return _lib


def abi_layout():
    out = np.zeros(8, dtype=np.uint32)
    lib().orc_abi_layout(out.ctypes.data)
    return out


def validate(tasks, i, impl):
    return lib().orc_validate(tasks.ctypes.data + i * tasks.dtype.itemsize, int(impl))


def run_task(tasks, i, impl, mode=MODE_F64CORE):
    """Run task i of a task array (host pointers inside)."""
    return lib().orc_run_task(tasks.ctypes.data + i * tasks.dtype.itemsize, int(impl), int(mode))


def run_stream(tasks, impls, mode=MODE_F64CORE, first=0, count=None, programs=None):
    """Run tasks[first:first+count] in order; returns the per-task status array.  programs: impl id
    -> (instruction array, n_inputs) for the tasks whose operator is a program."""
    n = len(tasks) - first if count is None else count
    impls = np.ascontiguousarray(impls, dtype=np.int32)
    assert len(impls) == len(tasks)
    status = np.zeros(n, dtype=np.int32)
    if not programs or not np.isin(impls[first: first + n], list(programs)).any():
        lib().orc_run_stream(tasks.ctypes.data + first * tasks.dtype.itemsize, n,
                             impls.ctypes.data + 4 * first, int(mode), status.ctypes.data)
        return status
    for k in range(n):
        i = first + k
        if int(impls[i]) in programs:
            code, nin = programs[int(impls[i])]
            status[k] = run_task_program(tasks, i, code, nin, mode)
        else:
            status[k] = run_task(tasks, i, impls[i], mode)
    return status


def validate_program(code, n_inputs):
    code = np.ascontiguousarray(code)
    return lib().orc_validate_program(code.ctypes.data, len(code), int(n_inputs))


def run_task_program(tasks, i, code, n_inputs, mode=MODE_F64CORE):
    """Run task i with the operator given as a program (instruction array of 8-byte records)."""
    code = np.ascontiguousarray(code)
    assert code.dtype.itemsize == 8
    return lib().orc_run_task_program(tasks.ctypes.data + i * tasks.dtype.itemsize, code.ctypes.data, len(code),
                                      int(n_inputs), int(mode))


def sum_last_f64(tasks, i, n_rows):
    s = np.zeros(n_rows, dtype=np.float64)
    l1 = np.zeros(n_rows, dtype=np.float64)
    rc = lib().orc_sum_last_f64(tasks.ctypes.data + i * tasks.dtype.itemsize, s.ctypes.data, l1.ctypes.data)
    if rc != 0:
        raise ValueError("orc_sum_last_f64 rc=%d" % rc)
    return s, l1


def rowop_f64(tasks, i, impl):
    """Unrounded fp64 results of a row operation (softmax family, layer norm) in the task's
    row-major shape."""
    t = tasks[i]
    shape = [int(x) for x in t["size"][: int(t["ndim"])]]
    y = np.zeros(shape, dtype=np.float64)
    rc = lib().orc_rowop_f64(tasks.ctypes.data + i * tasks.dtype.itemsize, int(impl), y.ctypes.data)
    if rc != 0:
        raise ValueError("orc_rowop_f64 rc=%d" % rc)
    return y
