"""Thin ctypes binding of include/gpuos.h: same names, argument marshalling only.

Every step of the hot path runs in the HIP library.  There is no CPU fallback: if libgpuos.so is
missing or fails to load, importing a symbol raises.  Tensor memory and streams come from
PyTorch (or any other allocator); the binding only passes raw device addresses through.

While a Runtime is alive its persistent worker kernel is resident on the GPU.  Do not call
torch.cuda.synchronize() (hipDeviceSynchronize waits for that kernel too) before shutdown();
synchronize the stream you are using instead, e.g. torch.cuda.current_stream().synchronize().
"""
import atexit
import ctypes
import os
import weakref

import numpy as np

from . import streams as S

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgpuos.so")

OK, E_INVAL, E_FULL, E_BADOP, E_TIMEOUT, E_DEAD, E_HIP, E_NOMEM, E_VERSION = 0, -1, -2, -3, -4, -5, -6, -7, -8
ALL = (1 << 64) - 1
MAX_OPS = 256


class Config(ctypes.Structure):
    _fields_ = [("device", ctypes.c_int32), ("threads_per_workgroup", ctypes.c_uint32),
                ("workgroups_per_cu", ctypes.c_uint32), ("nonblocking_submit", ctypes.c_uint32),
                ("harvester_thread", ctypes.c_uint32), ("defer_op_check", ctypes.c_uint32),
                ("idle_exit_ms", ctypes.c_uint32), ("wait_timeout_ms", ctypes.c_uint32),
                ("completion_log", ctypes.c_uint32), ("chunk_elems", ctypes.c_uint32),
                ("push_ring", ctypes.c_uint32), ("trace_entries", ctypes.c_uint32),
                ("markers", ctypes.c_uint32), ("phase_timers", ctypes.c_uint32), ("dep_wait_us", ctypes.c_uint32),
                ("jit_mode", ctypes.c_uint32), ("jit_workgroups_per_cu", ctypes.c_uint32), ("reserved", ctypes.c_uint32 * 1)]


class QueueState(ctypes.Structure):
    _fields_ = [("head_submitted", ctypes.c_uint64), ("tail_published", ctypes.c_uint64),
                ("claimed", ctypes.c_uint64), ("completed", ctypes.c_uint64),
                ("heartbeat", ctypes.c_uint64), ("capacity", ctypes.c_uint32),
                ("workgroups", ctypes.c_uint32), ("push_ring", ctypes.c_uint32), ("reserved", ctypes.c_uint32)]


class GpuosError(RuntimeError):
    def __init__(self, status, what=""):
        self.status = status
        msg = "%s: %s (%d)" % (what, strerror(status), status)
        if status == E_HIP:
            msg += " [" + last_hip_error() + "]"
        super().__init__(msg)


_lib = None


def lib():
    """Load libgpuos.so (built in-tree by paper_2604_17861_amd.build).  Raises if it is absent."""
    global _lib
    if _lib is not None:
        return _lib
    try:
        # PyTorch ships its own copy of the HIP runtime.  If this library were loaded first it would
        # bring in the system copy, and the process would end up with two runtimes that do not see
        # each other's devices and streams.  Loading torch first makes both use the same one.
        import torch  # noqa: F401
    except ImportError:
        pass
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            LIB_PATH + " is not built; run `python -m paper_2604_17861_amd.build` (there is no CPU fallback)")
    L = ctypes.CDLL(LIB_PATH)
    vp, u32, u64, i32 = ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint64, ctypes.c_int32
    P = ctypes.POINTER
    sig = {
        "gpuos_default_config": (None, [P(Config)]),
        "gpuos_init": (ctypes.c_int, [P(vp), u32, P(Config)]),
        "gpuos_init_static": (ctypes.c_int, [P(vp), u32, P(Config), vp, u64, vp]),
        "gpuos_register_op": (ctypes.c_int, [vp, u32, u32, P(u32)]),
        "gpuos_swap_op": (ctypes.c_int, [vp, u32, u32, P(u32)]),
        "gpuos_submit": (ctypes.c_int, [vp, vp, u32, P(u64)]),
        "gpuos_submit_flush": (ctypes.c_int, [vp, vp, u32, P(u64)]),
        "gpuos_flush": (ctypes.c_int, [vp]),
        "gpuos_wait": (ctypes.c_int, [vp, u64, u64]),
        "gpuos_get_completions": (ctypes.c_int, [vp, u64, u32, vp]),
        "gpuos_peek_queue": (ctypes.c_int, [vp, P(QueueState)]),
        "gpuos_worker_alive": (ctypes.c_int, [vp]),
        "gpuos_set_yield_every": (ctypes.c_int, [vp, u32]),
        "gpuos_shutdown": (ctypes.c_int, [vp]),
        "gpuos_stop_worker": (ctypes.c_int, [vp]),
        "gpuos_start_worker": (ctypes.c_int, [vp]),
        "gpuos_worker_elapsed_ms": (ctypes.c_int, [vp, P(ctypes.c_float)]),
        "gpuos_worker_stats": (ctypes.c_int, [vp, vp]),
        "gpuos_run_serial": (ctypes.c_int, [vp, vp, u32, vp]),
        "gpuos_launch_per_op": (ctypes.c_int, [i32, vp, u32, vp, i32, vp, P(ctypes.c_double)]),
        "gpuos_task_bytes": (ctypes.c_int, [vp, u32, P(u64)]),
        "gpuos_task_plan": (ctypes.c_int, [vp, u32, vp]),
        "gpuos_device_info": (ctypes.c_int, [i32, vp, vp, u32]),
        "gpuos_define_program": (ctypes.c_int, [vp, vp, u32, u32, P(u32)]),
        "gpuos_native_info": (ctypes.c_int, [vp, vp, vp, u32]),
        "gpuos_submit_from_threads": (ctypes.c_int, [vp, vp, u32, u32, u32, u32, P(ctypes.c_double)]),
        "gpuos_get_trace": (ctypes.c_int, [vp, u64, u32, vp]),
        "gpuos_op_counts": (ctypes.c_int, [vp, vp]),
        "gpuos_trace_origin": (ctypes.c_int, [vp, P(u64)]),
        "gpuos_kill_op": (ctypes.c_int, [vp, u32, P(u32)]),
        "gpuos_audit_log": (ctypes.c_int, [vp, u64, u32, vp, P(u64)]),
        "gpuos_strerror": (ctypes.c_char_p, [ctypes.c_int]),
        "gpuos_last_hip_error": (ctypes.c_char_p, []),
        "gpuos_abi_layout": (None, [vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)          # AttributeError if the library does not export it
        fn.restype = res
        fn.argtypes = args
    _lib = L
    return L


EXPORTS = ["gpuos_default_config", "gpuos_init", "gpuos_init_static", "gpuos_register_op", "gpuos_swap_op", "gpuos_submit", "gpuos_submit_flush",
           "gpuos_flush", "gpuos_wait", "gpuos_get_completions", "gpuos_peek_queue",
           "gpuos_worker_alive", "gpuos_set_yield_every", "gpuos_shutdown", "gpuos_stop_worker", "gpuos_start_worker",
           "gpuos_worker_elapsed_ms", "gpuos_worker_stats", "gpuos_run_serial", "gpuos_launch_per_op", "gpuos_task_bytes", "gpuos_task_plan", "gpuos_device_info", "gpuos_define_program", "gpuos_native_info", "gpuos_submit_from_threads", "gpuos_get_trace", "gpuos_op_counts",
           "gpuos_trace_origin", "gpuos_kill_op", "gpuos_audit_log", "gpuos_strerror",
           "gpuos_last_hip_error", "gpuos_abi_layout"]


STATIC_MAX_CAPACITY = 1024


def static_host_bytes(capacity):
    """GPUOS_STATIC_HOST_BYTES(capacity) of include/gpuos.h."""
    return 65536 + 512 * int(capacity)


def strerror(status):
    return lib().gpuos_strerror(int(status)).decode()


def last_hip_error():
    return lib().gpuos_last_hip_error().decode()


def abi_layout():
    out = np.zeros(8, dtype=np.uint32)
    lib().gpuos_abi_layout(out.ctypes.data)
    return out


TRACE_DT = np.dtype([("ticket", "<u8"), ("t_dequeue", "<u8"), ("t_start", "<u8"), ("t_done", "<u8"),
                     ("op_version", "<u4"), ("op_id", "<u2"), ("status", "i1"), ("reserved", "u1"),
                     ("nchunks", "<u4"), ("workgroup", "<u4")])
assert TRACE_DT.itemsize == 48
AUDIT_DT = np.dtype([("t_ns", "<u8"), ("head_ticket", "<u8"), ("kind", "<u4"), ("op_id", "<u4"), ("impl_id", "<u4"),
                     ("version", "<u4"), ("n_instr", "<u4"), ("n_inputs", "<u4"), ("code_hash", "<u8")])
assert AUDIT_DT.itemsize == 48
AUDIT_REGISTER, AUDIT_SWAP, AUDIT_KILL, AUDIT_DEFINE_PROGRAM = 1, 2, 3, 4


def device_info(device=0):
    """What the HIP runtime reports for `device` (gpuos_device_info)."""
    out = (ctypes.c_uint64 * 8)()
    name = ctypes.create_string_buffer(128)
    _check(lib().gpuos_device_info(int(device), out, name, 128), "gpuos_device_info")
    keys = ("compute_units", "core_clock_khz", "memory_clock_khz", "memory_bus_bits", "memory_bytes", "l2_bytes",
            "lds_bytes_per_workgroup", "wavefront")
    d = {k: int(v) for k, v in zip(keys, out)}
    d["name"] = name.value.decode()
    return d


def default_config():
    cfg = Config()
    lib().gpuos_default_config(ctypes.byref(cfg))
    return cfg


def _check(rc, what):
    if rc != OK:
        raise GpuosError(rc, what)
    return rc


def _tasks_ptr(tasks, first=0):
    assert tasks.dtype == S.TASK_DT and tasks.flags["C_CONTIGUOUS"]
    return tasks.ctypes.data + first * S.TASK_DT.itemsize


_live = weakref.WeakSet()


class Runtime:
    """One GPUOS context: gpuos_init ... gpuos_shutdown."""

    def __init__(self, queue_capacity=0, static=None, **cfg_fields):
        """gpuos_init; with static=(host_block_address, host_bytes, stream_handle): gpuos_init_static,
        the context that allocates nothing (the caller owns the block and the stream)."""
        L = lib()
        cfg = default_config()
        for k, v in cfg_fields.items():
            if not hasattr(cfg, k):
                raise TypeError("unknown config field " + k)
            setattr(cfg, k, v)
        self._ctx = ctypes.c_void_p()
        if static is None:
            _check(L.gpuos_init(ctypes.byref(self._ctx), queue_capacity, ctypes.byref(cfg)), "gpuos_init")
        else:
            block, nbytes, stream = static
            _check(L.gpuos_init_static(ctypes.byref(self._ctx), queue_capacity, ctypes.byref(cfg), block, nbytes, stream),
                   "gpuos_init_static")
        self.cfg = cfg
        _live.add(self)

    # -- operator table ------------------------------------------------------
    def register_op(self, op_id, impl_id):
        v = ctypes.c_uint32()
        _check(lib().gpuos_register_op(self._ctx, op_id, impl_id, ctypes.byref(v)), "gpuos_register_op")
        return v.value

    def swap_op(self, op_id, impl_id):
        v = ctypes.c_uint32()
        _check(lib().gpuos_swap_op(self._ctx, op_id, impl_id, ctypes.byref(v)), "gpuos_swap_op")
        return v.value

    def define_program(self, code, n_inputs):
        """gpuos_define_program: code is an array of 8-byte instructions {op, dst, a, b, imm}
        (streams.program assembles one); returns the implementation id to register / swap in."""
        code = np.ascontiguousarray(code)
        assert code.dtype.itemsize == 8
        v = ctypes.c_uint32()
        _check(lib().gpuos_define_program(self._ctx, code.ctypes.data, len(code), int(n_inputs), ctypes.byref(v)),
               "gpuos_define_program")
        return v.value

    def native_info(self):
        """gpuos_native_info: whether operator programs are served as native code, and by what."""
        out = (ctypes.c_uint64 * 8)()
        why = ctypes.create_string_buffer(512)
        _check(lib().gpuos_native_info(self._ctx, out, why, 512), "gpuos_native_info")
        keys = ("native", "generation", "programs", "compiled", "cache_hits", "units", "compile_us", "workgroups")
        d = {k: int(v) for k, v in zip(keys, out)}
        d["why"] = why.value.decode()
        return d

    def register_table(self, table, programs=None):
        """Bind every logical op of `table`.  programs: impl id -> (code, n_inputs) for the table's
        program entries; they are defined first, in id order, and must receive those ids."""
        for impl in sorted(programs or {}):
            code, nin = programs[impl]
            got = self.define_program(code, nin)
            if got != impl:
                raise ValueError("program defined as impl %d, the table expects %d" % (got, impl))
        for op, impl in table.items():
            self.register_op(op, impl)

    # -- submission ----------------------------------------------------------
    def submit(self, tasks, first=0, count=None, flush=True, check=True):
        """gpuos_submit (+ gpuos_flush).  Returns the first ticket; with check=False returns
        (status, first ticket) instead of raising."""
        n = len(tasks) - first if count is None else count
        t0 = ctypes.c_uint64()
        call = lib().gpuos_submit_flush if flush else lib().gpuos_submit
        rc = call(self._ctx, _tasks_ptr(tasks, first), n, ctypes.byref(t0))
        if not check:
            return rc, t0.value
        _check(rc, "gpuos_submit")
        return t0.value

    def flush(self):
        _check(lib().gpuos_flush(self._ctx), "gpuos_flush")

    def wait(self, ticket=ALL, timeout_ns=0, check=True):
        rc = lib().gpuos_wait(self._ctx, ticket, timeout_ns)
        if check and rc in (E_TIMEOUT, E_DEAD):
            # a wait that ran out of time, or whose worker left: say where the queue stands
            q = self.peek_queue()
            _check(rc, "gpuos_wait [submitted %d, published %d, units claimed %d, tasks completed %d, worker alive %s]" % (
                q.head_submitted, q.tail_published, q.claimed, q.completed, self.worker_alive()))
        if check:
            _check(rc, "gpuos_wait")
        return rc

    def completions(self, first, n):
        out = np.zeros(n, dtype=S.COMPLETION_DT)
        _check(lib().gpuos_get_completions(self._ctx, first, n, out.ctypes.data), "gpuos_get_completions")
        return out

    def run_serial(self, tasks, first=0, count=None):
        """gpuos_run_serial: one task at a time; returns per-task latencies in ns."""
        n = len(tasks) - first if count is None else count
        lat = np.zeros(n, dtype=np.uint64)
        _check(lib().gpuos_run_serial(self._ctx, _tasks_ptr(tasks, first), n, lat.ctypes.data), "gpuos_run_serial")
        return lat

    # -- introspection ---------------------------------------------------------
    def peek_queue(self):
        q = QueueState()
        _check(lib().gpuos_peek_queue(self._ctx, ctypes.byref(q)), "gpuos_peek_queue")
        return q

    def worker_alive(self):
        return bool(self._ctx) and lib().gpuos_worker_alive(self._ctx) == 1

    def set_yield_every(self, every):
        _check(lib().gpuos_set_yield_every(self._ctx, every), "gpuos_set_yield_every")

    # -- lifecycle ------------------------------------------------------------------
    def stop_worker(self, check=True):
        rc = lib().gpuos_stop_worker(self._ctx)
        if check:
            _check(rc, "gpuos_stop_worker")
        return rc

    def start_worker(self, check=True):
        """gpuos_start_worker: launch the worker again after stop_worker() or an idle exit."""
        rc = lib().gpuos_start_worker(self._ctx)
        if check:
            _check(rc, "gpuos_start_worker")
        return rc

    def worker_elapsed_ms(self):
        ms = ctypes.c_float()
        _check(lib().gpuos_worker_elapsed_ms(self._ctx, ctypes.byref(ms)), "gpuos_worker_elapsed_ms")
        return ms.value

    STAT_NAMES = ["disp_batches", "disp_records", "disp_units", "disp_ticks_stage", "disp_ticks_resolve",
                  "disp_ticks_write", "disp_ticks_busy", "disp_polls", "work_units", "work_ticks_wait",
                  "work_ticks_fetch", "work_ticks_dep", "work_ticks_exec", "work_ticks_complete",
                  "work_ticks_total", "disp_deferred"]

    def submit_from_threads(self, tasks, n_threads, batch=64, passes=1):
        """gpuos_submit_from_threads over the whole array; returns the seconds until all was submitted."""
        secs = ctypes.c_double()
        _check(lib().gpuos_submit_from_threads(self._ctx, _tasks_ptr(tasks, 0), len(tasks), int(n_threads), int(batch),
                                               int(passes), ctypes.byref(secs)), "gpuos_submit_from_threads")
        return secs.value

    def trace(self, first, n):
        """Device-written trace records of completed tickets [first, first + n) (gpuos_get_trace)."""
        out = np.zeros(n, dtype=TRACE_DT)
        _check(lib().gpuos_get_trace(self._ctx, int(first), int(n), out.ctypes.data), "gpuos_get_trace")
        return out

    def op_counts(self):
        out = np.zeros(256, dtype=np.uint64)
        _check(lib().gpuos_op_counts(self._ctx, out.ctypes.data), "gpuos_op_counts")
        return out

    def audit_log(self):
        """Every change of the operator table so far (gpuos_audit_log), oldest first."""
        total = ctypes.c_uint64()
        _check(lib().gpuos_audit_log(self._ctx, 0, 0, None, ctypes.byref(total)), "gpuos_audit_log")
        first = max(0, total.value - 65536)
        out = np.zeros(total.value - first, dtype=AUDIT_DT)
        _check(lib().gpuos_audit_log(self._ctx, first, len(out), out.ctypes.data, None), "gpuos_audit_log")
        return out

    def trace_origin_ns(self):
        v = ctypes.c_uint64()
        _check(lib().gpuos_trace_origin(self._ctx, ctypes.byref(v)), "gpuos_trace_origin")
        return v.value

    def kill_op(self, op_id):
        v = ctypes.c_uint32()
        _check(lib().gpuos_kill_op(self._ctx, int(op_id), ctypes.byref(v)), "gpuos_kill_op")
        return v.value

    def worker_stats(self):
        """Counters of the persistent kernel (after stop_worker); ticks are 10 ns."""
        out = np.zeros(16, dtype=np.uint64)
        _check(lib().gpuos_worker_stats(self._ctx, out.ctypes.data), "gpuos_worker_stats")
        return dict(zip(self.STAT_NAMES, (int(x) for x in out)))

    def shutdown(self, check=True):
        if not self._ctx:
            return OK
        ctx, self._ctx = self._ctx, ctypes.c_void_p()
        rc = lib().gpuos_shutdown(ctx)
        if check:
            _check(rc, "gpuos_shutdown")
        return rc

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.shutdown(check=exc[0] is None)
        return False

    def __del__(self):
        try:
            self.shutdown(check=False)
        except Exception:
            pass


def launch_per_op(tasks, table, device=0, sync_each=False, first=0, count=None):
    """gpuos_launch_per_op: the stream as one ordinary kernel launch per task.
    Returns (seconds, per-task latencies in ns or None)."""
    n = len(tasks) - first if count is None else count
    impl = np.zeros(MAX_OPS, dtype=np.uint32)
    for op, im in table.items():
        impl[op] = im
    lat = np.zeros(n, dtype=np.uint64) if sync_each else None
    secs = ctypes.c_double()
    rc = lib().gpuos_launch_per_op(device, _tasks_ptr(tasks, first), n, impl.ctypes.data, 1 if sync_each else 0,
                                   lat.ctypes.data if sync_each else None, ctypes.byref(secs))
    _check(rc, "gpuos_launch_per_op")
    return secs.value, lat


def task_bytes(tasks, impls):
    """Algorithmic HBM bytes of every task (gpuos_task_bytes)."""
    out = np.zeros(len(tasks), dtype=np.uint64)
    b = ctypes.c_uint64()
    L = lib()
    for i in range(len(tasks)):
        _check(L.gpuos_task_bytes(_tasks_ptr(tasks, i), int(impls[i]), ctypes.byref(b)), "gpuos_task_bytes")
        out[i] = b.value
    return out


PATHS = ("NOP", "CONTIG", "ROW2D", "GENERIC", "RED_CONTIG", "RED_GENERIC", "TILE2D", "ROW_FUSED", "ROW_GENERIC", "STAGED")


def task_plan(tasks, i, impl):
    """(path name, chunks, chunk size, merged dims) the host packs task i into (gpuos_task_plan)."""
    out = (ctypes.c_uint32 * 4)()
    _check(lib().gpuos_task_plan(_tasks_ptr(tasks, i), int(impl), out), "gpuos_task_plan")
    return PATHS[out[0]], int(out[1]), int(out[2]), int(out[3])


@atexit.register
def _shutdown_live():
    for rt in list(_live):
        try:
            rt.shutdown(check=False)
        except Exception:
            pass
