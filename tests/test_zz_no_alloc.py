"""gpuos_init_static, the entry point that allocates nothing (device-side state in a file-scope
device array of the library, host side in the caller's block, the caller's stream), against
gpuos_init on the same seeded streams: two calls in a row, the second with a smaller ring and a
smaller stream.  The outputs must equal those of the ordinary context byte for byte (the same
kernels run) and meet the oracle's bars."""
import ctypes

import numpy as np
import pytest

from paper_2604_17861_amd import runtime as R
from paper_2604_17861_amd import streams as S

pytestmark = pytest.mark.gpu

HOST_MALLOC_MAPPED, HOST_MALLOC_COHERENT, STREAM_NON_BLOCKING = 0x2, 0x40000000, 0x1


def _hip():
    R.lib()                                          # torch first, then the library: one HIP runtime in the process
    h = ctypes.CDLL("libamdhip64.so.7")
    h.hipHostMalloc.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_size_t, ctypes.c_uint]
    h.hipHostFree.argtypes = [ctypes.c_void_p]
    h.hipStreamCreateWithFlags.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_uint]
    h.hipStreamDestroy.argtypes = [ctypes.c_void_p]
    return h


def _run(stream, capacity, static=None):
    from gpu_helpers import DevicePools, run_stream
    dp = DevicePools(stream)
    with R.Runtime(capacity, static=static, idle_exit_ms=20000, wait_timeout_ms=20000, push_ring=0) as rt:
        rt.register_table(stream.table, stream.programs)
        t0 = run_stream(stream, rt, dp)
        comps = rt.completions(t0 + len(stream) - min(len(stream), capacity), min(len(stream), capacity))
        q = rt.peek_queue()
        assert q.capacity == capacity and q.completed == len(stream)
        assert rt.worker_alive()
    assert np.all(comps["status"] == 0)
    return dp.download(), comps


def test_static_context_matches_the_allocating_one_twice_in_a_row():
    import torch
    import parity_cases as C
    from gpu_helpers import compare_with_oracle
    assert torch.cuda.is_available()
    torch.cuda.set_device(0)
    hip = _hip()
    nbytes = R.static_host_bytes(R.STATIC_MAX_CAPACITY)
    block, block2, stream = ctypes.c_void_p(), ctypes.c_void_p(), ctypes.c_void_p()
    assert hip.hipHostMalloc(ctypes.byref(block), nbytes, HOST_MALLOC_MAPPED | HOST_MALLOC_COHERENT) == 0
    assert hip.hipHostMalloc(ctypes.byref(block2), nbytes, HOST_MALLOC_MAPPED | HOST_MALLOC_COHERENT) == 0
    assert hip.hipStreamCreateWithFlags(ctypes.byref(stream), STREAM_NON_BLOCKING) == 0
    ctypes.memset(block, 0xA5, nbytes)               # the library clears what it uses
    static = (block, nbytes, stream)
    try:
        # rejected sizes: a clear error and no context
        with pytest.raises(R.GpuosError) as e:
            R.Runtime(2 * R.STATIC_MAX_CAPACITY, static=static)
        assert e.value.status == R.E_INVAL
        assert "GPUOS_STATIC_MAX_CAPACITY" in R.lib().gpuos_last_hip_error().decode()
        cases = [(1024, S.config2(n_tasks=1500, in_pool_elems=1 << 21)),           # first call: the largest ring
                 (64, S.config3(n_chains=4, buffer_sets=1, Bs=(1, 2), Ss=(64, 128)))]   # second: a smaller ring, a smaller stream
        for capacity, s in cases:
            print("static context: ring", capacity, s.name, len(s), "tasks", flush=True)
            got, comps = _run(s, capacity, static=static)
            want, _ = _run(s, capacity)
            for k, (g, w) in enumerate(zip(got, want)):
                assert np.array_equal(np.asarray(g).view(np.uint8), np.asarray(w).view(np.uint8)), "pool %d differs" % k
            stats = compare_with_oracle(s, got)
            print(stats, flush=True)
        # one static context per GPU at a time: a second one is refused, not raced
        with R.Runtime(16, static=static, idle_exit_ms=20000) as rt:
            with pytest.raises(R.GpuosError) as e:
                R.Runtime(16, static=(block2, nbytes, stream))
            assert e.value.status == R.E_FULL
            assert rt.worker_alive()
    finally:                                         # (with no worker resident: freeing waits for the whole device)
        hip.hipStreamDestroy(stream)
        hip.hipHostFree(block)
        hip.hipHostFree(block2)
