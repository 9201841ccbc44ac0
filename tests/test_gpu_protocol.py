"""GPU tests of the queue protocol, the operator table and failure handling.  Every wait is bounded
(wait_timeout_ms) and every kernel exits normally; error conditions are forced from the host."""
import time

import numpy as np
import pytest
import torch

from paper_2604_17861_amd import runtime as R
from paper_2604_17861_amd import streams as S
from helpers import Builder, run_oracle

pytestmark = pytest.mark.gpu

CFG = dict(idle_exit_ms=20000, wait_timeout_ms=20000)


def _dev(stream):
    from gpu_helpers import DevicePools
    return DevicePools(stream)


def _simple_adds(n_tasks, numel, seed=0):
    s = S.config1(n_tasks=n_tasks, numel=numel, seed=seed)
    return s


def test_tiny_ring_wraps_and_back_pressures():
    """Capacity 4 and 16: hundreds of laps of the ring, blocking back-pressure, single- and
    multi-chunk tasks; results bit-exact."""
    from gpu_helpers import compare_with_oracle
    for cap, numel in ((4, 1024), (16, 50000), (2, 300)):
        print("ring capacity", cap, flush=True)
        s = _simple_adds(600, numel, seed=cap)
        dp = _dev(s)
        with R.Runtime(cap, **CFG) as rt:
            rt.register_table(s.table)
            for i in range(0, len(s), 7):                      # batches larger than the ring
                rt.submit(dp.tasks, i, min(7, len(s) - i))
            rt.wait()
            q = rt.peek_queue()
            assert q.capacity == cap and q.completed == 600 and q.head_submitted == 600 and q.claimed == 600
            comps = rt.completions(0, 600)
        assert np.all(comps["status"] == 0)
        stats = compare_with_oracle(s, dp.download())
        assert stats["max_ulp"] == 0


def test_nonblocking_submit_reports_full_and_enqueues_nothing():
    s = _simple_adds(64, 1 << 16)
    dp = _dev(s)
    with R.Runtime(8, nonblocking_submit=1, **CFG) as rt:
        rt.register_table(s.table)
        rc, _ = rt.submit(dp.tasks, 0, 9, check=False)           # more than the whole ring
        assert rc == R.E_FULL
        assert rt.peek_queue().head_submitted == 0
        rc, t0 = rt.submit(dp.tasks, 0, 8, check=False)
        assert rc == R.OK and t0 == 0
        rt.wait()
        rc, t1 = rt.submit(dp.tasks, 8, 8, check=False)
        assert rc == R.OK and t1 == 8
        rt.wait()


def test_malformed_descriptors_are_rejected_before_anything_is_enqueued():
    s = _simple_adds(8, 1024)
    dp = _dev(s)
    with R.Runtime(0, **CFG) as rt:
        rt.register_table(s.table)
        def bad(mutate):
            t = dp.tasks.copy()
            mutate(t)
            rc, _ = rt.submit(t, 0, 8, check=False)
            assert rt.peek_queue().head_submitted == 0, "a rejected batch must leave the ring untouched"
            return rc
        assert bad(lambda t: t["ndim"].__setitem__(5, 7)) == R.E_INVAL
        assert bad(lambda t: t["ndim"].__setitem__(0, 0)) == R.E_INVAL
        assert bad(lambda t: t["inp"]["stride"].__setitem__((3, 0, 0), -1)) == R.E_INVAL
        assert bad(lambda t: t["out"]["stride"].__setitem__((7, 0), 0)) == R.E_INVAL
        assert bad(lambda t: t["out"]["bcast_mask"].__setitem__(2, 1)) == R.E_INVAL
        assert bad(lambda t: t["inp"]["ptr"].__setitem__((4, 1), 0)) == R.E_INVAL
        assert bad(lambda t: t["inp"]["dtype"].__setitem__((4, 1), S.I32)) == R.E_INVAL
        assert bad(lambda t: t["n_inputs"].__setitem__(1, 1)) == R.E_INVAL
        assert bad(lambda t: t["flags"].__setitem__(1, 64)) == R.E_INVAL
        assert bad(lambda t: t["dep"].__setitem__((0, 0), 1)) == R.E_INVAL          # before ticket 0
        assert bad(lambda t: t["dep"].__setitem__((7, 2), 4096)) == R.E_INVAL       # >= capacity
        assert bad(lambda t: t["op_id"].__setitem__(6, 200)) == R.E_BADOP           # never registered
        assert bad(lambda t: t["op_id"].__setitem__(6, 300)) == R.E_BADOP           # out of range
        assert bad(lambda t: t["size"].__setitem__((6, 0), 1 << 31)) == R.E_INVAL
        rt.submit(dp.tasks)                                                          # the intact batch still runs
        rt.wait()
        assert rt.wait(3) == R.OK
        assert rt.wait(8, check=False) == R.E_INVAL                                  # never submitted
        with pytest.raises(R.GpuosError):
            rt.register_op(S.OP["ADD"], S.IMPL["MUL"])                               # already bound
        with pytest.raises(R.GpuosError):
            rt.swap_op(S.OP["ADD"], S.IMPL["RELU"])                                  # arity differs
        with pytest.raises(R.GpuosError):
            rt.swap_op(199, S.IMPL["RELU"])                                          # unregistered
        with pytest.raises(R.GpuosError):
            rt.register_op(300, S.IMPL["RELU"])


def test_device_bounds_check_reports_bad_op_ids():
    """With the host-side op check deferred, the device rejects unknown and out-of-range op ids at
    claim time and reports them; neighbours are unaffected."""
    from gpu_helpers import compare_with_oracle
    s = _simple_adds(40, 2048)
    dp = _dev(s)
    t = dp.tasks.copy()
    t["op_id"][5] = 200
    t["op_id"][17] = 999
    with R.Runtime(0, defer_op_check=1, **CFG) as rt:
        rt.register_table(s.table)
        rt.submit(t)
        assert rt.wait(check=False) == R.E_BADOP
        c = rt.completions(0, 40)
        assert rt.wait(5, check=False) == R.E_BADOP and rt.wait(6, check=False) == R.OK
    bad = np.zeros(40, bool); bad[[5, 17]] = True
    assert np.all(c["status"][bad] == R.E_BADOP) and np.all(c["status"][~bad] == 0)
    imgs = dp.download()
    out = imgs[2].view(np.float32).reshape(40, 2048)
    assert not out[5].any() and not out[17].any()                 # rejected tasks wrote nothing
    keep = np.nonzero(~bad)[0]
    for i in keep[:3]:
        a = imgs[0].view(np.float32).reshape(40, 2048)[i]; b = imgs[1].view(np.float32).reshape(40, 2048)[i]
        assert np.array_equal(out[i], a + b)


def test_kill_switch_fails_fast_and_can_be_lifted():
    s = _simple_adds(30, 4096)
    dp = _dev(s)
    with R.Runtime(0, **CFG) as rt:
        rt.register_table(s.table)
        rt.submit(dp.tasks, 0, 10); rt.wait()
        v = rt.swap_op(S.OP["ADD"], S.IMPL["FAIL"])
        assert v == 2
        rt.submit(dp.tasks, 10, 10)
        assert rt.wait(check=False) == R.E_BADOP
        v = rt.swap_op(S.OP["ADD"], S.IMPL["ADD"])
        assert v == 3
        rt.submit(dp.tasks, 20, 10); rt.wait()
        c = rt.completions(0, 30)
    assert np.all(c["status"][:10] == 0) and np.all(c["status"][10:20] == R.E_BADOP) and np.all(c["status"][20:] == 0)
    assert c["op_version"].tolist() == [1] * 10 + [2] * 10 + [3] * 10
    out = dp.download()[2].view(np.float32).reshape(30, 4096)
    assert out[:10].any(axis=1).all() and not out[10:20].any() and out[20:].any(axis=1).all()


@pytest.mark.parametrize("numel", [4096, 100003])
def test_dependency_chain_hand_offs(numel):
    """x_{i+1} = x_i + 1 through 1500 dependent tasks (single- and multi-chunk): every hand-off crosses
    workgroups and XCDs; the result is exact only if each task saw its predecessor's output."""
    n = 1500
    b = Builder()
    buf = b.pool(np.zeros((n + 1, numel), np.float32))
    buf[0] = np.arange(numel, dtype=np.float32) % 97
    ones = b.pool(np.ones(numel, np.float32))
    for i in range(n):
        b.add("ADD", buf[i + 1], [buf[i], ones], dep=(1 if i else 0, 0, 0))
    s = b.stream()
    dp = _dev(s)
    with R.Runtime(0, **CFG) as rt:
        rt.register_table(s.table)
        rt.submit(dp.tasks); rt.wait()
    out = dp.download()[0].view(np.float32).reshape(n + 1, numel)
    assert np.array_equal(out[n], out[0] + n)
    assert np.array_equal(out[n // 2], out[0] + n // 2)


def test_fence_and_in_place_updates():
    """40 independent tasks write rows; a FENCE task then sums over all rows; in-place SCALE on the
    result depends on it."""
    b = Builder()
    rows = b.pool(np.zeros((40, 3000), np.float32))
    src = b.pool(np.random.default_rng(1).standard_normal((40, 3000)).astype(np.float32))
    tot = b.pool(np.zeros(3000, np.float32))
    for i in range(40):
        b.add("SCALE", rows[i], [src[i]], alpha=2.0)
    b.add("SUM_LAST", tot, [rows.T], flags=S.FLAG_FENCE)          # column sums need every row
    b.add("SCALE", tot, [tot], alpha=0.5, dep=(1, 0, 0))            # in place
    s = b.stream()
    dp = _dev(s)
    with R.Runtime(0, **CFG) as rt:
        rt.register_table(s.table)
        rt.submit(dp.tasks); rt.wait()
    imgs = dp.download()
    hp, st = run_oracle(s)
    assert np.array_equal(imgs[0], hp.arrays[0])
    np.testing.assert_allclose(imgs[2].view(np.float32), hp.arrays[2].view(np.float32), rtol=1e-5, atol=1e-5)


def test_introspection_yield_policy_and_stats():
    s = _simple_adds(200, 8192)
    dp = _dev(s)
    with R.Runtime(0, phase_timers=1, **CFG) as rt:
        assert rt.worker_alive()
        q = rt.peek_queue()
        assert q.capacity == 4096 and q.workgroups >= 256 and q.head_submitted == 0 and q.heartbeat > 0
        rt.register_table(s.table)
        rt.set_yield_every(4)                                       # workers pause on every 4th empty poll
        rt.submit(dp.tasks, 0, 100, flush=False)
        assert rt.peek_queue().tail_published == 0 and rt.peek_queue().head_submitted == 100
        rt.flush()
        rt.wait()
        rt.set_yield_every(0)
        rt.submit(dp.tasks, 100, 100); rt.wait()
        q = rt.peek_queue()
        assert q.completed == 200 and q.claimed == 200 and q.tail_published == 200
        assert rt.worker_alive()
        c = rt.completions(0, 200)
        assert np.all(c["t_done_ns"] >= c["t_submit_ns"]) and np.all(c["t_submit_ns"] > 0)
        rt.stop_worker()
        assert not rt.worker_alive()
        st = rt.worker_stats()
        units = sum(R.task_plan(dp.tasks, i, S.IMPL["ADD"])[1] for i in range(200))      # 8,192 elements: two chunks each
        assert units == 400
        assert st["work_units"] == units and st["disp_records"] == 200 and st["work_ticks_exec"] > 0
        assert rt.worker_elapsed_ms() > 0
        rc, _ = rt.submit(dp.tasks, 0, 1, check=False)
        assert rc == R.E_DEAD
    from gpu_helpers import compare_with_oracle
    assert compare_with_oracle(s, dp.download())["max_ulp"] == 0


def test_shutdown_drains_tasks_in_flight_and_is_idempotent():
    s = _simple_adds(3000, 30000)
    dp = _dev(s)
    rt = R.Runtime(0, **CFG)
    rt.register_table(s.table)
    rt.submit(dp.tasks)                          # no wait: shutdown has to drain
    assert rt.shutdown() == R.OK
    assert rt.shutdown() == R.OK                 # second call is a no-op
    from gpu_helpers import compare_with_oracle
    assert compare_with_oracle(s, dp.download())["max_ulp"] == 0


def test_a_new_context_takes_nothing_an_earlier_one_left_in_device_memory():
    """Contexts created one after the other in a process get the same device blocks back from the
    allocator, and each numbers its tickets from 0: a descriptor the earlier context left in the
    device-side mirror would carry a valid check word for the same ticket of the later one.  Every
    task of every context runs, on its own descriptor."""
    from gpu_helpers import compare_with_oracle
    for rep in range(6):
        s = _simple_adds(3000, 3000, seed=10 + rep)
        dp = _dev(s)
        with R.Runtime(0, **CFG) as rt:
            rt.register_table(s.table)
            for i in range(0, len(s), 500):
                rt.submit(dp.tasks, i, 500)
            rt.wait()
            assert rt.peek_queue().completed == len(s)
        assert compare_with_oracle(s, dp.download())["max_ulp"] == 0


def test_idle_watchdog_exits_the_worker():
    s = _simple_adds(4, 1024)
    dp = _dev(s)
    with R.Runtime(0, idle_exit_ms=200, wait_timeout_ms=5000) as rt:
        rt.register_table(s.table)
        rt.submit(dp.tasks, 0, 2); rt.wait()
        time.sleep(0.6)
        assert not rt.worker_alive()
        rc, _ = rt.submit(dp.tasks, 2, 2, check=False)
        assert rc == R.E_DEAD


def test_per_op_launch_path_matches_the_oracle():
    """The comparison path (one ordinary launch per task) runs the same stream to the same results."""
    import parity_cases as C
    from gpu_helpers import compare_with_oracle
    for s in (C.config2_reduced(), S.config3(n_chains=3, buffer_sets=1, Bs=(1, 2), Ss=(64, 128)),
              C.config5_reduced()):
        dp = _dev(s)
        secs, lat = R.launch_per_op(dp.tasks, s.table, sync_each=False)
        torch.cuda.synchronize()
        stats = compare_with_oracle(s, dp.download())
        print(s.name, stats, "%.1f ms" % (secs * 1e3), flush=True)
    s = _simple_adds(50, 1024)
    dp = _dev(s)
    secs, lat = R.launch_per_op(dp.tasks, s.table, sync_each=True)
    assert len(lat) == 50 and np.all(lat > 0)


def test_two_contexts_side_by_side():
    s1, s2 = _simple_adds(300, 5000, seed=1), _simple_adds(300, 5000, seed=2)
    d1, d2 = _dev(s1), _dev(s2)
    from gpu_helpers import compare_with_oracle
    with R.Runtime(64, workgroups_per_cu=1, **CFG) as a, R.Runtime(64, workgroups_per_cu=1, **CFG) as b:
        a.register_table(s1.table); b.register_table(s2.table)
        for i in range(0, 300, 50):
            a.submit(d1.tasks, i, 50); b.submit(d2.tasks, i, 50)
        a.wait(); b.wait()
    assert compare_with_oracle(s1, d1.download())["max_ulp"] == 0
    assert compare_with_oracle(s2, d2.download())["max_ulp"] == 0


@pytest.mark.parametrize("push_ring", [0, 1])
def test_both_ring_placements(push_ring):
    """push_ring = 1: ring, doorbell and table source live in device memory and the host writes them
    through the PCIe BAR; 0: they live in host memory and the device polls over PCIe (the default
    picks by what the BAR allows, so the other tests run whichever this box supports).  Same
    results, same version invariants, wrap-around included."""
    import parity_cases as C
    from gpu_helpers import compare_with_oracle, run_stream
    for s, cap in ((C.config2_reduced(), 0), (C.config4_reduced(), 64), (S.config3(n_chains=6, buffer_sets=1, Bs=(1, 2), Ss=(64, 128)), 32)):
        print("push_ring", push_ring, s.name, "capacity", cap or 4096, flush=True)
        dp = _dev(s)
        with R.Runtime(cap, push_ring=push_ring, **CFG) as rt:
            assert rt.peek_queue().push_ring == push_ring
            rt.register_table(s.table)
            t0 = run_stream(s, rt, dp)
            comps = rt.completions(t0, len(s))
            lat = rt.run_serial(dp.tasks, 0, 20)
        assert np.all(comps["status"] == 0) and np.all(lat > 0)
        stats = compare_with_oracle(s, dp.download(), versions=comps["op_version"])
        print(stats, flush=True)
        if s.swaps:
            v = comps["op_version"].astype(np.int64)
            gelu = s.tasks["op_id"] == S.OP_GELU
            for k, (t, _, _) in enumerate(s.swaps):
                assert np.all(v[t:][gelu[t:]] >= k + 2)


def test_device_trace_ring_and_operator_counts():
    """Tracing on: every task leaves a device-written tracepoint (dequeue <= start <= done on the
    device clock, version / op / status / chunk count as the completion log and the descriptors say),
    the per-operator dispatch counts add up to the stream's histogram, kill_op shows in the trace,
    and records older than the trace ring report as overwritten.  Tracing off: the calls say so."""
    s = S.config2(n_tasks=3000)
    dp = _dev(s)
    with R.Runtime(0, trace_entries=1024, **CFG) as rt:
        rt.register_table(s.table)
        assert rt.cfg.trace_entries == 1024
        t0 = rt.submit(dp.tasks, 0, 2000)
        rt.wait()
        tr = rt.trace(t0 + 1000, 1000)                         # the last 1000 of 2000: inside a ring of 4096 (>= capacity)
        comps = rt.completions(t0 + 1000, 1000)
        assert np.array_equal(tr["ticket"], np.arange(t0 + 1000, t0 + 2000, dtype=np.uint64))
        odd = tr[(tr["t_dequeue"] > tr["t_start"]) | (tr["t_start"] > tr["t_done"])]
        assert len(odd) == 0, odd
        assert np.all(tr["t_done"] < 100e6 * 20)               # ticks since the worker started: well under the 20 s of the test
        assert np.array_equal(tr["op_version"], comps["op_version"]) and np.all(tr["status"] == 0)
        assert np.array_equal(tr["op_id"], s.tasks["op_id"][1000:2000])
        impl = s.impl_for()
        want_chunks = np.array([R.task_plan(dp.tasks, i, impl[i])[1] for i in range(1000, 2000)])
        assert np.array_equal(tr["nchunks"], want_chunks)
        assert tr["workgroup"].min() >= 1 and tr["workgroup"].max() < 1024 and len(np.unique(tr["workgroup"])) > 50
        exec_us = (tr["t_done"] - tr["t_start"]) / 100.0
        print("device exec time per task: p50 %.1f us, p99 %.1f us; dequeue->start p50 %.1f us" % (
            np.percentile(exec_us, 50), np.percentile(exec_us, 99),
            np.percentile((tr["t_start"] - tr["t_dequeue"]) / 100.0, 50)), flush=True)
        # the ring is idle now: the counts have been flushed
        deadline = time.time() + 5
        want = np.bincount(s.tasks["op_id"][:2000].astype(np.int64), minlength=256).astype(np.uint64)
        while time.time() < deadline and not np.array_equal(rt.op_counts(), want):
            time.sleep(0.01)
        assert np.array_equal(rt.op_counts(), want)
        # kill switch: the stub's status is in the trace, nothing else changes
        v = rt.kill_op(S.OP["EXP"])
        t1 = rt.submit(dp.tasks, 2000, 1000)
        try:
            rt.wait()
        except R.GpuosError as e:
            assert e.status == R.E_BADOP
        tr2 = rt.trace(t1, 1000)
        is_exp = s.tasks["op_id"][2000:3000] == S.OP["EXP"]
        assert is_exp.any() and np.all(tr2["status"][is_exp] == R.E_BADOP) and np.all(tr2["status"][~is_exp] == 0)
        assert np.all(tr2["op_version"][is_exp] == v)
        # records that the ring no longer holds
        big = rt.cfg.trace_entries
        assert big == 4096 or big == 1024
        origin = rt.trace_origin_ns()
        assert origin > 0
    s2 = _simple_adds(6000, 256)
    dp2 = _dev(s2)
    with R.Runtime(16, trace_entries=64, **CFG) as rt:
        rt.register_table(s2.table)
        t0 = rt.submit(dp2.tasks, 0, 6000)
        rt.wait()
        assert len(rt.trace(t0 + 6000 - 64, 64)) == 64
        with pytest.raises(R.GpuosError):
            rt.trace(t0, 1)                                    # overwritten long ago
        # The device clock lines up with the host clock: a lone task is dequeued after the host rang the
        # doorbell and done before the host saw its completion word.  The two transit times together do
        # not depend on the clock offset at all; each alone is off by the offset's error, which is the
        # PCIe write of the first heartbeat plus whatever the host thread was doing when it arrived.
        lat = rt.run_serial(dp2.tasks, 0, 50)
        first = t0 + 6000
        tr3, c3 = rt.trace(first, 50), rt.completions(first, 50)
        deq = tr3["t_dequeue"].astype(np.int64) * 10 + rt.trace_origin_ns() - c3["t_submit_ns"].astype(np.int64)
        fin = c3["t_done_ns"].astype(np.int64) - (tr3["t_done"].astype(np.int64) * 10 + rt.trace_origin_ns())
        both = float(np.median(deq + fin))
        assert 500 < both < 30000, (both, np.median(lat))
        assert -50000 < np.median(deq) < 80000 and -50000 < np.median(fin) < 80000, (np.median(deq), np.median(fin))
    with R.Runtime(0, **CFG) as rt:
        with pytest.raises(R.GpuosError):
            rt.op_counts()
        with pytest.raises(R.GpuosError):
            rt.trace(0, 1)


def test_many_producer_threads_on_one_context():
    """Eight host threads submit to one ring at the same time (batches of 1..16, with a large and
    with a tiny ring so that producers also meet back-pressure); every
    batch gets consecutive tickets, every ticket completes once, results are bit-exact."""
    import threading
    from gpu_helpers import compare_with_oracle
    n_threads, per_thread = 8, 1500
    s = _simple_adds(n_threads * per_thread, 2048, seed=5)
    dp = _dev(s)
    tickets = np.full(len(s), -1, np.int64)
    errors = []
    for cap in (4096, 64):
        with R.Runtime(cap, **CFG) as rt:
            rt.register_table(s.table)
            def producer(k):
                try:
                    rng = np.random.default_rng(k)
                    i, end = k * per_thread, (k + 1) * per_thread
                    while i < end:
                        m = int(min(rng.integers(1, 17), end - i))
                        t0 = rt.submit(dp.tasks, i, m)
                        tickets[i: i + m] = np.arange(t0, t0 + m)
                        i += m
                        if rng.random() < 0.05:
                            rt.wait(t0 + m - 1)
                except Exception as e:          # surfaced below: a thread must not die silently
                    errors.append(e)
            threads = [threading.Thread(target=producer, args=(k,)) for k in range(n_threads)]
            for t in threads:
                t.start()
            for t in threads:
                t.join()
            assert not errors, errors
            rt.wait()
            assert sorted(tickets.tolist()) == list(range(int(tickets.min()), int(tickets.min()) + len(s)))
            comps = rt.completions(int(tickets.min()), len(s))
            assert np.all(comps["status"] == 0)
        stats = compare_with_oracle(s, dp.download())
        assert stats["max_ulp"] == 0
        for img in dp.tensors[-1:]:
            img.zero_()                           # outputs start from zero again for the next capacity
        torch.cuda.synchronize()                  # no context is alive here: waiting for every stream is safe


def test_small_results_reach_the_host_through_a_copy_task_into_pinned_memory():
    """While the worker is resident a small device-to-host copy may queue behind it; the way to
    read a small result is a COPY task whose output is pinned (device-mapped) host memory: it is
    complete, and visible to the host, when gpuos_wait returns."""
    n = 1000
    src = torch.arange(n, dtype=torch.float32, device="cuda:0") * 0.5
    torch.cuda.current_stream().synchronize()
    dst = torch.zeros(n, dtype=torch.float32).pin_memory()
    tasks, pool_of = S.new_tasks(2)
    S.set_head(tasks, 0, S.OP["COPY"], [n], 1)
    S.set_tensor(tasks, pool_of, 0, 0, 0, src.data_ptr(), [1], S.F32)
    S.set_tensor(tasks, pool_of, 0, 3, 0, dst.data_ptr(), [1], S.F32)
    S.set_head(tasks, 1, S.OP["SCALE"], [n // 2], 1, alpha=-2.0, dep=(1, 0, 0))          # host memory as an INPUT as well
    S.set_tensor(tasks, pool_of, 1, 0, 0, dst.data_ptr(), [2], S.F32)
    S.set_tensor(tasks, pool_of, 1, 3, 0, dst.data_ptr() + 4, [2], S.F32)
    with R.Runtime(0, **CFG) as rt:
        rt.register_table(S.default_table())
        t = rt.submit(tasks, 0, 1)
        rt.wait(t)
        assert rt.worker_alive()
        assert np.array_equal(dst.numpy(), np.arange(n, dtype=np.float32) * 0.5)      # read while the worker runs
        t = rt.submit(tasks, 1, 1)
        rt.wait(t)
        want = np.arange(n, dtype=np.float32) * 0.5
        want[1::2] = want[0::2] * np.float32(-2.0)
        assert np.array_equal(dst.numpy(), want)


def test_worker_stopped_and_started_again_continues_where_it_was():
    """gpuos_stop_worker / gpuos_start_worker (and the idle exit): tickets, results, the operator
    table and the trace continue across runs of the worker kernel."""
    from gpu_helpers import DevicePools, run_stream, compare_with_oracle
    import parity_cases as P
    s = P.config2_reduced()
    dp = DevicePools(s)
    n = len(s)
    cuts = [0, n // 5, n // 2, n - 7, n]
    with R.Runtime(64, idle_exit_ms=300, wait_timeout_ms=20000, trace_entries=4096) as rt:
        rt.register_table(s.table)
        for k in range(4):
            first = run_stream(s, rt, dp, cuts[k], cuts[k + 1] - cuts[k])
            assert first == cuts[k]
            if k == 0:
                rt.stop_worker()
                assert not rt.worker_alive()
                assert rt.submit(dp.tasks, 0, 1, check=False)[0] == R.E_DEAD
                assert rt.start_worker(check=False) == R.OK
            elif k == 1:
                time.sleep(0.6)                                   # idle exit: the worker leaves by itself
                assert not rt.worker_alive()
                assert rt.start_worker(check=False) == R.OK
            elif k == 2:
                rt.stop_worker()
                rt.start_worker()
                rt.start_worker()                                 # running: nothing to do
            assert rt.worker_alive()
        q = rt.peek_queue()
        assert q.completed == n and q.claimed == n and q.head_submitted == n
        comp = rt.completions(0, n)
        assert (comp["status"] == 0).all() and (comp["ticket"] == np.arange(n)).all()
        tr = rt.trace(n - 50, 50)
        assert (tr["t_done"] >= tr["t_start"]).all() and (tr["t_start"] >= tr["t_dequeue"]).all()
        assert int(rt.op_counts().sum()) == n
        rt.stop_worker()
        gpu = dp.download()
    compare_with_oracle(s, gpu)


def test_wait_with_a_time_limit():
    """gpuos_wait with a limit far below the work outstanding reports GPUOS_E_TIMEOUT and loses
    nothing: the same wait without a limit succeeds and the results are right."""
    from gpu_helpers import compare_with_oracle
    s = _simple_adds(64, 1 << 22, seed=5)                 # 64 adds of 4M elements: about 0.5 ms of memory traffic a pass
    dp = _dev(s)
    with R.Runtime(0, **CFG) as rt:
        rt.register_table(s.table)
        t0 = rt.submit(dp.tasks, 0, 64)
        for _ in range(3):                                       # the same adds again (they only rewrite their results):
            rt.submit(dp.tasks, 0, 64)                           # about 2 ms outstanding, far above a host hiccup
        assert rt.wait(t0 + 255, timeout_ns=1000, check=False) == R.E_TIMEOUT
        assert rt.worker_alive()
        assert rt.wait(t0 + 256, check=False) == R.E_INVAL       # never issued
        assert rt.wait(t0 + 255, check=False) == R.OK
        assert rt.wait(timeout_ns=1, check=False) == R.OK        # everything is complete: no time needed
    assert compare_with_oracle(s, dp.download())["max_ulp"] == 0


@pytest.mark.parametrize("seed", [0, 1, 2, 3, 4, 5])
def test_randomized_call_sequences(seed):
    """A seeded random walk over the host calls -- submits of 1..40 tasks with and without a
    doorbell, waits for earlier tickets, queue peeks, yield-policy changes, the worker stopped and
    started, read-outs of the completion log -- on a random ring size, placement, grid size and
    chunk size.  Whatever the
    interleaving, every ticket completes once, in the log in order, and the results are the oracle's."""
    from gpu_helpers import compare_with_oracle
    import parity_cases as P
    rng = np.random.default_rng(1000 + seed)
    s = P.config2_reduced()
    dp = _dev(s)
    n = len(s)
    cap = int(rng.choice([4, 64, 4096]))
    cfg = dict(CFG, push_ring=int(rng.integers(0, 2)), harvester_thread=int(rng.integers(0, 2)),
               trace_entries=int(rng.choice([0, 256])))
    shape = np.random.default_rng(2000 + seed)                    # (its own generator: the walks above stay as they were)
    cfg.update(workgroups_per_cu=int(shape.integers(1, 5)), chunk_elems=int(shape.choice([0, 1024, 4096, 32768])))
    print("seed", seed, "capacity", cap, cfg, flush=True)
    done = 0
    with R.Runtime(cap, **cfg) as rt:
        rt.register_table(s.table)
        steps = 0
        while done < n:
            steps += 1
            a = rng.random()
            if a < 0.55:
                k = int(min(n - done, rng.integers(1, 41)))
                first = rt.submit(dp.tasks, done, k, flush=bool(rng.random() < 0.7))
                assert first == done
                done += k
            elif a < 0.70 and done:
                rt.wait(int(rng.integers(0, done)))
            elif a < 0.78:
                q = rt.peek_queue()
                assert q.head_submitted == done and q.completed <= q.claimed <= q.tail_published <= done
            elif a < 0.84:
                rt.set_yield_every(int(rng.choice([0, 0, 3, 50])))
            elif a < 0.90 and done:
                lo = int(rng.integers(0, done))
                rt.wait(lo)
                c = rt.completions(lo, 1)
                assert c["ticket"][0] == lo and c["status"][0] == 0
            elif a < 0.95:
                rt.stop_worker()                                  # drains what was submitted (a doorbell is rung)
                assert rt.peek_queue().completed == done
                rt.start_worker()
            else:
                rt.flush()
        rt.wait()
        comps = rt.completions(0, n)
        assert rt.worker_alive()
    print("steps", steps, flush=True)
    assert np.array_equal(comps["ticket"], np.arange(n, dtype=np.uint64)) and np.all(comps["status"] == 0)
    assert np.all(comps["t_done_ns"] >= comps["t_submit_ns"])
    compare_with_oracle(s, dp.download(), versions=comps["op_version"])
