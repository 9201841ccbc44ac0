#!/usr/bin/env python3
"""Benchmark of the GPUOS hot path on one MI355X.

A step is one pass of the whole hot path (descriptor packing, ring submission, persistent-kernel
dispatch, execution, completion harvesting) over the second configuration's stream: 10,000 mixed
elementwise tasks submitted in batches of 64.  `value` is persistent-queue tasks/s on that stream
with all tensors resident in HBM.  The same JSON line carries
  * the same stream issued as one ordinary kernel launch per task (throughput and latency mode),
  * p50 / p99 submit->done latency, one task of the stream at a time on both paths (p50_us against
    per_launch_p50_us), and of every task when the stream is submitted flat out (loaded_p50_us),
  * the other small-op streams (first and fourth configuration) against per-op launches,
  * "roofline": the persistent kernel over the fifth configuration (bandwidth stream): algorithmic
    bytes / kernel duration from HIP events on the worker's stream, against 8 TB/s,
  * "cpu_baseline": the CPU oracle timed on a bounded sample of the same stream on one host core.
Inputs are seeded and synthetic (paper_2604_17861_amd/streams.py).
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
KNOBS = {}                  # gpuos_config fields every context of this run is created with (--workgroups-per-cu)


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class DevicePools:
    """Pools of a stream in device memory (torch only allocates and copies)."""

    def __init__(self, stream, torch, device="cuda:0"):
        self.tensors = []
        for p in stream.pools:
            if p.tile is not None:
                t = torch.from_numpy(np.ascontiguousarray(p.tile)).to(device)
                reps = -(-p.nbytes // p.tile.nbytes)
                t = t.repeat(reps)[: p.nbytes].contiguous()
            elif p.data is not None:
                t = torch.from_numpy(np.ascontiguousarray(p.data)).to(device)
            else:
                t = torch.zeros(p.nbytes, dtype=torch.uint8, device=device)
            self.tensors.append(t)
        torch.cuda.current_stream().synchronize()
        self.bases = [t.data_ptr() for t in self.tensors]
        self.tasks = stream.materialize(self.bases)


def submit_pass(rt, stream, tasks):
    """One pass over the stream: batches of stream.batch, hot swaps where scheduled, then wait.
    The batches between two swaps are submitted by the library's own loop
    (gpuos_submit_from_threads with one thread: gpuos_submit + gpuos_flush per batch in the calling
    thread), so that the interpreter is not part of what is timed."""
    n = len(tasks)
    batch = stream.batch or n
    cuts = sorted({0, n} | {t for t, _, _ in stream.swaps if 0 < t < n})
    swaps = {t: (op, impl) for t, op, impl in stream.swaps}
    first = rt.peek_queue().head_submitted
    for lo, hi in zip(cuts[:-1], cuts[1:]):
        if lo in swaps and lo > 0:
            rt.swap_op(*swaps[lo])
        rt.submit_from_threads(tasks[lo:hi], 1, batch, 1)
    rt.wait()
    return first


def percentile_us(ns, q):
    return float(np.percentile(ns, q)) / 1e3 if len(ns) else None


def bench_persistent(R, stream, dp, steps, warmup, harvester=True, capacity=0, **cfg):
    with R.Runtime(capacity, harvester_thread=1 if harvester else 0, idle_exit_ms=60000, **KNOBS, **cfg,
                   completion_log=max(1 << 20, 1 << int(np.ceil(np.log2(len(stream) + 1))))) as rt:
        rt.register_table(stream.table)
        for _ in range(warmup):
            submit_pass(rt, stream, dp.tasks)
            _reset_swaps(rt, stream)
        lat = []
        dt = 0.0
        for _ in range(steps):
            t0 = time.perf_counter()
            first = submit_pass(rt, stream, dp.tasks)          # ends with gpuos_wait: the step is complete
            dt += time.perf_counter() - t0
            # between steps, not timed: the table back to its initial binding, the latency log read out
            _reset_swaps(rt, stream)
            if len(stream) <= (1 << 20):
                c = rt.completions(first, len(stream))
                lat.append((c["t_done_ns"] - c["t_submit_ns"]).astype(np.int64))
        q = rt.peek_queue()
        wg, push = q.workgroups, q.push_ring
    lat = np.concatenate(lat) if lat else np.zeros(0, np.int64)
    return dict(tasks_per_s=steps * len(stream) / dt, seconds=dt, p50_us=percentile_us(lat, 50),
                p99_us=percentile_us(lat, 99), workgroups=wg, ring="device memory (host writes through the BAR)" if push
                else "host memory (device polls over PCIe)")


def _reset_swaps(rt, stream):
    """After a pass with an odd number of swaps put the table back to its initial binding."""
    if stream.swaps and len(stream.swaps) % 2 == 1:
        op = stream.swaps[0][1]
        rt.swap_op(op, stream.table[op])


def bench_multi_producer(R, stream, dp, passes=8, **cfg):
    """tasks/s of the headline stream when 1, 2, 4, 8 and 16 host threads (native threads started
    by the library) submit disjoint parts of it to ONE context at the same time, batches of 64."""
    out = {}
    n = len(stream)
    for nt in (1, 2, 4, 8, 16):
        with R.Runtime(0, harvester_thread=1, idle_exit_ms=60000, **KNOBS, **cfg) as rt:
            rt.register_table(stream.table)
            rt.submit_from_threads(dp.tasks, nt, 64, 1)
            rt.wait()
            t0 = time.perf_counter()
            rt.submit_from_threads(dp.tasks, nt, 64, passes)
            rt.wait()
            dt = time.perf_counter() - t0
        out["threads_%d" % nt] = passes * n / dt
    return out


def bench_program(R, s5, dp5, impl5, n_tasks=1500):
    """The ADD tasks of the bandwidth stream with ADD bound to the built-in implementation, to a
    one-instruction program and to a six-instruction program, each program served as native code
    (compiled at run time into the second resident worker kernel) and interpreted by the resident
    kernel: what an operator added at run time costs when it is bound by memory.  GB/s by the wall
    time of submit + wait (the kernels' lifetimes also hold the run-time compilation).  The native legs
    run with 2 + 1 workgroups per compute unit (what a context with workgroups_per_cu = 2 gets: the
    fourth place stays free for other kernels), and with 3 + 1 and 2 + 2, which fill the compute units."""
    from paper_2604_17861_amd import streams as S
    idx = np.nonzero(impl5 == S.IMPL["ADD"])[0][:n_tasks]
    sub = dp5.tasks[idx].copy()
    sub["dep"] = 0
    nbytes = int(R.task_bytes(dp5.tasks[idx], impl5[idx]).sum())
    out = {}
    one = S.program(("ADD", 0, 0, 1))
    six = S.program(("SUB", 4, 0, 1), ("MUL", 4, 4, 3), ("ABS", 4, 4), ("IMM", 5, 1.0), ("ADD", 4, 4, 5), ("DIV", 0, 0, 4))
    legs = [("builtin_add_gbps", None, {}), ("builtin_add_2wg_gbps", None, dict(workgroups_per_cu=2)),
            ("program_add_1_instr_2plus1wg_gbps", one, dict(workgroups_per_cu=2)),
            ("program_6_instr_2plus1wg_gbps", six, dict(workgroups_per_cu=2)),
            ("program_6_instr_3plus1wg_gbps", six, dict(jit_workgroups_per_cu=1)),
            ("program_6_instr_2plus2wg_gbps", six, dict(workgroups_per_cu=2, jit_workgroups_per_cu=2)),
            ("program_add_1_instr_interpreted_gbps", one, dict(jit_mode=2)), ("program_6_instr_interpreted_gbps", six, dict(jit_mode=2))]
    for label, code, cfg in legs:
        with R.Runtime(0, idle_exit_ms=60000, **{**KNOBS, **cfg}) as rt:
            table = dict(s5.table)
            if code is not None:
                table[S.OP["ADD"]] = rt.define_program(code, 2)
            rt.register_table(table)
            native = rt.native_info()
            if code is not None and not cfg.get("jit_mode"):
                out["native_path"] = dict(live=native["native"], workgroups=native["workgroups"], why=native["why"],
                                          last_compile_ms=native["compile_us"] / 1e3)
            rt.submit_from_threads(sub[:128], 1, 64, 1)        # warm-up: both kernels have run once
            rt.wait()
            t0 = time.perf_counter()
            rt.submit_from_threads(sub, 1, 64, 1)
            rt.wait()
            out[label] = nbytes / (time.perf_counter() - t0) / 1e9
    # In these legs every task is a program task, so only the run-time kernel's workgroups work: one per
    # compute unit streams 4.6-4.8 TB/s whatever it executes, two stream what two of the library's do.
    out["program_6_instr_gbps"] = out["program_6_instr_2plus2wg_gbps"]
    out["program_6_instr_gbps_note"] = "2 + 2 workgroups per compute unit; to be read against builtin_add_2wg_gbps"
    out["native_6_instr_vs_builtin"] = out["program_6_instr_2plus2wg_gbps"] / out["builtin_add_2wg_gbps"]
    return out


def bench_dispatch(steps=2000):
    """Eager PyTorch code (a chain of relu(t * c + b) on 1,024-element tensors: 3 small operations
    per step) on PyTorch's own launch path and under the dispatch filter, which turns every one of
    them into a task.  The filter's hook is Python: this leg shows what the integration layer costs,
    not what the queue can do."""
    import torch
    from paper_2604_17861_amd.dispatch import GpuosMode
    g = torch.Generator().manual_seed(0)
    a = torch.randn(32, 32, generator=g).to("cuda:0")
    b = torch.randn(32, 32, generator=g).to("cuda:0")

    def chain(n):
        t = a
        for _ in range(n):
            t = torch.relu(t * 0.99 + b)
        return t
    stream = torch.cuda.current_stream()
    chain(200)
    stream.synchronize()
    t0 = time.perf_counter()
    want = chain(steps)
    stream.synchronize()
    eager = 3 * steps / (time.perf_counter() - t0)
    mode = GpuosMode(idle_exit_ms=60000)
    try:
        with mode:
            chain(200)
        t0 = time.perf_counter()
        with mode:
            got = chain(steps)                       # leaving the block waits for the last task
        routed = 3 * steps / (time.perf_counter() - t0)
        same = bool(torch.equal(got.cpu(), want.cpu()))
        st = {k: v for k, v in mode.stats.items() if k != "by_op"}
    finally:
        mode.close()
    return dict(eager_ops_per_s=eager, filtered_ops_per_s=routed, bit_identical=same, stats=st)


def bench_pingpong(R, stream, dp, n=5000, **cfg):
    """Unloaded latency: one task at a time, timed inside the library (gpuos_run_serial), the same
    way the per-launch path times launch + synchronize."""
    with R.Runtime(0, idle_exit_ms=60000, **KNOBS, **cfg) as rt:
        rt.register_table(stream.table)
        rt.run_serial(dp.tasks, 0, min(200, len(stream)))
        lat = np.concatenate([rt.run_serial(dp.tasks, 0, min(len(stream), n - k)) for k in range(0, n, len(stream))])
    return percentile_us(lat, 50), percentile_us(lat, 99)


def bench_roofline(R, stream, dp, impls):
    """The persistent kernel alone over the bandwidth stream: one worker lifetime that holds
    nothing but this stream, timed by HIP events on the worker's own stream."""
    nbytes = int(R.task_bytes(dp.tasks, impls).sum())
    with R.Runtime(0, idle_exit_ms=60000, **KNOBS) as rt:
        rt.register_table(stream.table)
        t0 = time.perf_counter()
        submit_pass(rt, stream, dp.tasks)
        wall = time.perf_counter() - t0
        rt.stop_worker()
        kernel_ms = rt.worker_elapsed_ms()
        wg = rt.peek_queue().workgroups
    return dict(bytes=nbytes, wall_s=wall, kernel_ms=kernel_ms, workgroups=wg)


def source_hash():
    """A hash of the sources libgpuos.so is built from: a counter profile under profiles/ is only
    quoted for the kernels it was taken with."""
    import hashlib
    h = hashlib.sha1()
    csrc = os.path.join(ROOT, "paper_2604_17861_amd", "csrc")
    for path in sorted(os.path.join(csrc, f) for f in os.listdir(csrc) if f.endswith((".hip", ".cpp", ".h"))) + [
            os.path.join(ROOT, "include", "gpuos.h")]:
        with open(path, "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def measured_traffic(n_tasks):
    """HBM bytes of the persistent kernel over the bandwidth stream as measured with rocprofv3
    counters (summary under profiles/, from two --pmc runs scaled by a copy kernel of known size).
    Returns (bytes, note): bytes is None unless a measurement for this task count AND for the
    sources this library was built from is on file (the summary records their hash)."""
    path = os.path.join(ROOT, "profiles", "gpuos_worker_kernel_config5_hbm_traffic.md")
    here = source_hash()
    found, taken = None, None
    try:
        for line in open(path):
            f = line.split()
            if len(f) == 4 and f[0] == "tasks:" and f[2] == "hbm_bytes_per_launch:" and int(f[1]) == n_tasks:
                found = int(f[3])
            if len(f) == 2 and f[0] == "source_hash:":
                taken = f[1]
    except (OSError, ValueError):
        pass
    rel = "profiles/gpuos_worker_kernel_config5_hbm_traffic.md"
    if found is None:
        return None, "no counter measurement for %d tasks in %s" % (n_tasks, rel)
    if taken != here:
        return None, "%s was taken with sources %s, this library is built from %s: not quoted" % (rel, taken, here)
    return found, "rocprofv3 FETCH_SIZE + WRITE_SIZE (separate runs, scaled by a copy kernel), %s, sources %s" % (rel, here)


def time_oracle_subsample(stream, every, seconds, label):
    """The CPU oracle on every `every`-th task of a stream (seeded: the stream is), one core, for at
    most `seconds`: tasks/s and algorithmic GB/s over what it got through."""
    import oracle
    from paper_2604_17861_amd import runtime as R
    host_arrays = [np.array(p.host_image(), dtype=np.uint8, copy=True) for p in stream.pools]
    tasks = stream.materialize([a.ctypes.data for a in host_arrays])
    impl = stream.impl_for()
    idx = np.arange(0, len(stream), every)
    nbytes = R.task_bytes(tasks[idx], impl[idx])
    L = oracle.lib()
    done, moved = 0, 0
    t0 = time.perf_counter()
    for k, i in enumerate(idx):
        L.orc_run_task(tasks.ctypes.data + int(i) * tasks.dtype.itemsize, int(impl[i]), 0)
        done += 1
        moved += int(nbytes[k])
        if time.perf_counter() - t0 > seconds:
            break
    dt = time.perf_counter() - t0
    return dict(tasks_per_s=done / dt, gbps=moved / dt / 1e9, cores=1, kind="oracle",
                sample="%s: every %dth task, %d of the %d sampled tasks in %.1f s (time-boxed)" % (label, every, done, len(idx), dt))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--skip-extras", action="store_true", help="only the headline stream and the roofline leg")
    ap.add_argument("--report", default="", help="directory for one JSON report per configuration")
    ap.add_argument("--only-roofline", action="store_true",
                    help="run nothing but the bandwidth stream through the persistent kernel (for profiler runs)")
    ap.add_argument("--only-config3", action="store_true",
                    help="run nothing but the third configuration (chains, then one fused task per chain) through the "
                         "persistent kernel, one worker lifetime each (for profiler runs)")
    ap.add_argument("--only-transposed", action="store_true",
                    help="only a stream of elementwise tasks over transposed matrices (the LDS-tiled path), one worker lifetime")
    ap.add_argument("--only-strided", action="store_true",
                    help="run nothing but 2,000 elementwise tasks over stride-2 inputs (1M elements each) through the "
                         "persistent kernel (for profiler runs: traffic of the LDS-staged gather path)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run one ordinary COPY kernel over 1 GiB (counter calibration for profiler runs) and exit")
    ap.add_argument("--cfg5-tasks", type=int, default=20000)
    ap.add_argument("--cfg4-tasks", type=int, default=1000000)
    ap.add_argument("--workgroups-per-cu", type=int, default=0, help="0: the library's default")
    ap.add_argument("--chunk-elems", type=int, default=0, help="0: the library's default")
    ap.add_argument("--cpu-seconds", type=float, default=10.0, help="CPU time given to the oracle baseline")
    args = ap.parse_args()
    if args.workgroups_per_cu:
        KNOBS["workgroups_per_cu"] = args.workgroups_per_cu
    if args.chunk_elems:
        KNOBS["chunk_elems"] = args.chunk_elems
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU (one ring, one persistent kernel and one operator table "
                 "per GPU; there is no multi-GPU path to measure). Use --gpus 1.")

    import torch
    from paper_2604_17861_amd import runtime as R
    from paper_2604_17861_amd import streams as S

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU (the HIP path has no CPU fallback)")
    R.lib()
    prop = torch.cuda.get_device_properties(0)
    log("device:", prop.name, "CUs:", prop.multi_processor_count, "mem GiB: %.0f" % (prop.total_memory / 2 ** 30))
    log("host cores:", os.cpu_count(), "affinity:", len(os.sched_getaffinity(0)))

    if args.copy_calibration:
        n = 1 << 28                                            # 1 GiB of fp32 in, 1 GiB out
        src = torch.zeros(n, dtype=torch.float32, device="cuda:0")
        dst = torch.empty(n, dtype=torch.float32, device="cuda:0")
        torch.cuda.synchronize()
        t, pool_of = S.new_tasks(1)
        S.set_head(t, 0, S.OP["COPY"], [n], 1)
        S.set_tensor(t, pool_of, 0, 0, 0, src.data_ptr(), [1], S.F32)
        S.set_tensor(t, pool_of, 0, 3, 0, dst.data_ptr(), [1], S.F32)
        for _ in range(3):
            secs, _ = R.launch_per_op(t, S.default_table())
        print(json.dumps(dict(calibration="one gpuos_single_task_kernel COPY launch", read_bytes=4 * n, write_bytes=4 * n,
                              seconds=secs, gbps=8 * n / secs / 1e9)), flush=True)
        return

    out = {}
    if args.only_roofline:
        s5 = S.config5(n_tasks=args.cfg5_tasks)
        dp5 = DevicePools(s5, torch)
        rf = bench_roofline(R, s5, dp5, s5.impl_for())
        achieved = rf["bytes"] / (rf["kernel_ms"] * 1e-3) / 1e9
        print(json.dumps(dict(workload="config5: %d bandwidth tasks" % len(s5), roofline=dict(
            bound="hbm", achieved=achieved, peak=HBM_PEAK_GBPS, unit="GB/s", frac=achieved / HBM_PEAK_GBPS,
            kernel="gpuos_worker_kernel", kernel_ms=rf["kernel_ms"], algorithmic_bytes=rf["bytes"]))), flush=True)
        return
    if args.only_config3:
        res3 = {}
        for name, s3 in (("chains", S.config3()), ("fused", S.config3_fused())):
            dp3 = DevicePools(s3, torch)
            rf = bench_roofline(R, s3, dp3, s3.impl_for())
            res3[name] = dict(tasks=len(s3), kernel_ms=rf["kernel_ms"], algorithmic_bytes=rf["bytes"],
                              gbps=rf["bytes"] / (rf["kernel_ms"] * 1e-3) / 1e9, workgroups=rf["workgroups"])
            del dp3
        print(json.dumps(dict(workload="config3: 2,000 softmax chains of six tasks, then the same as one fused task per chain",
                              **res3)), flush=True)
        return
    if args.only_transposed:
        n, side = 2000, 1024
        numel = side * side
        src = torch.randn(8 * numel, dtype=torch.float32, device="cuda:0")
        dst = torch.empty(8 * numel, dtype=torch.float32, device="cuda:0")
        torch.cuda.synchronize()
        t, pool_of = S.new_tasks(n)
        for i in range(n):                                     # out[r, c] = 0.5 * x[c, r]: eight input / output regions in turn
            S.set_head(t, i, S.OP["SCALE"], [side, side], 1, alpha=0.5)
            S.set_tensor(t, pool_of, i, 0, 0, src.data_ptr() + (i % 8) * numel * 4, [1, side], S.F32)
            S.set_tensor(t, pool_of, i, 3, 0, dst.data_ptr() + (i % 8) * numel * 4, [side, 1], S.F32)
        path = R.task_plan(t, 0, S.IMPL["SCALE"])[0]
        with R.Runtime(0, idle_exit_ms=60000, **KNOBS) as rt:
            rt.register_table(S.default_table())
            rt.submit_from_threads(t, 1, 64, 1)
            rt.wait()
            rt.stop_worker()
            kernel_ms = rt.worker_elapsed_ms()
        print(json.dumps(dict(workload="%d SCALE tasks over the transposed view of a %d x %d fp32 matrix" % (n, side, side), path=path,
                              algorithmic_bytes=n * numel * 8, kernel_ms=kernel_ms, gbps=n * numel * 8 / (kernel_ms * 1e-3) / 1e9)), flush=True)
        return
    if args.only_strided:
        n, numel = 2000, 1 << 20
        src = torch.randn(8 * 2 * numel + 64, dtype=torch.float32, device="cuda:0")
        dst = torch.empty(8 * numel, dtype=torch.float32, device="cuda:0")
        torch.cuda.synchronize()
        t, pool_of = S.new_tasks(n)
        for i in range(n):                                     # out[k] = 0.5 * x[2k]: eight input / output regions in turn
            S.set_head(t, i, S.OP["SCALE"], [numel], 1, alpha=0.5)
            S.set_tensor(t, pool_of, i, 0, 0, src.data_ptr() + (i % 8) * 2 * numel * 4, [2], S.F32)
            S.set_tensor(t, pool_of, i, 3, 0, dst.data_ptr() + (i % 8) * numel * 4, [1], S.F32)
        path = R.task_plan(t, 0, S.IMPL["SCALE"])[0]
        with R.Runtime(0, idle_exit_ms=60000, **KNOBS) as rt:
            rt.register_table(S.default_table())
            t0 = time.perf_counter()
            rt.submit_from_threads(t, 1, 64, 1)
            rt.wait()
            wall = time.perf_counter() - t0
            rt.stop_worker()
            kernel_ms = rt.worker_elapsed_ms()
        # algorithmic bytes: the elements read and the elements written (4 + 4 bytes per output element)
        print(json.dumps(dict(workload="%d SCALE tasks, %d fp32 elements each, input stride 2" % (n, numel), path=path,
                              algorithmic_bytes=n * numel * 8, covering_span_bytes=n * numel * 12, kernel_ms=kernel_ms, wall_s=wall,
                              gbps=n * numel * 8 / (kernel_ms * 1e-3) / 1e9)), flush=True)
        return
    # ---- headline: second configuration --------------------------------------------------
    s2 = S.config2()
    dp2 = DevicePools(s2, torch)
    res = bench_persistent(R, s2, dp2, args.steps, args.warmup)
    log("config2 persistent:", res)
    secs, _ = R.launch_per_op(dp2.tasks, s2.table)                       # warm-up pass
    t0 = time.perf_counter()
    for _ in range(max(1, args.steps // 4)):
        secs, _ = R.launch_per_op(dp2.tasks, s2.table)
    per_launch_tps = max(1, args.steps // 4) * len(s2) / (time.perf_counter() - t0)
    _, lat = R.launch_per_op(dp2.tasks, s2.table, sync_each=True, count=3000)
    log("config2 per-launch: %.0f tasks/s, p50 %.1f us" % (per_launch_tps, percentile_us(lat, 50)))
    # the like-for-like of the per-launch latency (launch + synchronize, one task at a time): the same
    # tasks through the persistent kernel one at a time (submit + wait)
    u50, u99 = bench_pingpong(R, s2, dp2, n=3000)
    log("config2 one task at a time: persistent p50 %.1f us, p99 %.1f us" % (u50, u99))
    out.update(value=res["tasks_per_s"], ms_per_step=1e3 * res["seconds"] / args.steps,
               per_launch_tasks_per_s=per_launch_tps, speedup_vs_per_launch=res["tasks_per_s"] / per_launch_tps,
               p50_us=u50, p99_us=u99, loaded_p50_us=res["p50_us"], loaded_p99_us=res["p99_us"],
               per_launch_p50_us=percentile_us(lat, 50), per_launch_p99_us=percentile_us(lat, 99),
               workgroups=res["workgroups"], ring=res["ring"])

    extras = {}
    if not args.skip_extras:
        # ---- unloaded latency: one task at a time ---------------------------------------
        s1 = S.config1()
        dp1 = DevicePools(s1, torch)
        p50, p99 = bench_pingpong(R, s1, dp1)
        _, lat1 = R.launch_per_op(dp1.tasks, s1.table, sync_each=True)
        extras["pingpong"] = dict(persistent_p50_us=p50, persistent_p99_us=p99,
                                  per_launch_p50_us=percentile_us(lat1, 50), per_launch_p99_us=percentile_us(lat1, 99))
        log("pingpong:", extras["pingpong"])
        # ---- the other ring placement: host memory polled by the device over PCIe ------------------
        pp50, pp99 = bench_pingpong(R, s1, dp1, push_ring=0)
        rpull = bench_persistent(R, s2, dp2, max(4, args.steps // 2), 1, push_ring=0)
        extras["host_ring_mode"] = dict(config2_tasks_per_s=rpull["tasks_per_s"], pingpong_p50_us=pp50, pingpong_p99_us=pp99)
        log("ring in host memory:", extras["host_ring_mode"])
        # ---- several producer threads on one ring (ticket reservation is serialised, packing is not) ----
        extras["multi_producer"] = bench_multi_producer(R, s2, dp2)
        log("multi producer:", extras["multi_producer"])
        # ---- first configuration ----------------------------------------------------------
        r1 = bench_persistent(R, s1, dp1, max(20, args.steps), args.warmup)
        R.launch_per_op(dp1.tasks, s1.table)
        t0 = time.perf_counter()
        for _ in range(10):
            R.launch_per_op(dp1.tasks, s1.table)
        pl1 = 10 * len(s1) / (time.perf_counter() - t0)
        extras["config1"] = dict(persistent_tasks_per_s=r1["tasks_per_s"], per_launch_tasks_per_s=pl1,
                                 speedup=r1["tasks_per_s"] / pl1, p50_us=r1["p50_us"], p99_us=r1["p99_us"])
        log("config1:", extras["config1"])
        del dp1
        # ---- third configuration (dependent softmax chains) -------------------------------------
        s3 = S.config3()
        dp3 = DevicePools(s3, torch)
        b3 = int(R.task_bytes(dp3.tasks, s3.impl_for()).sum())
        r3 = bench_persistent(R, s3, dp3, 2, 1)
        R.launch_per_op(dp3.tasks, s3.table, count=1200)
        t0 = time.perf_counter()
        R.launch_per_op(dp3.tasks, s3.table)
        pl3 = time.perf_counter() - t0
        extras["config3"] = dict(persistent_tasks_per_s=r3["tasks_per_s"], per_launch_tasks_per_s=len(s3) / pl3,
                                 speedup=r3["tasks_per_s"] / (len(s3) / pl3), persistent_gbps=b3 * r3["tasks_per_s"] / len(s3) / 1e9,
                                 per_launch_gbps=b3 / pl3 / 1e9, chains=len(s3) // 6)
        log("config3:", extras["config3"])
        del dp3
        # ---- the same softmax as ONE fused task per chain (row operation, rows in registers) -------
        s3f = S.config3_fused()
        dp3f = DevicePools(s3f, torch)
        b3f = int(R.task_bytes(dp3f.tasks, s3f.impl_for()).sum())
        r3f = bench_persistent(R, s3f, dp3f, 3, 1)
        R.launch_per_op(dp3f.tasks, s3f.table, count=200)
        t0 = time.perf_counter()
        R.launch_per_op(dp3f.tasks, s3f.table)
        pl3f = time.perf_counter() - t0
        extras["config3_fused"] = dict(persistent_softmax_per_s=r3f["tasks_per_s"], per_launch_softmax_per_s=len(s3f) / pl3f,
                                       chain_softmax_per_s=r3["tasks_per_s"] / 6,
                                       speedup_vs_chain=r3f["tasks_per_s"] / (r3["tasks_per_s"] / 6),
                                       persistent_gbps=b3f * r3f["tasks_per_s"] / len(s3f) / 1e9,
                                       per_launch_gbps=b3f / pl3f / 1e9, tasks=len(s3f))
        log("config3 fused:", extras["config3_fused"])
        del dp3f
        # ---- the paper's micro-benchmark shape: sequences of 100 dependent small operations ----------
        # The tasks between the oldest incomplete ticket and the newest submitted one are what is in
        # flight, so the ring's capacity bounds the number of sequences that advance at the same time:
        # issued one after the other, the default ring of 4,096 holds 41 sequences of 100, one of
        # 16,384 slots 164.  Both are reported for that order.
        seq = {}
        for il in (1, 16, 256):
            sq = S.sequences(n_seq=1000, length=100, interleave=il)
            dpq = DevicePools(sq, torch)
            rq = bench_persistent(R, sq, dpq, 2, 1, capacity=16384)
            seq["persistent_interleave_%d_tasks_per_s" % il] = rq["tasks_per_s"]
            if il == 1:
                seq["persistent_interleave_1_ring_4096_tasks_per_s"] = bench_persistent(R, sq, dpq, 2, 1)["tasks_per_s"]
            if il == 1:
                t0 = time.perf_counter()
                R.launch_per_op(dpq.tasks, sq.table)
                seq["per_launch_tasks_per_s"] = len(sq) / (time.perf_counter() - t0)
            del dpq
        seq["ring_slots"] = 16384
        extras["sequences_100x1000"] = seq
        log("sequences of 100 dependent operations x 1000:", seq)
        # ---- fourth configuration (hot swaps while running) -----------------------------------
        s4 = S.config4(n_tasks=args.cfg4_tasks)
        dp4 = DevicePools(s4, torch)
        r4 = bench_persistent(R, s4, dp4, 2, 1)          # the first pass faults in 1 M descriptors and the log
        t0 = time.perf_counter()
        R.launch_per_op(dp4.tasks, s4.table, count=min(len(s4), 200000))
        pl4 = min(len(s4), 200000) / (time.perf_counter() - t0)
        extras["config4"] = dict(persistent_tasks_per_s=r4["tasks_per_s"], per_launch_tasks_per_s=pl4,
                                 speedup=r4["tasks_per_s"] / pl4, swaps=len(s4.swaps), tasks=len(s4),
                                 p50_us=r4["p50_us"], p99_us=r4["p99_us"])
        log("config4:", extras["config4"])
        del dp4
    del dp2

    # ---- roofline: fifth configuration through the persistent kernel ---------------------------
    s5 = S.config5(n_tasks=args.cfg5_tasks)
    dp5 = DevicePools(s5, torch)
    impl5 = s5.impl_for()
    rf = bench_roofline(R, s5, dp5, impl5)
    achieved = rf["bytes"] / (rf["kernel_ms"] * 1e-3) / 1e9
    log("config5 roofline:", rf, "-> %.1f GB/s by kernel time, %.1f GB/s by wall" % (achieved, rf["bytes"] / rf["wall_s"] / 1e9))
    t0 = time.perf_counter()
    R.launch_per_op(dp5.tasks, s5.table, count=min(len(s5), 4000))
    pl5 = sum(R.task_bytes(dp5.tasks[: min(len(s5), 4000)], impl5)) / (time.perf_counter() - t0) / 1e9
    extras["config5"] = dict(persistent_gbps_wall=rf["bytes"] / rf["wall_s"] / 1e9, per_launch_gbps=float(pl5),
                             tasks=len(s5), tasks_per_s=len(s5) / rf["wall_s"])
    roofline = dict(bound="hbm", achieved=achieved, peak=HBM_PEAK_GBPS, unit="GB/s", frac=achieved / HBM_PEAK_GBPS,
                    traffic=None, kernel="gpuos_worker_kernel", kernel_ms=rf["kernel_ms"],
                    algorithmic_bytes=rf["bytes"], workload="config5: %d bandwidth tasks" % len(s5))
    roofline["traffic"], roofline["traffic_note"] = measured_traffic(len(s5))
    if not args.skip_extras:
        # ---- an operator defined at run time as a program against the built-in it re-implements -----
        # (side legs after the figures of record: a failure in one is reported in its place and does
        # not cost the line)
        for name, leg in (("operator_program", lambda: bench_program(R, s5, dp5, impl5)), ("torch_dispatch", bench_dispatch)):
            try:
                extras[name] = leg()
            except Exception as e:                                  # noqa: BLE001
                extras[name] = dict(error=repr(e))
            log(name + ":", extras[name])
    del dp5

    # ---- CPU oracle on a bounded sample of the headline stream (one core) ------------------------
    import oracle
    host_arrays = [np.array(p.host_image(), dtype=np.uint8, copy=True) for p in s2.pools]
    hp_tasks = s2.materialize([a.ctypes.data for a in host_arrays])
    impl2 = s2.impl_for()
    L = oracle.lib()
    t0 = time.perf_counter()
    done = 0
    while time.perf_counter() - t0 < args.cpu_seconds:        # whole passes over the stream, in task order
        for i in range(len(s2)):
            L.orc_run_task(hp_tasks.ctypes.data + i * hp_tasks.dtype.itemsize, int(impl2[i]), 0)
        done += len(s2)
    cpu_s = time.perf_counter() - t0
    cpu_baseline = dict(value=done / cpu_s, unit="tasks/s", cores=1, kind="oracle",
                        sample="%d passes over the second configuration's 10,000-task stream (%d tasks, %.1f s)" % (
                            done // len(s2), done, cpu_s))
    log("cpu oracle:", cpu_baseline)
    if not args.skip_extras:
        # the oracle on a seeded 1-in-20 subsample of the fourth and fifth configurations (time-boxed: the
        # fifth one's tasks have up to 16M elements, the oracle walks them one element at a time)
        del host_arrays, hp_tasks
        extras["cpu_oracle_config4"] = time_oracle_subsample(S.config4(n_tasks=args.cfg4_tasks), 20, args.cpu_seconds / 2, "config4")
        extras["cpu_oracle_config5"] = time_oracle_subsample(S.config5(n_tasks=args.cfg5_tasks), 20, args.cpu_seconds, "config5")
        log("cpu oracle, configs 4 and 5:", extras["cpu_oracle_config4"], extras["cpu_oracle_config5"])

    line = dict(metric="small-op tasks/sec and p50 submit->done latency vs per-op launch; HBM GB/s",
                value=out["value"], unit="tasks/s", n_gpus=1, steps=args.steps, warmup=args.warmup,
                ms_per_step=out["ms_per_step"], higher_is_better=True, scaling="weak", vs_baseline=None,
                dtype="f32", data="synthetic",
                config=dict(workload="config2: 10,000 mixed elementwise tasks (fp32/fp16/bf16 50/25/25, numel "
                                     "log-uniform 256..65536, 30% strided inputs, 20% broadcast), batches of 64",
                            queue_capacity=4096, workgroups=out["workgroups"], ring=out["ring"]),
                per_launch_tasks_per_s=out["per_launch_tasks_per_s"],
                speedup_vs_per_launch=out["speedup_vs_per_launch"],
                p50_us=out["p50_us"], p99_us=out["p99_us"], per_launch_p50_us=out["per_launch_p50_us"],
                per_launch_p99_us=out["per_launch_p99_us"],
                loaded_p50_us=out["loaded_p50_us"], loaded_p99_us=out["loaded_p99_us"],
                latency_note="p50_us / p99_us and per_launch_*: submit -> completion seen by the host, one task of the "
                             "stream at a time, on both paths; loaded_*: every task of the timed steps, submitted flat "
                             "out in batches of 64, queueing in a ring of 4096 included",
                extras=extras,
                roofline=roofline, cpu_baseline=cpu_baseline)
    print(json.dumps(line), flush=True)
    if args.report:
        write_reports(args.report, R, line)


def host_info():
    model = ""
    try:
        with open("/proc/cpuinfo") as f:
            for ln in f:
                if ln.startswith("model name"):
                    model = ln.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    return dict(nproc=os.cpu_count(), usable_cpus=len(os.sched_getaffinity(0)), cpu_model=model)


def common_cus(R):
    return int(R.device_info(0)["compute_units"])


def write_reports(directory, R, line):
    """One JSON per configuration: what was run, on what, with which knobs, and the figures measured
    by this process.  Parity figures are written by the GPU tests of the full configurations (they
    own the comparison with the oracle), beside these files."""
    os.makedirs(directory, exist_ok=True)
    common = dict(device=R.device_info(0), host=host_info(),
                  knobs=dict(queue_capacity=4096, workgroups=line["config"]["workgroups"], threads_per_workgroup=256,
                             workgroups_per_cu=line["config"]["workgroups"] // common_cus(R)), hbm_peak_gbps=HBM_PEAK_GBPS)
    ex = line["extras"]
    per = {
        "config2": dict(seed=1, tasks=10000, persistent_tasks_per_s=line["value"],
                        per_launch_tasks_per_s=line["per_launch_tasks_per_s"], speedup=line["speedup_vs_per_launch"],
                        p50_us=line["p50_us"], p99_us=line["p99_us"], per_launch_p50_us=line["per_launch_p50_us"],
                        per_launch_p99_us=line["per_launch_p99_us"], loaded_p50_us=line["loaded_p50_us"],
                        loaded_p99_us=line["loaded_p99_us"], latency_note=line["latency_note"],
                        oracle_tasks_per_s=line["cpu_baseline"]["value"],
                        oracle_sample=line["cpu_baseline"]["sample"], host_ring_mode=ex.get("host_ring_mode"), multi_producer=ex.get("multi_producer")),
        "config1": dict(seed=0, tasks=1000, pingpong=ex.get("pingpong"), **ex.get("config1", {})),
        "config3": dict(seed=2, tasks=12000, **ex.get("config3", {})),
        "config4": dict(seed=3, **ex.get("config4", {})),
        "config5": dict(seed=4, roofline=line["roofline"], **ex.get("config5", {})),
    }
    for name, body in per.items():
        with open(os.path.join(directory, "perf_%s.json" % name), "w") as f:
            json.dump(dict(config=name, **common, **body), f, indent=1)


if __name__ == "__main__":
    main()
