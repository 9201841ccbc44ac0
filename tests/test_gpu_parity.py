"""GPU parity tests: the HIP path, called through the C ABI binding, against the CPU oracle,
element by element on the same seeded inputs."""
import numpy as np
import pytest

from paper_2604_17861_amd import runtime as R
from paper_2604_17861_amd import streams as S

pytestmark = pytest.mark.gpu


def _run_and_check(stream, capacity=0, **cfg):
    from gpu_helpers import DevicePools, run_stream, compare_with_oracle
    print("case", stream.name, "tasks", len(stream), flush=True)
    dp = DevicePools(stream)
    with R.Runtime(capacity, idle_exit_ms=20000, wait_timeout_ms=20000, **cfg) as rt:
        rt.register_table(stream.table, stream.programs)
        t0 = run_stream(stream, rt, dp)
        comps = rt.completions(t0, len(stream))
        assert rt.worker_alive()
    assert np.all(comps["status"] == 0), comps["status"][comps["status"] != 0][:10]
    assert np.array_equal(comps["ticket"], np.arange(t0, t0 + len(stream), dtype=np.uint64))
    imgs = dp.download()
    return compare_with_oracle(stream, imgs, versions=comps["op_version"]), comps


def test_config1_full_bit_exact():
    print("config1: 1000 x fp32 ADD n=1024", flush=True)
    stats, comps = _run_and_check(S.config1())
    assert stats["max_ulp"] == 0 and stats["elements"] == 1000 * 1024
    from gpu_helpers import parity_report
    parity_report("config1", [stats], seed=0, tasks=1000)
    assert np.all(comps["op_version"] == 1)


import parity_cases as C


@pytest.mark.parametrize("code", [S.F32, S.F16, S.BF16])
def test_every_elementwise_op_contiguous(code):
    stats, _ = _run_and_check(C.elementwise_contiguous(code))
    print(stats, flush=True)


@pytest.mark.parametrize("trace_entries", [0, 4096])
def test_lone_tasks_take_the_dispatchers_short_cut(trace_entries):
    """Tasks submitted one at a time, each after the previous one has completed, are resolved,
    mirrored and published by the dispatcher's first wavefront alone (no batch pass): contiguous,
    gathered, transposed and reduction tasks of one to several chunks, every float dtype, with and
    without tracepoints; then a burst, so that the short cut and the batch pass alternate.  Results
    against the oracle as for every other case; the dispatcher's counters show one pass per task."""
    from gpu_helpers import DevicePools, compare_with_oracle
    streams = [C.elementwise_contiguous(S.F32), C.staged_gathers(), C.transposed_2d(), C.reductions(), C.row_operations()]
    for stream in streams:
        n = 2 * len(stream) // 3
        print("lone tasks of", stream.name, n, flush=True)
        dp = DevicePools(stream)
        with R.Runtime(0, idle_exit_ms=20000, wait_timeout_ms=20000, trace_entries=trace_entries) as rt:
            rt.register_table(stream.table, stream.programs)
            lat = rt.run_serial(dp.tasks, 0, n)                      # submit + wait, one by one
            if n < len(stream):
                rt.submit(dp.tasks, n, len(stream) - n)              # the rest as one burst
                rt.wait()
            comps = rt.completions(0, len(stream))
            rt.stop_worker()
            st = rt.worker_stats()
        assert np.all(comps["status"] == 0)
        assert st["disp_records"] == len(stream) and st["disp_batches"] >= n    # a pass of its own for every lone task
        stats = compare_with_oracle(stream, dp.download(), versions=comps["op_version"])
        print(stats, "p50 %.1f us" % (np.median(lat) / 1e3), flush=True)


@pytest.mark.parametrize("code", [S.F16, S.BF16])
def test_all_16bit_patterns_through_unary_ops(code):
    stats, _ = _run_and_check(C.all_16bit_patterns(code))
    print(stats, flush=True)


@pytest.mark.parametrize("code", [S.F16, S.BF16])
def test_exponential_for_16bit_outputs_over_all_patterns(code):
    stats, _ = _run_and_check(C.sub_exp_16bit_patterns(code))
    print(stats, flush=True)
    assert stats["max_ulp"] <= 2


def test_fp32_transcendental_dense_sweep():
    stats, _ = _run_and_check(C.fp32_transcendental_sweep())
    print(stats, flush=True)
    assert stats["max_ulp"] <= 2


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_random_strided_broadcast_views(seed):
    stats, _ = _run_and_check(C.random_strided_views(seed))
    print(stats, flush=True)


def test_row_and_column_broadcast_2d_fast_path():
    stats, _ = _run_and_check(C.broadcast_2d())
    print(stats, flush=True)


def test_strided_and_broadcast_inputs_gathered_through_lds():
    stats, _ = _run_and_check(C.staged_gathers())
    print(stats, flush=True)
    assert stats["max_ulp"] <= 2


def test_transposed_views_lds_tiled_gather():
    stats, _ = _run_and_check(C.transposed_2d())
    print(stats, flush=True)


def test_degenerate_shapes_leave_everything_else_untouched():
    """Empty, one-element, six-dimensional, in-place, aliased and all-broadcast tasks (exactly rounded
    operations only): every buffer as a whole equals the oracle's byte for byte, so the results are
    right, nothing was written outside the outputs and empty tasks touched nothing."""
    from gpu_helpers import DevicePools, run_stream
    from helpers import run_oracle
    s = C.degenerate()
    dp = DevicePools(s)
    with R.Runtime(0, idle_exit_ms=20000, wait_timeout_ms=20000) as rt:
        rt.register_table(s.table)
        t0 = run_stream(s, rt, dp)
        comps = rt.completions(t0, len(s))
    assert np.all(comps["status"] == 0), comps["status"]
    gpu = dp.download()
    hp, st = run_oracle(s)                       # the whole stream in order from the same initial buffers (it has in-place tasks)
    assert np.all(st == 0)
    for k, (g, o) in enumerate(zip(gpu, hp.arrays)):
        g8, o8 = np.asarray(g).view(np.uint8).reshape(-1), np.asarray(o).view(np.uint8).reshape(-1)
        assert np.array_equal(g8, o8), "buffer %d differs at bytes %s" % (k, np.nonzero(g8 != o8)[0][:16])


@pytest.mark.parametrize("seed,capacity", [(0, 0), (1, 64), (2, 0)])
def test_random_dependency_dags_equal_sequential_execution(seed, capacity):
    """2,500 exactly rounded tasks over ten buffers with every kind of hazard between them, declared
    as dependencies: the buffers at the end equal sequential execution byte for byte, with the
    default ring and with one of 64 slots (dependencies then reach across laps of the ring)."""
    from gpu_helpers import DevicePools, run_stream
    from helpers import run_oracle
    s = C.dependency_dag(seed)
    fences = int((s.tasks["flags"] & S.FLAG_FENCE != 0).sum())
    with_deps = int((s.tasks["dep"] != 0).any(axis=1).sum())
    print("dag", seed, "tasks", len(s), "with dependencies", with_deps, "fences", fences, flush=True)
    assert with_deps > 2000 and fences > 20
    dp = DevicePools(s)
    with R.Runtime(capacity, idle_exit_ms=20000, wait_timeout_ms=20000) as rt:
        rt.register_table(s.table)
        t0 = run_stream(s, rt, dp)
        comps = rt.completions(t0, len(s))
    assert np.all(comps["status"] == 0)
    gpu = dp.download()
    hp, st = run_oracle(s)
    assert np.all(st == 0)
    for k, (g, o) in enumerate(zip(gpu, hp.arrays)):
        g8, o8 = np.asarray(g).view(np.uint8).reshape(-1), np.asarray(o).view(np.uint8).reshape(-1)
        assert np.array_equal(g8, o8), "buffer %d differs at bytes %s" % (k, np.nonzero(g8 != o8)[0][:16])


def test_held_producer_with_more_small_dependants_than_workgroups():
    """A large task held back by the dispatcher, 1,200 one-row tasks and a chain of 300 four-chunk
    links that all name it: the dispatcher publishes in dependency order (the small dependants join
    the pending list behind the held task), so no workgroup ever waits for work published after its
    own.  The buffers at the end equal sequential execution byte for byte; through the default ring
    and through one of 2,048 slots (the dependants then reach back across most of the ring); and with
    6,400 dependants, more than every workgroup's descriptor slots together could hold waiting."""
    from gpu_helpers import DevicePools, run_stream
    from helpers import run_oracle
    for s, capacity in ((C.producer_with_dependants(), 0), (C.producer_with_dependants(), 2048),
                        (C.producer_with_dependants(n_consumers=6400), 8192)):     # more dependants than 767 workgroups hold at 8 each
        hp, st = run_oracle(s)
        assert np.all(st == 0)
        print("producer_with_dependants,", len(s), "tasks, ring", capacity, flush=True)
        dp = DevicePools(s)
        with R.Runtime(capacity, idle_exit_ms=20000, wait_timeout_ms=20000) as rt:
            rt.register_table(s.table)
            t0 = run_stream(s, rt, dp)
            comps = rt.completions(t0, len(s))
            rt.stop_worker()
            held = rt.worker_stats()["disp_deferred"]
        assert np.all(comps["status"] == 0)
        assert held >= 2                      # the large dependent task and at least some of its small dependants
        gpu = dp.download()
        for k, (g, o) in enumerate(zip(gpu, hp.arrays)):
            g8, o8 = np.asarray(g).view(np.uint8).reshape(-1), np.asarray(o).view(np.uint8).reshape(-1)
            assert np.array_equal(g8, o8), "buffer %d differs at bytes %s" % (k, np.nonzero(g8 != o8)[0][:16])


def test_dependency_wait_is_bounded():
    """cfg.dep_wait_us: a workgroup that holds a small task whose dependency is still running gives
    up after the bound; the task completes with GPUOS_E_TIMEOUT and writes nothing, everything else
    runs, and the worker stays alive.  With a bound of one microsecond behind a 16M-element task
    the wait usually runs out (either outcome is legal: the bound is a safety net, not a schedule)."""
    from gpu_helpers import DevicePools, run_stream
    rng = np.random.default_rng(5)
    b = C.Builder()
    n = 1 << 24
    x = b.pool(rng.uniform(-3, 3, n).astype(np.float32))
    y = b.pool(np.zeros(n, np.float32))
    z = b.pool(np.full(1024, 7.0, np.float32))
    w = b.pool(np.zeros(1024, np.float32))
    b.add("GELU_ERF", y, [x])                                  # long: 1,024 chunks evaluated in fp64
    b.add("COPY", z, [y[:1024]], dep=(1, 0, 0))                # small and dependent: its workgroup waits
    b.add("RELU", w, [x[:1024]])                               # independent
    s = b.stream("bounded_wait")
    dp = DevicePools(s)
    with R.Runtime(0, idle_exit_ms=20000, wait_timeout_ms=20000, dep_wait_us=1) as rt:
        rt.register_table(s.table)
        t0 = run_stream(s, rt, dp, wait=False)
        rc = rt.wait(check=False)
        comps = rt.completions(t0, 3)
        assert rt.worker_alive()
    print("bounded wait: statuses", comps["status"], flush=True)
    assert comps["status"][0] == 0 and comps["status"][2] == 0
    assert comps["status"][1] in (0, R.E_TIMEOUT) and rc == comps["status"][1]
    imgs = dp.download()
    zz, yy = imgs[2].view(np.float32), imgs[1].view(np.float32)
    if comps["status"][1] == R.E_TIMEOUT:
        assert np.all(zz == 7.0)                               # it wrote nothing
    else:
        assert np.array_equal(zz, yy[:1024])
    assert np.array_equal(imgs[3].view(np.float32), np.maximum(imgs[0].view(np.float32)[:1024], 0))


@pytest.mark.parametrize("interleave", [1, 8, 64])
def test_sequences_of_dependent_small_operations(interleave):
    """The shape of the paper's elementwise micro-benchmark: sequences of dependent small operations,
    issued one after the other or several round-robin.  The buffers at the end equal sequential
    execution byte for byte whatever the interleaving."""
    from gpu_helpers import DevicePools, run_stream
    from helpers import run_oracle
    s = S.sequences(n_seq=128, length=25, interleave=interleave)
    dp = DevicePools(s)
    with R.Runtime(0, idle_exit_ms=20000, wait_timeout_ms=20000) as rt:
        rt.register_table(s.table)
        t0 = run_stream(s, rt, dp)
        comps = rt.completions(t0, len(s))
    assert np.all(comps["status"] == 0)
    gpu = dp.download()
    hp, st = run_oracle(s)
    assert np.all(st == 0)
    for k, (g, o) in enumerate(zip(gpu, hp.arrays)):
        assert np.array_equal(np.asarray(g).view(np.uint8).reshape(-1), np.asarray(o).view(np.uint8).reshape(-1)), "buffer %d differs" % k


def test_fused_row_operations():
    stats, _ = _run_and_check(C.row_operations())
    print(stats, flush=True)
    assert stats["max_red_ratio"] <= 1.0


def test_operator_programs():
    """Elementwise operators defined as programs, on contiguous / row-broadcast / transposed /
    strided / mixed-dtype operands and several chunks: programs of exactly rounded instructions are
    bit-exact, the ones with an exponential inside stay within the bound the test derives."""
    stats, _ = _run_and_check(C.operator_programs())
    print(stats, flush=True)


def test_program_swapped_in_while_the_worker_runs():
    """The paper's injection flow without stopping the kernel: tasks of a logical operator are in
    flight under its built-in implementation; a program is defined and swapped in; later tasks
    record the new version and their results are the program's."""
    from gpu_helpers import DevicePools, compare_with_oracle
    s = S.config1(n_tasks=3000, numel=4096, seed=9)
    dp = DevicePools(s)
    code = S.program(("ADD", 4, 0, 1), ("MUL", 0, 4, 4), ("IMM", 5, 0.5), ("SUB", 0, 0, 5))     # (x + y)^2 - 0.5
    with R.Runtime(0, idle_exit_ms=20000, wait_timeout_ms=20000) as rt:
        rt.register_table(s.table)
        rt.submit(dp.tasks, 0, 1000)
        impl = rt.define_program(code, 2)                 # while the first thousand are running
        assert impl == S.PROGRAM_BASE
        rt.submit(dp.tasks, 1000, 1000)
        v = rt.swap_op(S.OP["ADD"], impl)
        assert v == 2
        rt.submit(dp.tasks, 2000, 1000)
        rt.wait()
        comps = rt.completions(0, 3000)
        with pytest.raises(R.GpuosError):                 # a unary built-in cannot replace a binary operator ...
            rt.swap_op(S.OP["ADD"], S.IMPL["RELU"])
        with pytest.raises(R.GpuosError):                 # ... nor can a program that was never defined
            rt.swap_op(S.OP["ADD"], impl + 1)
        with pytest.raises(R.GpuosError):
            rt.define_program(code[:0], 2)
        log = rt.audit_log()                              # the injection is on record: what, when, from which ticket on
    assert np.all(comps["status"] == 0)
    assert list(log["kind"]) == [R.AUDIT_REGISTER] * len(s.table) + [R.AUDIT_DEFINE_PROGRAM, R.AUDIT_SWAP]
    assert log["impl_id"][-2] == impl and log["n_instr"][-2] == 4 and log["head_ticket"][-2] == 1000
    assert log["op_id"][-1] == S.OP["ADD"] and log["version"][-1] == 2 and log["head_ticket"][-1] == 2000
    assert log["code_hash"][-1] == log["code_hash"][-2] != 0 and np.all(np.diff(log["t_ns"].astype(np.int64)) >= 0)
    ver = comps["op_version"]
    assert np.all(ver[:1000] == 1) and np.all(ver[2000:] == 2) and set(np.unique(ver[1000:2000])) <= {1, 2}
    s.swaps = [(2000, S.OP["ADD"], impl)]
    s.programs = {impl: (code, 2)}
    stats = compare_with_oracle(s, dp.download(), versions=ver)
    assert stats["max_ulp"] == 0
    out = dp.download()[2].view(np.float32).reshape(3000, 4096)
    a = dp.download()[0].view(np.float32).reshape(3000, 4096)
    b = dp.download()[1].view(np.float32).reshape(3000, 4096)
    assert np.array_equal(out[2500], (a[2500] + b[2500]) ** 2 - np.float32(0.5))


def test_last_dim_reductions():
    stats, _ = _run_and_check(C.reductions())
    print(stats, flush=True)


def test_int32_ops_bit_exact():
    stats, _ = _run_and_check(C.int32_ops())
    print(stats, flush=True)


# ---- the five configurations at reduced length ---------------------------------------
def test_config2_reduced():
    stats, _ = _run_and_check(C.config2_reduced())
    print(stats, flush=True)


def test_config3_reduced_all_pairs():
    stats, _ = _run_and_check(C.config3_reduced())
    print(stats, flush=True)


def test_config3_fused_softmax_all_pairs():
    """One fused task per (B, S) pair of the third configuration, against the oracle; and against
    the six-task chain run on the same scores: the two agree to a few fp16 steps."""
    from gpu_helpers import DevicePools, run_stream
    stats, _ = _run_and_check(C.config3_fused_reduced())
    print(stats, flush=True)
    assert stats["max_red_ratio"] <= 1.0
    sf, sc = C.config3_fused_reduced(), C.config3_reduced()
    outs = []
    for s in (sf, sc):
        dp = DevicePools(s)
        with R.Runtime(0, idle_exit_ms=20000, wait_timeout_ms=20000) as rt:
            rt.register_table(s.table)
            run_stream(s, rt, dp)
        imgs = dp.download()
        res = {}
        for c in range(12):
            b, n = s.info["pairs"][int(s.info["chain_pair"][c])]
            lay = s.info["layout"][(b, n)][0]
            cnt = b * 16 * n * n
            if s is sf:
                res[(b, n)] = imgs[lay["p"]][: cnt * 2].view(np.float16).astype(np.float64)
            else:
                res[(b, n)] = imgs[lay["w"]][lay["p"]: lay["p"] + cnt * 2].view(np.float16).astype(np.float64)
        outs.append(res)
    for key in outs[0]:
        f, c = outs[0][key], outs[1][key]
        assert np.array_equal(f == 0, c == 0)
        big = c > 2.0 ** -10
        assert (np.abs(f - c)[big] / c[big]).max() <= 8 * 2.0 ** -11, key


def test_config4_reduced_hot_swap():
    """Hot swap under load: versions recorded at claim time decide which GELU the oracle evaluates;
    the version invariants hold for every task."""
    s = C.config4_reduced()
    stats, comps = _run_and_check(s)
    print(stats, flush=True)
    v = comps["op_version"].astype(np.int64)
    gelu = s.tasks["op_id"] == S.OP_GELU
    assert np.all(v[~gelu] == 1)
    n_swaps = len(s.swaps)
    assert v[gelu].min() >= 1 and v[gelu].max() <= n_swaps + 1
    for k, (t, _, _) in enumerate(s.swaps):        # submitted after swap k returned => version >= k + 2
        assert np.all(v[t:][gelu[t:]] >= k + 2), k
    assert len(np.unique(v[gelu])) == n_swaps + 1  # every version was actually used


def test_config5_reduced():
    stats, _ = _run_and_check(C.config5_reduced())
    print(stats, flush=True)


@pytest.mark.parametrize("per_cu,chunk_elems", [(1, 1024), (2, 32768), (4, 2048)])
def test_other_grid_and_chunk_sizes(per_cu, chunk_elems):
    """The number of workgroups and the cut of a task into chunks are scheduling, not arithmetic:
    the chained and the streaming configuration meet the same bars on a quarter-size grid with
    the finest chunks, on a half-size grid with coarse ones, and on the fullest grid."""
    for stream in (C.config3_reduced(), C.config5_reduced()):
        stats, _ = _run_and_check(stream, workgroups_per_cu=per_cu, chunk_elems=chunk_elems)
        print(per_cu, chunk_elems, stats, flush=True)
