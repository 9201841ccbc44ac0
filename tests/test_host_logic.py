"""CPU tests of the product's host logic: the library loads and exports the C ABI, its struct
layout matches the generator's and the oracle's, and its descriptor validation agrees with the
oracle's independent implementation on randomly damaged descriptors.  No compute call is made."""
import ctypes
import os
import re

import numpy as np

import oracle
from paper_2604_17861_amd import runtime as R
from paper_2604_17861_amd import streams as S
from helpers import HostPools
import parity_cases as C

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "gpuos.h")).read()
    declared = set(re.findall(r"\b(gpuos_[a-z_]+)\s*\(", header))
    assert declared == set(R.EXPORTS), declared ^ set(R.EXPORTS)
    L = R.lib()
    for name in declared:
        assert hasattr(L, name), name


def test_abi_layout_agrees_between_library_generator_and_oracle():
    lay = R.abi_layout()
    assert np.array_equal(lay, oracle.abi_layout())
    assert lay[0] == S.TASK_DT.itemsize and lay[7] == S.COMPLETION_DT.itemsize
    assert ctypes.sizeof(R.Config) == 72 and ctypes.sizeof(R.QueueState) == 56


def test_strerror_and_statuses():
    assert R.strerror(0) == "ok" and "ring full" in R.strerror(R.E_FULL)
    for code in range(-8, 1):
        assert R.strerror(code)


def _status(tasks, i, impl):
    b = ctypes.c_uint64()
    return R.lib().gpuos_task_bytes(tasks.ctypes.data + i * tasks.dtype.itemsize, int(impl), ctypes.byref(b)), b.value


def _damage_and_compare(s, rng, trials):
    hp = HostPools(s)
    T = hp.tasks
    impl = s.impl_for()
    n_bad = 0
    for trial in range(trials):
        i = int(rng.integers(len(T)))
        t = T[i:i + 1].copy()
        kind = int(rng.integers(13))
        if kind == 0: t["ndim"][0] = rng.integers(0, 9)
        elif kind == 1: t["n_inputs"][0] = rng.integers(0, 4)
        elif kind == 2: t["inp"]["stride"][0, rng.integers(3), rng.integers(6)] = rng.integers(-3, 3)
        elif kind == 3: t["out"]["stride"][0, rng.integers(6)] = rng.integers(-1, 2)
        elif kind == 4: t["out"]["bcast_mask"][0] = rng.integers(0, 4)
        elif kind == 5: t["inp"]["ptr"][0, rng.integers(3)] = 0
        elif kind == 6: t["inp"]["dtype"][0, rng.integers(3)] = rng.integers(0, 6)
        elif kind == 7: t["out"]["dtype"][0] = rng.integers(0, 6)
        elif kind == 8: t["size"][0, rng.integers(6)] = rng.choice([-1, 0, 1, 1 << 20, 1 << 31, (1 << 31) - 1])
        elif kind == 9: t["inp"]["bcast_mask"][0, rng.integers(3)] = rng.integers(0, 64)
        elif kind == 10: t["inp"]["stride"][0, rng.integers(3), rng.integers(6)] = 1 << 31
        elif kind == 12:                                  # an address that may be no multiple of the element size
            if rng.integers(2): t["inp"]["ptr"][0, rng.integers(3)] += rng.integers(1, 4)
            else: t["out"]["ptr"][0] += rng.integers(1, 4)
        use_impl = int(impl[i]) if kind != 11 else int(rng.integers(0, 20))
        got, _ = _status(t, 0, use_impl)
        want = oracle.validate(t, 0, use_impl)
        assert got == want, (trial, kind, i, use_impl, got, want)
        n_bad += want != 0
    return n_bad


def test_validation_agrees_with_the_oracle_on_damaged_descriptors():
    """Differential test of two independently written validators."""
    rng = np.random.default_rng(77)
    n_bad = 0
    for s in (C.config2_reduced(), C.row_operations(), C.reductions()):
        n_bad += _damage_and_compare(s, rng, 2000)
    assert n_bad > 300


def test_task_bytes_counts_each_distinct_element_once():
    s = S.config1(n_tasks=3)
    hp = HostPools(s)
    rc, nbytes = _status(hp.tasks, 0, S.IMPL["ADD"])
    assert rc == 0 and nbytes == 3 * 1024 * 4
    c3 = S.config3(n_chains=1, Bs=(2,), Ss=(64,), heads=4, buffer_sets=1)
    hp = HostPools(c3)
    n = 2 * 4 * 64 * 64
    rows = 2 * 4 * 64
    want = [2 * n * 2, 2 * n * 2 + 64 * 64 * 2, n * 2 + rows * 4, 2 * n * 2 + rows * 4, n * 2 + rows * 4, 2 * n * 2 + rows * 4]
    got = [_status(hp.tasks, i, c3.impl_for()[i])[1] for i in range(6)]
    assert got == want
    assert sum(want) == 20 * n + 64 * 64 * 2 + 4 * rows * 4      # 20 bytes per score element plus the small vectors


def test_task_plan_picks_the_execution_path_the_layout_calls_for():
    """The host classifies each task by the strides left after merging dims: contiguous ->
    vector path, row vector / per-row scalar -> 2-D path, a transposed input under a contiguous
    output -> LDS tiles, anything else -> the generic walk; reductions by row contiguity."""
    from helpers import Builder
    b = Builder()
    f = lambda *shape: b.pool(np.zeros(shape, np.float32))
    a, c = f(4, 96, 80), f(4, 96, 80)
    o = f(4, 96, 80)
    at = f(4, 80, 96).transpose(0, 2, 1)
    b.add("ADD", o, [a, c])                                              # 0 contiguous: dims merge to 1
    b.add("ADD", o[0], [a[0], np.broadcast_to(f(80), (96, 80))])         # 1 row vector
    b.add("SUB_EXP", o[0], [a[0], np.broadcast_to(f(96)[:, None], (96, 80))])   # 2 per-row scalar
    b.add("MUL", o, [at, c])                                             # 3 transposed input, batched
    b.add("MUL", o[0], [at[0], at[1]])                                   # 4 rank 2, both transposed
    b.add("MUL", o[0, :4, :4], [at[0, :4, :4], c[0, :4, :4]])            # 5 output not contiguous
    b.add("COPY", o.transpose(0, 2, 1), [f(4, 80, 96)])                  # 6 transposed OUTPUT: generic
    b.add("COPY", o, [at])                                               # 7 same-dtype copy keeps raw bits: generic
    b.add("RELU", o[:, ::2, :], [a[:, ::2, :]])                          # 8 gapped rows: generic
    b.add("SUM_LAST", f(4, 96), [a])                                     # 9 contiguous rows
    b.add("MAX_LAST", f(4, 96), [at])                                    # 10 strided rows
    b.add("ADD", f(4, 5)[:0], [f(4, 5)[:0], f(4, 5)[:0]])                # 11 empty
    s = b.stream()
    hp = HostPools(s)
    impl = s.impl_for()
    got = [R.task_plan(hp.tasks, i, impl[i]) for i in range(len(s))]
    paths = [g[0] for g in got]
    assert paths == ["CONTIG", "ROW2D", "ROW2D", "TILE2D", "TILE2D", "GENERIC", "GENERIC", "GENERIC", "GENERIC",
                     "RED_CONTIG", "RED_GENERIC", "NOP"], paths
    assert got[0][3] == 1                                  # [4, 96, 80] contiguous merges to one dim
    assert got[3][1] * got[3][2] >= 4 * 3 * 3 and got[3][3] == 3      # 4 batches of 3 x 3 tiles
    # contiguous output, inputs strided / broadcast / of another dtype: gathered through LDS
    g = Builder()
    f = lambda *shape: g.pool(np.zeros(shape, np.float32))
    h = lambda *shape: g.pool(np.zeros(shape, np.float16))
    x2 = f(2 * 5000 + 1)
    g.add("RELU", f(5000), [x2[1::2]])                                   # 0 a stride-2 slice that starts at element 1
    g.add("ADD", f(33, 77), [f(33, 77), np.broadcast_to(f(77), (33, 77))])          # 1 row vector, 77 is no multiple of the vector width
    g.add("MUL", f(33, 77), [f(33, 77), np.broadcast_to(f(33)[:, None], (33, 77))]) # 2 column vector: read along the rows through LDS tiles
    g.add("ADD", f(6, 9, 5), [f(6, 5, 9).transpose(0, 2, 1), f(6, 9, 5)])           # 3 small transposes (5 columns: no LDS tiles)
    g.add("SUB", h(400), [f(400), h(400)])                               # 4 mixed dtypes
    g.add("COPY", f(5000), [x2[::2]])                                    # 5 same-dtype copy keeps raw bits: generic
    g.add("RELU", f(5001)[1:], [x2[: 10000: 2]])                         # 6 output not 16-byte aligned: generic
    i32 = g.pool(np.zeros(200, np.int32))
    g.add("ADD", g.pool(np.zeros(100, np.int32)), [i32[::2], i32[1::2]]) # 7 integers: generic
    g.add("ADD", f(3, 4, 5, 6), [f(3, 4, 5, 6), np.broadcast_to(f(4, 1, 6)[None], (3, 4, 5, 6))])   # 8 four dims that do not merge: generic
    sg = g.stream()
    hg = HostPools(sg)
    got = [R.task_plan(hg.tasks, i, sg.impl_for()[i])[0] for i in range(len(sg))]
    assert got == ["STAGED", "STAGED", "TILE2D", "STAGED", "STAGED"] + ["GENERIC"] * 4, got
    # a large transposed task splits into at most 1024 units that cover every tile
    big = Builder()
    src = big.pool(np.zeros((3000, 2100), np.float16)).T
    big.add("RELU", big.pool(np.zeros((2100, 3000), np.float16)), [src])
    sb = big.stream()
    path, chunks, per, nd = R.task_plan(HostPools(sb).tasks, 0, S.IMPL["RELU"])
    tiles = ((2100 + 31) // 32) * ((3000 + 31) // 32)
    assert path == "TILE2D" and chunks <= 1024 and (chunks - 1) * per < tiles <= chunks * per


def test_small_tasks_are_cut_into_more_chunks_than_their_size_alone_would_give():
    """How the host cuts a task into work units (gpuos_task_plan -> path, chunks, elements or tiles per
    chunk): the regular chunk of an fp32 binary operator is 16,384 elements, 8,192 up to 2^20 elements;
    a task of at most four such chunks becomes up to four of at least 4,096; a gathered task is spread
    over up to 32 workgroups with two rounds of 1,024 elements each at least; a transposed one over one
    workgroup per 32 x 32 tile, up to 64.  Every element is covered exactly once."""
    from helpers import Builder
    def plan(build):
        b = Builder()
        build(b)
        s = b.stream()
        return R.task_plan(HostPools(s).tasks, 0, s.impl_for()[0])
    f32 = lambda b, *shape: b.pool(np.zeros(shape, np.float32))
    def contig(n):
        return plan(lambda b: b.add("ADD", f32(b, n), [f32(b, n), f32(b, n)]))
    want = {1000: (1, 4096), 4096: (1, 4096), 4097: (2, 4096), 16384: (4, 4096), 20000: (4, 5120), 32768: (4, 8192),
            40000: (5, 8192), 1 << 20: (128, 8192), (1 << 20) + 1: (65, 16384), 1 << 24: (1024, 16384)}
    for n, (chunks, per) in want.items():
        path, c, p, _ = contig(n)
        assert (path, c, p) == ("CONTIG", chunks, per), (n, path, c, p)
        assert (c - 1) * p < n <= c * p
    # a unary operator moves 8 bytes per element instead of 12: its chunks hold half as many elements again
    path, c, p, _ = plan(lambda b: b.add("RELU", f32(b, 1 << 20), [f32(b, 1 << 20)]))
    assert (path, p) == ("CONTIG", 12288) and (c - 1) * p < (1 << 20) <= c * p
    def staged(n):
        return plan(lambda b: b.add("RELU", f32(b, n), [f32(b, 2 * n + 1)[1::2]]))
    for n, (chunks, per) in {1500: (1, 2048), 5000: (3, 2048), 60000: (30, 2048), 65536: (32, 2048), 100000: (25, 4096),
                             600000: (49, 12288)}.items():
        path, c, p, _ = staged(n)
        assert (path, c, p) == ("STAGED", chunks, per), (n, path, c, p)
    def tiled(r, cc):
        return plan(lambda b: b.add("RELU", f32(b, r, cc), [f32(b, cc, r).T]))
    for (r, cc), (chunks, per) in {(64, 64): (4, 1), (66, 228): (24, 1), (256, 256): (64, 1), (512, 256): (64, 2),
                                   (1024, 1024): (128, 8)}.items():
        path, c, p, _ = tiled(r, cc)
        tiles = ((r + 31) // 32) * ((cc + 31) // 32)
        assert (path, c, p) == ("TILE2D", chunks, per) and (c - 1) * p < tiles <= c * p, ((r, cc), path, c, p)


def test_task_plan_for_row_operations():
    """Rows of whole aligned vectors (at most 256 of them), one dtype, contiguous -> rows in
    registers, with further inputs laid out like x, repeated every `period` rows, or one row;
    everything else takes the three-pass path."""
    from helpers import Builder
    b = Builder()
    f = lambda *shape: b.pool(np.zeros(shape, np.float32))
    h = lambda *shape: b.pool(np.zeros(shape, np.float16))
    x = f(2, 3, 64, 64)
    b.add("SOFTMAX_LAST", f(2, 3, 64, 64), [x])                                              # 0 fused
    b.add("MASKED_SOFTMAX_LAST", f(2, 3, 64, 64), [x, np.broadcast_to(f(64, 64), (2, 3, 64, 64))])   # 1 fused, period 64
    b.add("MASKED_SOFTMAX_LAST", f(2, 3, 64, 64), [x, f(2, 3, 64, 64)])                      # 2 fused, full
    b.add("MASKED_SOFTMAX_LAST", f(2, 3, 64, 64), [x, np.broadcast_to(f(64), (2, 3, 64, 64))])       # 3 fused, one row
    b.add("MASKED_SOFTMAX_LAST", f(2, 3, 64, 64), [x, np.broadcast_to(f(2, 1, 64, 64), (2, 3, 64, 64))])  # 4 mask skips a middle dim
    b.add("LAYERNORM_LAST", f(50, 1024), [f(50, 1024), np.broadcast_to(f(1024), (50, 1024)), np.broadcast_to(f(1024), (50, 1024))])  # 5
    b.add("LAYERNORM_LAST", f(50, 1024), [f(50, 1024), f(50, 1024), np.broadcast_to(f(1024), (50, 1024))])   # 6 per-element gamma
    b.add("SOFTMAX_LAST", f(10, 1028), [f(10, 1028)])                                        # 7 257 vectors: a workgroup per row
    b.add("SOFTMAX_LAST", f(10, 30), [f(10, 30)])                                            # 8 not whole vectors
    b.add("SOFTMAX_LAST", f(10, 32), [h(10, 32)])                                            # 9 mixed dtypes
    b.add("SOFTMAX_LAST", f(10, 32), [f(10, 64)[:, ::2]])                                    # 10 strided
    b.add("SOFTMAX_LAST", f(10, 32), [f(10, 36)[:, :32]])                                    # 11 row pitch
    b.add("SOFTMAX_LAST", f(32), [f(32)])                                                    # 12 one row, rank 1
    b.add("SOFTMAX_LAST", h(4, 2048), [h(4, 2048)])                                          # 13 fp16: 256 vectors
    b.add("LAYERNORM_LAST", h(50, 1024), [h(50, 1024), np.broadcast_to(f(1024), (50, 1024)), np.broadcast_to(f(1024), (50, 1024))])  # 14 fp32 parameters under fp16 x
    b.add("LAYERNORM_LAST", h(50, 1024), [h(50, 1024), np.broadcast_to(f(1024), (50, 1024)), np.broadcast_to(h(1024), (50, 1024))])  # 15 gamma fp32, beta fp16
    s = b.stream()
    hp = HostPools(s)
    impl = s.impl_for()
    got = [R.task_plan(hp.tasks, i, impl[i]) for i in range(len(s))]
    want = ["ROW_FUSED"] * 4 + ["ROW_GENERIC", "ROW_FUSED", "ROW_GENERIC", "ROW_FUSED", "ROW_GENERIC", "ROW_GENERIC",
                                "ROW_GENERIC", "ROW_GENERIC", "ROW_FUSED", "ROW_FUSED", "ROW_FUSED", "ROW_GENERIC"]
    assert [g[0] for g in got] == want, [g[0] for g in got]
    rows = 2 * 3 * 64
    assert (got[0][1] - 1) * got[0][2] < rows <= got[0][1] * got[0][2]
    # bytes: x and y once, the mask at its true size
    assert R.task_bytes(hp.tasks[1:2], impl[1:2])[0] == 2 * rows * 64 * 4 + 64 * 64 * 4


def test_bench_refuses_more_than_one_gpu():
    """This build measures one GPU's share; bench.py says so instead of running with --gpus N > 1."""
    import os, subprocess, sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=300)
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr)
