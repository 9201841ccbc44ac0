"""Tensors at the size limit of the descriptor (numel just under 2^31, 4 GiB per fp16 tensor): the
contiguous, row-broadcast, LDS-tiled transposed, reduction and fused-row paths at extents where
32-bit element offsets and per-chunk buffer windows are closest to overflowing.  The oracle cannot
run 2^31 elements in reasonable time, so rows / slices sampled at the start, in the middle
(unaligned) and at the very end are compared against it, to the same bars as everywhere else."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_17861_amd import runtime as R
from paper_2604_17861_amd import streams as S
from helpers import Builder, run_oracle
from gpu_helpers import rowop_error_scale

pytestmark = pytest.mark.gpu
CFG = dict(idle_exit_ms=30000, wait_timeout_ms=30000)


def _task(op, shape, ins, out, alpha=0.0):
    """ins / out: (device pointer, strides in elements, dtype)."""
    tasks, pool_of = S.new_tasks(1)
    S.set_head(tasks, 0, S.OP[op], shape, len(ins), alpha=alpha)
    for k, (ptr, st, dt) in enumerate(ins):
        S.set_tensor(tasks, pool_of, 0, k, 0, ptr, st, dt)
    S.set_tensor(tasks, pool_of, 0, 3, 0, out[0], out[1], out[2])
    return tasks


def _oracle(op, out_like, ins, alpha=0.0):
    b = Builder()
    views = [b.pool(np.ascontiguousarray(a)) for a in ins]
    o = b.pool(np.zeros_like(out_like))
    b.add(op, o, views, alpha=alpha)
    s = b.stream()
    hp, st = run_oracle(s)
    assert np.all(st == 0)
    p, off = b._locate(o)
    return hp.arrays[p][off: off + o.nbytes].view(o.dtype).reshape(o.shape), s, hp


def test_tensors_just_under_two_to_the_31_elements():
    N = (1 << 31) - 4096
    assert 1048574 * 2048 == N and 32767 * 65536 <= N          # every view below stays inside the N-element buffers
    dev = "cuda:0"
    x = torch.empty(N, dtype=torch.float16, device=dev).uniform_(-2.0, 2.0)
    outs = [torch.zeros(N, dtype=torch.float16, device=dev) for _ in range(4)]     # one per case: compared after shutdown
    C_, R_ = 65536, 32767                                   # R_ * C_ = 2^31 - 65536 <= N
    rowvec = torch.empty(C_, dtype=torch.float16, device=dev).uniform_(-1.0, 1.0)
    rows, n = 1048574, 2048                                 # rows * n = 2^31 - 4096 = N
    red = torch.zeros(rows, dtype=torch.float32, device=dev)
    torch.cuda.current_stream().synchronize()
    px, pr, pred = x.data_ptr(), rowvec.data_ptr(), red.data_ptr()
    po = [o.data_ptr() for o in outs]
    F16, F32 = S.F16, S.F32
    cases = [
        ("contiguous", _task("SCALE", [N], [(px, [1], F16)], (po[0], [1], F16), alpha=1.5), "CONTIG", 1024),
        ("row broadcast", _task("ADD", [R_, C_], [(px, [C_, 1], F16), (pr, [0, 1], F16)], (po[1], [C_, 1], F16)), "ROW2D", None),
        ("transposed", _task("RELU", [C_, R_], [(px, [1, C_], F16)], (po[2], [R_, 1], F16)), "TILE2D", None),
        ("reduction", _task("SUM_LAST", [rows, n], [(px, [n, 1], F16)], (pred, [1], F32)), "RED_CONTIG", None),
        ("fused softmax", _task("SOFTMAX_LAST", [rows, n], [(px, [n, 1], F16)], (po[3], [n, 1], F16)), "ROW_FUSED", None),
    ]
    # Everything runs first; results are read after the context is gone (a small device-to-host copy
    # can be queued behind the resident worker kernel and would then wait for it to exit).
    with R.Runtime(0, **CFG) as rt:
        rt.register_table(S.default_table())
        for name, tasks, want_path, want_chunks in cases:
            print(name, flush=True)
            path, chunks, per, nd = R.task_plan(tasks, 0, S.default_table()[int(tasks["op_id"][0])])
            assert path == want_path, (name, path)
            assert want_chunks is None or chunks == want_chunks, (name, chunks)
            t = rt.submit(tasks, 0, 1)
            rt.wait(t)
            assert rt.completions(t, 1)["status"][0] == 0
    # 1. contiguous SCALE over all N elements: 1024 chunks, the last one ragged
    for lo, cnt in ((0, 5000), (N // 2 - 1001, 4099), (N - 5003, 5003)):
        got = outs[0][lo: lo + cnt].cpu().numpy()
        want, _, _ = _oracle("SCALE", got, [x[lo: lo + cnt].cpu().numpy()], alpha=1.5)
        assert np.array_equal(got.view(np.uint16), want.view(np.uint16)), lo
    # 2. [R, C] + row vector (the 2-D broadcast path)
    rv = rowvec.cpu().numpy()
    for r in (0, 16383, R_ - 1):
        got = outs[1][r * C_: (r + 1) * C_].cpu().numpy()
        want, _, _ = _oracle("ADD", got, [x[r * C_: (r + 1) * C_].cpu().numpy(), rv])
        assert np.array_equal(got.view(np.uint16), want.view(np.uint16)), r
    # 3. transposed input through the LDS tiles: out[c, r] = relu(x[r, c])
    x2 = x[: R_ * C_].view(R_, C_)
    for c in (0, 40001, C_ - 1):
        got = outs[2][c * R_: (c + 1) * R_].cpu().numpy()
        want, _, _ = _oracle("RELU", got, [x2[:, c].contiguous().cpu().numpy()])
        assert np.array_equal(got.view(np.uint16), want.view(np.uint16)), c
    # 4. row sums of [1048574, 2048]
    g = red.cpu().numpy()
    for r in (0, 1, 524288, rows - 2, rows - 1):
        row = x[r * n: (r + 1) * n].cpu().numpy().astype(np.float64)
        s64, l1 = row.sum(), np.abs(row).sum()
        assert abs(float(g[r]) - s64) <= 1e-5 * max(abs(s64), l1 / np.sqrt(n)), r
    assert np.all(np.isfinite(g)) and np.count_nonzero(g) > rows - 100       # every row was written
    # 5. fused softmax over the same rows (256 vectors per row: the widest rows-in-registers case)
    for r in (0, 524287, rows - 1):
        got = outs[3][r * n: (r + 1) * n].cpu().numpy()
        _, s, hp = _oracle("SOFTMAX_LAST", got[None, :], [x[r * n: (r + 1) * n].cpu().numpy()[None, :]])
        y64 = oracle.rowop_f64(hp.tasks, 0, S.IMPL["SOFTMAX_LAST"])
        scale = rowop_error_scale(hp.tasks, 0, S.IMPL["SOFTMAX_LAST"], y64)
        tol = 2.0 ** -22 * scale + 2.0 ** (np.floor(np.log2(np.maximum(y64, 2.0 ** -14))) - 10)
        assert np.all(np.abs(got.astype(np.float64)[None, :] - y64) <= tol), r
    assert abs(float(outs[3][(rows - 1) * n: rows * n].float().sum()) - 1.0) < 1e-2
