"""The five configurations at their full sizes, in the launch configuration bench.py times (default
capacity 4096, the default 3 workgroups per CU, the stream's own batch size), against the oracle: everything
that survives in memory is compared element by element; where buffers are reused by design, the
last writers are compared and properties that hold at any size are checked for the rest."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

from paper_2604_17861_amd import runtime as R
from paper_2604_17861_amd import streams as S

pytestmark = pytest.mark.gpu
CFG = dict(idle_exit_ms=30000, wait_timeout_ms=30000)


def test_config2_full():
    from gpu_helpers import DevicePools, run_stream, compare_with_oracle, parity_report
    s = S.config2()
    print("config2 full: 10,000 tasks", flush=True)
    dp = DevicePools(s)
    with R.Runtime(0, **CFG) as rt:
        rt.register_table(s.table)
        t0 = run_stream(s, rt, dp)
        comps = rt.completions(t0, len(s))
    assert np.all(comps["status"] == 0)
    imgs = dp.download()
    with ThreadPoolExecutor(8) as ex:                      # harness parallelism over disjoint ticket ranges
        parts = list(ex.map(lambda k: compare_with_oracle(s, imgs, first=k * 1250, count=1250), range(8)))
    parity_report("config2", parts, seed=1, tasks=len(s))
    assert max(p["max_ulp"] for p in parts) <= 2


def test_config3_full_2000_chains():
    """All 2,000 chains run; the chains that last used each buffer set (24 of them) are compared task
    by task, and every surviving probability tensor is checked for the softmax properties."""
    from gpu_helpers import DevicePools, run_stream, compare_with_oracle, parity_report
    s = S.config3()
    print("config3 full: 12,000 tasks", flush=True)
    dp = DevicePools(s)
    with R.Runtime(0, **CFG) as rt:
        rt.register_table(s.table)
        t0 = run_stream(s, rt, dp)
        comps = rt.completions(t0, len(s))
    assert np.all(comps["status"] == 0)
    imgs = dp.download()
    last = {}
    for c in range(2000):
        last[(int(s.info["chain_pair"][c]), int(s.info["chain_set"][c]))] = c
    assert len(last) == 24
    # compare backwards inside a chain: each task's inputs are still what the GPU left there
    with ThreadPoolExecutor(8) as ex:
        parts = list(ex.map(lambda c: compare_with_oracle(s, imgs, first=c * 6, count=6), sorted(last.values())))
    parity_report("config3", parts, seed=2, tasks=len(s), note="the 24 chains that last wrote each buffer set, task "
                   "by task; softmax properties on every surviving probability tensor")
    for (pi, k), c in last.items():
        b, n = s.info["pairs"][pi]
        lay = s.info["layout"][(b, n)][k]
        p = imgs[lay["w"]][lay["p"]: lay["p"] + b * 16 * n * n * 2].view(np.float16).astype(np.float32).reshape(-1, n, n)
        iu = np.triu_indices(n, 1)
        assert not p[:, iu[0], iu[1]].any()                          # exactly 0 above the diagonal
        assert np.abs(p.sum(-1) - 1).max() <= n * 2.0 ** -11         # rows sum to 1


def test_config4_full_million_tasks_with_hot_swaps():
    """1,000,000 tasks with 99 swaps under load.  Window w is copied back after its last task
    completed and before window w+2 (same memory) is submitted; every 5th window is compared in full
    against the oracle for the recorded versions; the version invariants are checked for all tasks."""
    from gpu_helpers import DevicePools, compare_with_oracle, parity_report
    s = S.config4()
    window = s.info["window"]
    n_win = len(s) // window
    print("config4 full: %d tasks, %d windows" % (len(s), n_win), flush=True)
    dp = DevicePools(s)
    swaps = {t: (op, impl) for t, op, impl in s.swaps}
    kept = {}
    versions = np.zeros(len(s), np.uint32)
    with R.Runtime(0, completion_log=1 << 21, **CFG) as rt:
        rt.register_table(s.table)
        for w in range(n_win):
            lo = w * window
            if lo in swaps:
                rt.swap_op(*swaps[lo])
            for i in range(lo, lo + window, s.batch):
                rt.submit(dp.tasks, i, min(s.batch, lo + window - i))
            if w >= 1:                                   # window w-1 must be complete before w+1 reuses its memory
                rt.wait((w * window) - 1)
                prev = w - 1
                if prev % 5 == 0:
                    half = s.info["window_bytes"]
                    off = (prev % 2) * half
                    kept[prev] = dp.tensors[1][off: off + half].cpu().numpy()
        rt.wait()
        for k in range(0, len(s), 1 << 18):
            m = min(1 << 18, len(s) - k)
            c = rt.completions(k, m)
            assert np.all(c["status"] == 0)
            versions[k: k + m] = c["op_version"]
    gelu = s.tasks["op_id"] == S.OP_GELU
    v = versions.astype(np.int64)
    assert np.all(v[~gelu] == 1) and v[gelu].min() >= 1 and v[gelu].max() <= len(s.swaps) + 1
    for k, (t, _, _) in enumerate(s.swaps):
        assert v[t: t + window][gelu[t: t + window]].min() >= k + 2
    assert len(np.unique(v[gelu])) == len(s.swaps) + 1
    in_img = dp.tensors[0].cpu().numpy()
    def check(w):
        img_out = np.zeros(2 * s.info["window_bytes"], np.uint8)
        off = (w % 2) * s.info["window_bytes"]
        img_out[off: off + s.info["window_bytes"]] = kept[w]
        return compare_with_oracle(s, [in_img, img_out], versions=versions, first=w * window, count=window)
    with ThreadPoolExecutor(8) as ex:
        parts = list(ex.map(check, sorted(kept)))
    parity_report("config4", parts, seed=3, tasks=len(s), swaps=len(s.swaps), windows_compared=sorted(kept),
                   distinct_gelu_versions=int(len(np.unique(v[gelu]))))


def test_config5_full_bandwidth_stream():
    """20,000 large tasks; outputs rotate through 64 slots, so the last 64 tasks are compared in full
    (inputs are read-only pools)."""
    from gpu_helpers import compare_with_oracle, parity_report
    from bench import DevicePools as BenchPools, submit_pass
    s = S.config5()
    print("config5 full: 20,000 tasks", flush=True)
    dp = BenchPools(s, torch)
    with R.Runtime(0, **CFG) as rt:
        rt.register_table(s.table)
        t0 = submit_pass(rt, s, dp.tasks)
        comps = rt.completions(t0, len(s))
    assert np.all(comps["status"] == 0)
    imgs = [t.cpu().numpy() for t in dp.tensors]
    first = len(s) - s.info["out_slots"]
    with ThreadPoolExecutor(8) as ex:
        parts = list(ex.map(lambda k: compare_with_oracle(s, imgs, first=first + 8 * k, count=8), range(8)))
    parity_report("config5", parts, seed=4, tasks=len(s), note="the last 64 tasks (one per output slot) in full")
