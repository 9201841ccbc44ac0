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
    """All 2,000 chains, EVERY task compared with the oracle.  A pair's chains reuse two buffer sets
    in turn, so the stream is submitted one generation (12 chains, one per (B, S) pair, all on the
    same set index) at a time: generation g's work buffers are copied back once it has completed and
    before generation g+2, which overwrites them, is submitted, while generation g+1 runs.  Each
    chain's six tasks are then compared task by task on what the GPU left in its buffers (every
    intermediate of a chain survives in its work buffer), oracle instances over disjoint chains on
    all host cores.  The surviving probability tensors are also checked for the softmax properties."""
    from gpu_helpers import DevicePools, compare_with_oracle, parity_report
    s = S.config3()
    n_chains = len(s) // 6
    pairs = s.info["pairs"]
    per_gen = len(pairs)
    n_gen = -(-n_chains // per_gen)
    print("config3 full: %d tasks, %d generations of %d chains" % (len(s), n_gen, per_gen), flush=True)
    dp = DevicePools(s)
    dummy = np.zeros(16, np.uint8)
    fixed = {}                                              # pools no task writes: masks and scores
    for (b, n), sets in s.info["layout"].items():
        for lay in sets:
            fixed[lay["s"]] = s.pools[lay["s"]].host_image()
    for k, p in enumerate(s.pools):
        if p.name.startswith("mask"):
            fixed[k] = p.host_image()

    def check_chain(c, work_img):
        b, n = pairs[int(s.info["chain_pair"][c])]
        lay = s.info["layout"][(b, n)][int(s.info["chain_set"][c])]
        imgs = [fixed.get(k, dummy) for k in range(len(s.pools))]
        imgs[lay["w"]] = work_img
        st = compare_with_oracle(s, imgs, first=c * 6, count=6)
        p = work_img[lay["p"]: lay["p"] + b * 16 * n * n * 2].view(np.float16).astype(np.float32).reshape(-1, n, n)
        iu = np.triu_indices(n, 1)
        assert not p[:, iu[0], iu[1]].any()                          # exactly 0 above the diagonal
        assert np.abs(p.sum(-1) - 1).max() <= n * 2.0 ** -11         # rows sum to 1
        return st

    def snapshot(g):                                        # generation g has completed: its work buffers, chain by chain
        out = []
        for c in range(g * per_gen, min(n_chains, (g + 1) * per_gen)):
            b, n = pairs[int(s.info["chain_pair"][c])]
            lay = s.info["layout"][(b, n)][int(s.info["chain_set"][c])]
            out.append((c, dp.tensors[lay["w"]].cpu().numpy()))
        return out

    futures = []
    with ThreadPoolExecutor(16) as ex, R.Runtime(0, **CFG) as rt:
        rt.register_table(s.table)
        last_ticket = {}
        for g in range(n_gen + 2):
            if g >= 2:                                      # generation g-2 wrote the buffers generation g is about to reuse
                rt.wait(last_ticket[g - 2])
                for c, img in snapshot(g - 2):
                    futures.append(ex.submit(check_chain, c, img))
                while sum(not f.done() for f in futures) > 48:      # bound the snapshots kept in host memory
                    next(f for f in futures if not f.done()).result()
            if g < n_gen:
                lo, hi = g * per_gen * 6, min(len(s), (g + 1) * per_gen * 6)
                for i in range(lo, hi, s.batch):
                    rt.submit(dp.tasks, i, min(s.batch, hi - i))
                last_ticket[g] = hi - 1
        rt.wait()
        comps = rt.completions(0, len(s))
        assert np.all(comps["status"] == 0)
        parts = [f.result() for f in futures]
    assert len(parts) == n_chains
    parity_report("config3", parts, seed=2, tasks=len(s), note="every task of every chain, generation by generation")


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
    """20,000 large tasks, flat out, in the launch configuration bench.py times; outputs rotate through
    64 slots, so the last 64 tasks are compared in full (inputs are read-only pools)."""
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
    parity_report("config5_flat_out", parts, seed=4, tasks=len(s), note="the last 64 tasks (one per output slot) in full")


def test_config5_full_every_task():
    """The same 20,000 tasks at their full shapes with EVERY task compared with the oracle.  A task
    overwrites the output slot of the task 64 tickets before it, so the stream is submitted one lap
    of 64 tasks at a time: once a lap has completed its outputs (only the bytes each task wrote) are
    copied into pinned host memory, the next lap is submitted, and the lap is compared task by task
    while the GPU runs on: the oracle reads the read-only input pools and writes scratch memory of
    its own, oracle instances over disjoint tasks on all host cores."""
    from gpu_helpers import compare_with_oracle, parity_report
    from bench import DevicePools as BenchPools
    s = S.config5()
    lap = s.info["out_slots"]
    n_laps = -(-len(s) // lap)
    impls = s.impl_for()
    T = s.tasks
    red = np.isin(impls, [S.IMPL["SUM_LAST"], S.IMPL["MAX_LAST"]])
    es = np.where(T["out"]["dtype"] == S.F32, 4, 2).astype(np.int64)
    out_bytes = np.where(red, T["size"][:, 0], T["size"][:, 0] * T["size"][:, 1]).astype(np.int64) * es
    lap_bytes = max(int(((out_bytes[k * lap: (k + 1) * lap] + 255) // 256 * 256).sum()) for k in range(n_laps))
    print("config5 full, every task: %d laps of %d, at most %.0f MB of outputs per lap" % (n_laps, lap, lap_bytes / 1e6), flush=True)
    dp = BenchPools(s, torch)
    in_imgs = [dp.tensors[0].cpu().numpy(), dp.tensors[1].cpu().numpy()]
    n_stage = 6                                             # laps whose outputs are kept while their comparison runs
    stage = [torch.empty(lap_bytes, dtype=torch.uint8, pin_memory=True) for _ in range(n_stage)]
    scratch = [np.empty(lap_bytes, np.uint8) for _ in range(n_stage)]
    copy_stream = torch.cuda.Stream()
    base = s.materialize([in_imgs[0].ctypes.data, in_imgs[1].ctypes.data, 0])     # inputs: the host images of the pools

    def check_tasks(tg, to, t0, lo, hi):
        return compare_with_oracle(s, None, first=lo, count=hi - lo, task_arrays=(tg, to, t0))

    busy = [[] for _ in range(n_stage)]
    parts = []
    with ThreadPoolExecutor(16) as ex, R.Runtime(0, **CFG) as rt:
        rt.register_table(s.table)
        for k in range(n_laps):
            lo, hi = k * lap, min(len(s), (k + 1) * lap)
            for i in range(lo, hi, s.batch):
                rt.submit(dp.tasks, i, min(s.batch, hi - i))
            b = k % n_stage
            parts += [f.result() for f in busy[b]]          # the staging buffer's previous lap has been compared
            busy[b] = []
            rt.wait(hi - 1)
            tg, to = base[lo:hi].copy(), base[lo:hi].copy()
            off = 0
            with torch.cuda.stream(copy_stream):
                for j, i in enumerate(range(lo, hi)):
                    nb = int(out_bytes[i])
                    src = dp.tensors[2][int(T["out"]["ptr"][i]): int(T["out"]["ptr"][i]) + nb]
                    stage[b][off: off + nb].copy_(src, non_blocking=True)
                    tg["out"]["ptr"][j] = stage[b].data_ptr() + off
                    to["out"]["ptr"][j] = scratch[b].ctypes.data + off
                    off += (nb + 255) // 256 * 256
            copy_stream.synchronize()                       # the lap is on the host: the next lap may overwrite the slots
            for a in range(lo, hi, 4):
                busy[b].append(ex.submit(check_tasks, tg, to, lo, a, min(hi, a + 4)))
        rt.wait()
        comps = rt.completions(0, len(s))
        assert np.all(comps["status"] == 0)
        for b in range(n_stage):
            parts += [f.result() for f in busy[b]]
    assert sum(p["tasks"] for p in parts) == len(s)
    parity_report("config5", parts, seed=4, tasks=len(s), note="every task, lap by lap of 64 (the span after which an output slot is reused)")
