"""The seeded stream generators: determinism, the proportions each configuration names, and that
every generated descriptor is valid for the oracle (and runs) at reduced length."""
import numpy as np
import pytest

import oracle
from paper_2604_17861_amd import streams as S
from helpers import HostPools


def test_config1_shape_and_determinism():
    a, b = S.config1(), S.config1()
    assert len(a) == 1000 and a.tasks.tobytes() == b.tasks.tobytes()
    assert np.all(a.tasks["size"][:, 0] == 1024) and np.all(a.tasks["op_id"] == S.OP["ADD"])
    assert a.pools[0].data.tobytes() == b.pools[0].data.tobytes()
    v = a.pools[0].data.view(np.float32)
    assert v.min() >= -1 and v.max() <= 1 and abs(float(v.mean())) < 0.01
    assert S.config1(seed=1).pools[0].data.tobytes() != a.pools[0].data.tobytes()


def test_config2_proportions():
    s = S.config2(n_tasks=4000, in_pool_elems=1 << 20)
    t = s.tasks
    dt = t["out"]["dtype"]
    frac = [(dt == k).mean() for k in (S.F32, S.F16, S.BF16)]
    assert abs(frac[0] - 0.5) < 0.04 and abs(frac[1] - 0.25) < 0.04 and abs(frac[2] - 0.25) < 0.04
    numel = np.prod(np.where(np.arange(6)[None, :] < t["ndim"][:, None], t["size"], 1), axis=1)
    assert numel.min() >= 128 and numel.max() <= 140000
    assert abs(np.log(numel).mean() - (np.log(256) + np.log(65536)) / 2) < 0.15
    assert set(np.unique(t["ndim"])) == {1, 2, 3, 4}
    n_inputs_total = t["n_inputs"].sum()
    assert abs(s.info["noncontig_inputs"] / n_inputs_total - 0.3) < 0.05
    assert abs(s.info["broadcast_ops"] / s.info["binary_ops"] - 0.2) < 0.04
    ops = set(np.unique(t["op_id"]))
    assert ops == {S.OP[n] for n in ("ADD", "MUL", "SUB", "RELU", "EXP", "GELU_TANH", "SCALE")}
    assert s.batch == 64


def test_config3_chain_structure():
    s = S.config3(n_chains=40, buffer_sets=2)
    assert len(s) == 240
    ops = s.tasks["op_id"].reshape(-1, 6)
    want = [S.OP[n] for n in ("SCALE", "ADD", "MAX_LAST", "SUB_EXP", "SUM_LAST", "DIV")]
    assert np.all(ops == np.array(want)[None, :])
    assert np.all(s.tasks["dep"][:, 0].reshape(-1, 6)[:, 1:] == 1)
    assert len(set(s.info["chain_pair"][:12])) == 12        # round-robin over the 12 (B, S) pairs
    # a chain reusing a buffer set depends on that set's previous chain
    first_dep = s.tasks["dep"][::6, 0]
    assert np.all(first_dep[:24] == 0) and np.all(first_dep[24:] > 0)
    m = s.pools[0].data.view(np.float16)
    side = int(np.sqrt(m.size)); m = m.reshape(side, side)
    assert np.all(np.isneginf(m[np.triu_indices(side, 1)])) and np.all(np.tril(m) == 0)


def test_config4_swaps_and_windows():
    s = S.config4(n_tasks=50000, swap_every=10000, window=10000)
    assert [t for t, _, _ in s.swaps] == [10000, 20000, 30000, 40000]
    assert [i for _, _, i in s.swaps] == [S.IMPL["GELU_TANH"], S.IMPL["GELU_ERF"]] * 2
    n = s.tasks["size"][:, 0]
    assert n.min() >= 1024 and n.max() <= 16384
    # outputs inside a window never overlap
    for w in range(5):
        sel = slice(w * 10000, (w + 1) * 10000)
        off = s.tasks["out"]["ptr"][sel].astype(np.int64); nb = n[sel] * 4
        order = np.argsort(off)
        assert np.all(off[order][1:] >= (off + nb)[order][:-1])
    v = np.ones(len(s), np.uint32); v[10000:20000] = 2
    impl = s.impl_for(v)
    g = s.tasks["op_id"] == S.OP_GELU
    assert np.all(impl[g][: (g[:10000]).sum()] == S.IMPL["GELU_ERF"])
    assert np.all(impl[10000:20000][g[10000:20000]] == S.IMPL["GELU_TANH"])


def test_config5_shapes_and_slots():
    s = S.config5(n_tasks=2000, in_pool_bytes=1 << 28, tile_elems=1 << 16)
    r, c = s.tasks["size"][:, 0], s.tasks["size"][:, 1]
    assert r.min() >= 64 and r.max() <= 4096 and c.min() >= 256 and c.max() <= 16384
    assert (r * c).max() <= 1 << 24
    assert np.all(s.tasks["dep"][64:, 0] == 64) and np.all(s.tasks["dep"][:64, 0] == 0)
    assert set(np.unique(s.tasks["out"]["dtype"])) == {S.F32, S.BF16}


@pytest.mark.parametrize("make", [
    lambda: S.config1(n_tasks=20),
    lambda: S.config2(n_tasks=300, in_pool_elems=1 << 19),
    lambda: S.config3(n_chains=4, Bs=(1, 2), Ss=(64, 128), heads=2),
    lambda: S.config4(n_tasks=400, swap_every=100, window=100, in_pool_elems=1 << 16),
    lambda: S.config5(n_tasks=24, rows_range=(4, 64), cols_range=(16, 512), max_numel=1 << 14,
                      in_pool_bytes=1 << 20, out_slots=8, tile_elems=1 << 12),
])
def test_generated_descriptors_are_valid_and_run(make):
    s = make()
    hp = HostPools(s)
    impl = s.impl_for()
    for i in range(len(s)):
        assert oracle.validate(hp.tasks, i, impl[i]) == 0, i
        for k in range(4):                      # every referenced region lies inside its pool
            if s.pool_of[i, k] < 0:
                continue
    st = oracle.run_stream(hp.tasks, impl)
    assert np.all(st == 0)
    out_pool = hp.arrays[int(s.pool_of[0, 3])]
    assert out_pool.any()
