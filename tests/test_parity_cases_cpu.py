"""CPU checks of the streams the GPU parity tests submit: every tensor lies inside its pool (no GPU
run may name memory outside its buffers) and the oracle accepts and runs every task."""
import numpy as np
import pytest

import oracle
from paper_2604_17861_amd import streams as S
import parity_cases as C
from helpers import HostPools


@pytest.mark.parametrize("name", sorted(C.CPU_CHECKED))
def test_case_is_in_bounds_and_valid(name):
    s = C.CPU_CHECKED[name]()
    assert C.stream_extent_violations(s) == []
    hp = HostPools(s)
    impl = s.impl_for()
    stand_in = {1: S.IMPL["RELU"], 2: S.IMPL["DIV"], 3: S.IMPL["FMA"]}      # a program validates like a float built-in of its arity
    def check(i):
        k = int(impl[i])
        return oracle.validate(hp.tasks, i, stand_in[s.programs[k][1]] if k in s.programs else k)
    bad = [i for i in range(len(s)) if check(i) != 0]
    assert bad == []
    if name not in ("config3_reduced", "config3_fused_reduced", "config5_reduced"):      # these take long on the CPU; the GPU suite runs them
        st = oracle.run_stream(hp.tasks, impl, programs=s.programs)
        assert np.all(st == 0)


def test_extent_check_catches_a_view_past_its_pool():
    s = C.config2_reduced()
    s.tasks["inp"]["ptr"][5, 0] = s.pools[int(s.pool_of[5, 0])].nbytes - 8
    assert C.stream_extent_violations(s) == [5]


def _run_in_random_dependency_order(s, seed, honour_deps=True):
    """The oracle, one task at a time, in a random order that respects nothing but the declared
    dependencies and fences: what an out-of-order executor is allowed to do."""
    import random
    rng = random.Random(seed)
    hp = HostPools(s)
    impl = s.impl_for()
    n = len(s)
    dep, fence = s.tasks["dep"], (s.tasks["flags"] & S.FLAG_FENCE) != 0
    done = np.zeros(n, bool)
    window = 48                                        # tasks the executor looks ahead over
    floor = 0
    while floor < n:
        ready = []
        for i in range(floor, min(n, floor + window)):
            if done[i]:
                continue
            if honour_deps and (any(d and not done[i - int(d)] for d in dep[i]) or (fence[i] and not done[:i].all())):
                continue
            ready.append(i)
        i = rng.choice(ready)
        assert oracle.run_stream(hp.tasks, impl, first=i, count=1)[0] == 0
        done[i] = True
        while floor < n and done[floor]:
            floor += 1
    return hp.arrays


def test_dependency_dag_declares_exactly_what_out_of_order_execution_needs():
    """The hazard-laden stream of the GPU test: executed out of order under its declared dependencies
    it equals sequential execution (they are sufficient); with the declarations ignored it does not
    (the stream really has hazards, so the GPU test can fail)."""
    from helpers import run_oracle
    s = C.dependency_dag(0, n_tasks=400)
    want, st = run_oracle(s)
    assert np.all(st == 0)
    for seed in (1, 2):
        got = _run_in_random_dependency_order(s, seed)
        assert all(np.array_equal(g, w) for g, w in zip(got, want.arrays))
    got = _run_in_random_dependency_order(s, 3, honour_deps=False)
    assert not all(np.array_equal(g, w) for g, w in zip(got, want.arrays))
