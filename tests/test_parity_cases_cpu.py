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
