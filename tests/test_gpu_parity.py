"""GPU parity tests: the HIP path, called through the C ABI binding, against the CPU oracle,
element by element on the same seeded inputs."""
import numpy as np
import pytest
import torch

from paper_2604_17861_amd import runtime as R
from paper_2604_17861_amd import streams as S

pytestmark = pytest.mark.gpu


def _run_and_check(stream, capacity=0, **cfg):
    from gpu_helpers import DevicePools, run_stream, compare_with_oracle
    dp = DevicePools(stream)
    with R.Runtime(capacity, idle_exit_ms=20000, wait_timeout_ms=20000, **cfg) as rt:
        rt.register_table(stream.table)
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
    assert np.all(comps["op_version"] == 1)
