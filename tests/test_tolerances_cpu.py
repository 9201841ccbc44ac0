"""The error bounds the GPU tests hold fused row operations to are test logic (tests/gpu_helpers.py),
not outputs of the oracle.  Hand values pin them, so that a slip cannot loosen the gate unseen."""
import math

import numpy as np

import oracle
from paper_2604_17861_amd import streams as S
from helpers import Builder, HostPools
import gpu_helpers as G


def _scale(build):
    b = Builder()
    build(b)
    s = b.stream()
    hp = HostPools(s)
    impl = int(s.impl_for()[0])
    y = oracle.rowop_f64(hp.tasks, 0, impl)
    return y, G.rowop_error_scale(hp.tasks, 0, impl, y)


def test_softmax_error_scale_hand_values():
    def build(b):
        x = b.pool(np.array([[0.0, 0.0], [0.0, -math.log(4.0)], [5.0, -np.inf]], np.float32))
        b.add("SOFTMAX_LAST", b.pool(np.zeros((3, 2), np.float32)), [x])
    y, sc = _scale(build)
    lg = 1.0                                             # log2 of the row length
    assert np.allclose(y, [[0.5, 0.5], [0.8, 0.2], [1.0, 0.0]], rtol=1e-7)
    want = [[0.5 * (8 + lg), 0.5 * (8 + lg)],
            [0.8 * (8 + lg), 0.2 * (math.log(4.0) + 8 + lg)],     # the smaller entry lies ln 4 below the maximum
            [1.0 * (8 + lg), 0.0]]                                # a result that is exactly 0 carries no error
    assert np.allclose(sc, want, rtol=1e-6, atol=0)


def test_masked_softmax_error_scale_sees_the_scaled_and_masked_argument():
    def build(b):
        x = b.pool(np.array([[8.0, 0.0, 3.0]], np.float32))
        m = b.pool(np.array([[0.0, -1.0, -np.inf]], np.float32))
        b.add("MASKED_SOFTMAX_LAST", b.pool(np.zeros((1, 3), np.float32)), [x, m], alpha=0.25)
    y, sc = _scale(build)
    # arguments t = 0.25 x + mask = [2, -1, -inf]: distances to the maximum 0, 3, (masked)
    e = math.exp(-3.0)
    assert np.allclose(y, [[1 / (1 + e), e / (1 + e), 0.0]], rtol=1e-12)
    lg = math.log2(3)
    assert np.allclose(sc, [[y[0, 0] * (8 + lg), y[0, 1] * (3 + 8 + lg), 0.0]], rtol=1e-9)


def test_layernorm_error_scale_hand_values():
    def build(b):
        x = b.pool(np.array([[1.0, 3.0], [10.0, 10.0]], np.float32))
        g = b.pool(np.array([2.0, -2.0], np.float32))
        be = b.pool(np.array([1.0, -1.0], np.float32))
        b.add("LAYERNORM_LAST", b.pool(np.zeros((2, 2), np.float32)), [x, np.broadcast_to(g, (2, 2)), np.broadcast_to(be, (2, 2))],
              alpha=0.0 + 1.0)                           # epsilon 1: variance 1 + 1 in row 0, 0 + 1 in row 1
    y, sc = _scale(build)
    r0 = 1 / math.sqrt(2.0)
    # row 0: mean 2, deviations -1, +1 (max 1), rstd 1/sqrt 2; row 1: mean 10, deviations 0, rstd 1
    want = [[(1 + 2 + 1) * r0 * 2 + 1, (3 + 2 + 1) * r0 * 2 + 1],
            [(10 + 10 + 0) * 1 * 2 + 1, (10 + 10 + 0) * 1 * 2 + 1]]
    assert np.allclose(sc, want, rtol=1e-12)
    assert np.allclose(y, [[-r0 * 2 + 1, r0 * -2 - 1], [1.0, -1.0]], rtol=1e-12)


def test_fp32_softmax_bound_is_inside_one_part_in_1e5():
    """What the gate comes to for fp32 outputs of the third configuration's rows (256 entries, arguments
    up to about 20 below the maximum): 2^-22 * (20 + 8 + 8) relative, under 1e-5."""
    assert G.ROW_REL * (20 + 8 + math.log2(256)) < 1e-5
