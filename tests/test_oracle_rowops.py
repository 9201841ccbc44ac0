"""Pins for the oracle's fused row operations (softmax over the last dim, the scaled + masked
variant, layer normalisation): closed forms, hand-worked rows, fp64 library routines (scipy's
softmax, torch's layer_norm on the CPU), invariants, the special-value rows, strided / broadcast
operands against materialised numpy arrays, and the already pinned six-task softmax chain."""
import math

import numpy as np
import pytest
import scipy.special
import torch

import oracle
from paper_2604_17861_amd import streams as S
from helpers import Builder, HostPools, run_oracle, bf16_bits_to_f32


def _run(build):
    """build(b) adds tasks to a Builder and returns the output views; -> (stream, HostPools, outs)."""
    b = Builder()
    outs = build(b)
    s = b.stream()
    hp, st = run_oracle(s)
    assert np.all(st == 0), st
    res = []
    for o in outs:                       # read each output view back from the oracle's copy of the pools
        p, off = b._locate(o)
        img = hp.arrays[p]
        flat = img[off:].view(o.dtype)
        res.append(np.lib.stride_tricks.as_strided(flat, shape=o.shape, strides=o.strides).copy())
    return s, hp, res


def _f64(s, hp, i=0):
    return oracle.rowop_f64(hp.tasks, i, s.impl_for()[i])


# ---- softmax ---------------------------------------------------------------------------------
def test_softmax_two_elements_is_the_logistic_function():
    rows = np.array([[0.0, 0.0], [1.0, -1.0], [-3.5, 2.25], [10.0, 9.0], [-50.0, 50.0]], np.float32)
    def build(b):
        x = b.pool(rows)
        o = b.pool(np.zeros_like(rows))
        b.add("SOFTMAX_LAST", o, [x])
        return [o]
    s, hp, (y,) = _run(build)
    y64 = _f64(s, hp)
    for k, (a, c) in enumerate(rows.astype(np.float64)):
        want0 = 1.0 / (1.0 + math.exp(c - a))
        assert abs(y64[k, 0] - want0) <= 4e-16 and abs(y64[k, 1] - (1.0 - want0)) <= 4e-16
        assert y[k, 0] == np.float32(y64[k, 0])             # the stored value is the double rounded once to fp32
    assert y[4, 0] == 0.0 or y[4, 0] < 1e-43               # exp(-100): far below fp32's normal range


def test_softmax_of_equal_values_is_exactly_uniform_and_rows_are_shift_invariant():
    def build(b):
        x = b.pool(np.full((3, 64), 7.25, np.float32))
        o = b.pool(np.zeros((3, 64), np.float32))
        b.add("SOFTMAX_LAST", o, [x])
        rng = np.random.default_rng(0)
        z = rng.standard_normal((5, 200)).astype(np.float32)
        z = np.round(z * 256) / 256                       # multiples of 2^-8: adding 16 is exact in fp32
        x1, x2 = b.pool(z), b.pool(z + np.float32(16.0))
        o1, o2 = b.pool(np.zeros_like(z)), b.pool(np.zeros_like(z))
        b.add("SOFTMAX_LAST", o1, [x1])
        b.add("SOFTMAX_LAST", o2, [x2])
        return [o, o1, o2]
    s, hp, (u, y1, y2) = _run(build)
    assert np.all(u == np.float32(1.0 / 64))
    assert np.array_equal(y1, y2)
    assert np.abs(y1.astype(np.float64).sum(-1) - 1).max() < 200 * 2.0 ** -25


@pytest.mark.parametrize("code", [S.F32, S.F16, S.BF16])
def test_softmax_matches_scipy_on_strided_views(code):
    rng = np.random.default_rng(code)
    raw = (rng.standard_normal((6, 40, 50)) * 3).astype(np.float32)
    if code == S.F16:
        stored = raw.astype(np.float16)
        as64 = stored.astype(np.float64)
    elif code == S.BF16:
        stored = (raw.view(np.uint32) >> 16).astype(np.uint16)        # truncation is fine for an input
        as64 = bf16_bits_to_f32(stored).astype(np.float64)
    else:
        stored, as64 = raw, raw.astype(np.float64)
    def build(b):
        x = b.pool(stored)
        xt = x.transpose(0, 2, 1)[:, ::2, 1:]             # last dim strided by 50, rows by 2
        o = b.pool(np.zeros((6, 25, 39), np.float32))
        b.add("SOFTMAX_LAST", o, [xt])
        return [o]
    s, hp, (y,) = _run(build)
    want = scipy.special.softmax(as64.transpose(0, 2, 1)[:, ::2, 1:], axis=-1)
    y64 = _f64(s, hp)
    assert np.abs(y64 - want).max() <= 1e-15
    assert np.array_equal(y, want.astype(np.float32))


def test_masked_softmax_scales_then_masks_and_broadcasts_the_mask():
    rng = np.random.default_rng(5)
    B, H, n = 2, 3, 16
    xs = (rng.standard_normal((B, H, n, n)) * 2).astype(np.float16)
    mask = np.where(np.tril(np.ones((n, n), bool)), 0.0, -np.inf).astype(np.float16)
    mask[3, 1] = np.float16(-2.5)                       # a finite entry, so "mask is added" is visible
    alpha = 0.125
    def build(b):
        x = b.pool(xs)
        m = b.pool(mask)
        o = b.pool(np.zeros((B, H, n, n), np.float16))
        b.add("MASKED_SOFTMAX_LAST", o, [x, np.broadcast_to(m, (B, H, n, n))], alpha=alpha)
        return [o]
    s, hp, (y,) = _run(build)
    t = alpha * xs.astype(np.float64) + mask.astype(np.float64)
    want = scipy.special.softmax(t, axis=-1)
    y64 = _f64(s, hp)
    assert np.abs(y64 - want).max() <= 1e-15
    iu = np.triu_indices(n, 1)
    assert not y[:, :, iu[0], iu[1]].any()              # exp(-inf) is exactly 0
    assert np.array_equal(y, want.astype(np.float32).astype(np.float16))
    # without the scale or without the mask the result differs: both terms are in
    assert np.abs(scipy.special.softmax(xs.astype(np.float64) + mask, -1) - y64).max() > 1e-3
    assert np.abs(scipy.special.softmax(alpha * xs.astype(np.float64), -1) - y64).max() > 1e-3


def test_softmax_special_rows():
    inf, nan = np.inf, np.nan
    rows = np.array([[1.0, nan, 2.0, 0.0],          # a NaN poisons its row
                     [-inf, -inf, -inf, -inf],      # nothing to normalise: inf - inf
                     [1.0, inf, 2.0, 0.0],          # a +inf maximum: inf - inf at that element, NaN sum
                     [-inf, 0.0, -inf, 0.0],        # masked entries are 0, the rest share the mass
                     [5.0, 5.0, 5.0, 5.0]], np.float32)
    def build(b):
        x = b.pool(rows)
        o = b.pool(np.zeros_like(rows))
        b.add("SOFTMAX_LAST", o, [x])
        return [o]
    _, _, (y,) = _run(build)
    assert np.isnan(y[0]).all() and np.isnan(y[1]).all() and np.isnan(y[2]).all()
    assert np.array_equal(y[3], np.array([0, 0.5, 0, 0.5], np.float32))
    assert np.array_equal(y[4], np.full(4, 0.25, np.float32))


def test_fused_masked_softmax_agrees_with_the_six_task_chain():
    """SCALE -> ADD mask -> MAX_LAST -> SUB_EXP -> SUM_LAST -> DIV (each pinned on its own, fp16
    intermediates) against the one fused task: the chain rounds five times to fp16 on the way, so
    the two agree to a few fp16 ulps, and where the chain is exactly 0 so is the fused result."""
    rng = np.random.default_rng(11)
    B, n = 8, 64
    xs = (rng.standard_normal((B, n, n)) * 2).astype(np.float16)
    mask = np.where(np.tril(np.ones((n, n), bool)), 0.0, -np.inf).astype(np.float16)
    alpha = 0.125
    def build(b):
        x = b.pool(xs)
        m = np.broadcast_to(b.pool(mask), (B, n, n))
        s1, s2, e, p = (b.pool(np.zeros((B, n, n), np.float16)) for _ in range(4))
        mx, l = b.pool(np.zeros((B, n), np.float32)), b.pool(np.zeros((B, n), np.float32))
        b.add("SCALE", s1, [x], alpha=alpha)
        b.add("ADD", s2, [s1, m])
        b.add("MAX_LAST", mx, [s2])
        b.add("SUB_EXP", e, [s2, np.broadcast_to(mx[:, :, None], (B, n, n))])
        b.add("SUM_LAST", l, [e])
        b.add("DIV", p, [e, np.broadcast_to(l[:, :, None], (B, n, n))])
        f = b.pool(np.zeros((B, n, n), np.float16))
        b.add("MASKED_SOFTMAX_LAST", f, [x, m], alpha=alpha)
        return [p, f]
    _, _, (chain, fused) = _run(build)
    assert np.array_equal(chain == 0, fused == 0)
    c, f = chain.astype(np.float64), fused.astype(np.float64)
    assert np.abs(c - f).max() <= 6 * 2.0 ** -11 * np.maximum(c, 2.0 ** -14).max()
    rel = np.abs(c - f)[c > 2.0 ** -10] / c[c > 2.0 ** -10]
    assert rel.max() <= 8 * 2.0 ** -11


# ---- layer normalisation -------------------------------------------------------------------------
def test_layernorm_hand_worked_rows():
    """[1,2,3,4]: mean 2.5, biased variance 1.25 -> (x - 2.5) / sqrt(1.25) = -3/sqrt5, -1/sqrt5, ...
    (an unbiased variance, 5/3, would give -1.1619).  [-1,1] with eps = 3: variance 1, so the
    divisor is sqrt(1 + 3) = 2 (eps outside the root, or added to the deviation, would not give
    0.5).  gamma / beta: y * 2 - 1 on the first row."""
    def build(b):
        x = b.pool(np.array([[1, 2, 3, 4]], np.float32))
        one, zero = b.pool(np.ones(4, np.float32)), b.pool(np.zeros(4, np.float32))
        o1 = b.pool(np.zeros((1, 4), np.float32))
        b.add("LAYERNORM_LAST", o1, [x, np.broadcast_to(one, (1, 4)), np.broadcast_to(zero, (1, 4))], alpha=0.0)
        x2 = b.pool(np.array([[-1, 1]], np.float32))
        o2 = b.pool(np.zeros((1, 2), np.float32))
        b.add("LAYERNORM_LAST", o2, [x2, np.broadcast_to(one[:2], (1, 2)), np.broadcast_to(zero[:2], (1, 2))], alpha=3.0)
        g = b.pool(np.array([2, 2, 2, -2], np.float32))
        be = b.pool(np.array([-1, -1, 0, 1], np.float32))
        o3 = b.pool(np.zeros((1, 4), np.float32))
        b.add("LAYERNORM_LAST", o3, [x, np.broadcast_to(g, (1, 4)), np.broadcast_to(be, (1, 4))], alpha=0.0)
        return [o1, o2, o3]
    _, _, (y1, y2, y3) = _run(build)
    r5 = math.sqrt(5.0)
    assert np.array_equal(y1[0], np.array([-3 / r5, -1 / r5, 1 / r5, 3 / r5]).astype(np.float32))
    assert np.array_equal(y2[0], np.array([-0.5, 0.5], np.float32))
    assert np.array_equal(y3[0], np.array([-6 / r5 - 1, -2 / r5 - 1, 2 / r5, -6 / r5 + 1]).astype(np.float32))


@pytest.mark.parametrize("code", [S.F32, S.F16, S.BF16])
def test_layernorm_matches_torch_float64_on_strided_views(code):
    rng = np.random.default_rng(20 + code)
    R_, n = 37, 96
    raw = (rng.standard_normal((R_, 2 * n)) * 3 + 1.5).astype(np.float32)
    graw = rng.standard_normal(n).astype(np.float32)
    braw = rng.standard_normal(n).astype(np.float32)
    def store(a):
        if code == S.F16:
            st = a.astype(np.float16)
            return st, st.astype(np.float64)
        if code == S.BF16:
            st = (a.view(np.uint32) >> 16).astype(np.uint16)
            return st, bf16_bits_to_f32(st).astype(np.float64)
        return a, a.astype(np.float64)
    xs, x64 = store(raw)
    gs, g64 = store(graw)
    eps = 1e-5
    def build(b):
        x = b.pool(xs)[:, ::2]                              # every other column
        g = np.broadcast_to(b.pool(gs), (R_, n))
        be = np.broadcast_to(b.pool(braw), (R_, n))        # beta stays fp32: dtypes mix per operand
        o = b.pool(np.zeros((R_, n), np.float32))
        b.add("LAYERNORM_LAST", o, [x, g, be], alpha=eps)
        return [o]
    s, hp, (y,) = _run(build)
    want = torch.nn.functional.layer_norm(torch.from_numpy(x64[:, ::2].copy()), (n,), torch.from_numpy(g64),
                                          torch.from_numpy(braw.astype(np.float64)),
                                          eps=float(np.float32(eps))).numpy()
    y64 = _f64(s, hp)
    assert np.abs(y64 - want).max() <= 1e-13
    assert np.abs(y.astype(np.float64) - want).max() <= 2.0 ** -23 * np.abs(want).max()


def test_layernorm_output_statistics_closed_form():
    """With gamma = 1, beta = 0 every output row has mean 0 and biased variance var / (var + eps)."""
    rng = np.random.default_rng(3)
    xs = (rng.standard_normal((16, 512)) * np.arange(1, 17)[:, None]).astype(np.float32)
    eps = 0.5
    def build(b):
        x = b.pool(xs)
        one, zero = b.pool(np.ones(512, np.float32)), b.pool(np.zeros(512, np.float32))
        o = b.pool(np.zeros_like(xs))
        b.add("LAYERNORM_LAST", o, [x, np.broadcast_to(one, xs.shape), np.broadcast_to(zero, xs.shape)], alpha=eps)
        return [o]
    s, hp, _ = _run(build)
    y64 = _f64(s, hp)
    var = xs.astype(np.float64).var(-1)
    assert np.abs(y64.mean(-1)).max() < 1e-14
    assert np.abs(y64.var(-1) - var / (var + eps)).max() < 1e-13


# ---- output rounding and validation ----------------------------------------------------------------
def test_rowop_outputs_round_through_fp32_to_the_output_dtype():
    rng = np.random.default_rng(4)
    xs = rng.standard_normal((9, 33)).astype(np.float32)
    def build(b):
        x = b.pool(xs)
        oh = b.pool(np.zeros((9, 33), np.float16))
        ob = b.pool(np.zeros((9, 33), np.uint16))
        b.add("SOFTMAX_LAST", oh, [x])
        b.add("SOFTMAX_LAST", ob, [x])
        return [oh, ob]
    s, hp, (yh, yb) = _run(build)
    y64 = _f64(s, hp)
    f32 = y64.astype(np.float32)
    assert np.array_equal(yh, f32.astype(np.float16))
    assert np.array_equal(yb, torch.from_numpy(f32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16))


def test_rowop_validation():
    b = Builder()
    xi = b.pool(np.zeros((4, 8), np.int32))
    xf = b.pool(np.zeros((4, 8), np.float32))
    of = b.pool(np.zeros((4, 8), np.float32))
    oi = b.pool(np.zeros((4, 8), np.int32))
    b.add("SOFTMAX_LAST", oi, [xi])                                   # integers: not defined
    b.add("SOFTMAX_LAST", of, [xf, xf], n_inputs=2)                   # one input too many
    b.add("MASKED_SOFTMAX_LAST", of, [xf], n_inputs=1)                # the mask is missing
    b.add("LAYERNORM_LAST", of, [xf, xf], n_inputs=2)                 # beta is missing
    b.add("LAYERNORM_LAST", of[:, :0], [xf[:, :0]] * 3)               # empty rows: nothing to do, accepted
    b.add("SOFTMAX_LAST", of, [xf])
    s = b.stream()
    hp = HostPools(s)
    impl = s.impl_for()
    rc = [oracle.validate(hp.tasks, i, impl[i]) for i in range(len(s))]
    assert rc == [-1, -1, -1, -1, 0, 0]
    assert oracle.run_task(hp.tasks, 4, impl[4]) == 0
