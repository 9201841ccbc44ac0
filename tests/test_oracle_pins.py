"""Pins for the CPU oracle: hand values, numpy strided views, exhaustive 16-bit sweeps, closed
forms and invariants.  The paper prints no worked example or tensor values, so nothing here is
copied from it; tests/golden/ holds hand-derived values with the definition they follow."""
import math
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2604_17861_amd import streams as S
from helpers import Builder, run_oracle, ulp_distance, bf16_bits_to_f32

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def run1(name, out, ins, **kw):
    b = Builder()
    bases = {}
    def reg(a):
        root = a
        while root.base is not None:
            root = root.base
        if id(root) not in bases:
            bases[id(root)] = True
            b.bases.append(root)
        return a
    for a in ins:
        reg(a)
    reg(out)
    b.add(name, out, ins, **kw)
    s = b.stream()
    hp, st = run_oracle(s)
    # the oracle wrote into a COPY of the pools; copy results back into `out`
    p = s.pool_of[0, 3]
    root = b.bases[p]
    root.view(np.uint8).reshape(-1)[:] = hp.arrays[p]
    return st[0]


# ---- ABI -------------------------------------------------------------------
def test_abi_layout_matches_generator():
    lay = oracle.abi_layout()
    dt = S.TASK_DT
    assert lay[0] == dt.itemsize and lay[1] == S.TENSOR_DT.itemsize
    assert lay[2] == dt.fields["size"][1] and lay[3] == dt.fields["inp"][1]
    assert lay[4] == dt.fields["out"][1] and lay[5] == dt.fields["alpha"][1]
    assert lay[6] == dt.fields["dep"][1] and lay[7] == S.COMPLETION_DT.itemsize


# ---- 16-bit conversions: exhaustive / against numpy and torch -----------------
def test_f16_to_f32_all_patterns():
    L = oracle.lib()
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float32)
    got = np.array([L.orc_f16_to_f32(int(b)) for b in bits], dtype=np.float32)
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), ref[~nan].view(np.uint32))


def _interesting_floats(rng, n):
    a = rng.standard_normal(n).astype(np.float32) * np.float32(10.0) ** rng.integers(-9, 6, n).astype(np.float32)
    bits = rng.integers(0, 1 << 32, n, dtype=np.uint64).astype(np.uint32).view(np.float32)
    special = np.array([0.0, -0.0, np.inf, -np.inf, np.nan, 65504.0, 65519.99, 65520.0, 65536.0,
                        2049.0, 2051.0, 2050.0, 6.1035156e-05, 6.0975552e-05, 5.9604645e-08,
                        2.9802322e-08, 2.9802326e-08, 8.940697e-08, 1e-10, 1.0009766, 1.0004883,
                        1.0014648], dtype=np.float32)
    return np.concatenate([a, bits, special, -special])


def test_f32_to_f16_matches_numpy_rne():
    L = oracle.lib()
    x = _interesting_floats(np.random.default_rng(11), 20000)
    with np.errstate(over="ignore"):
        ref = x.astype(np.float16).view(np.uint16)
    got = np.array([L.orc_f32_to_f16(float(v)) if not np.isnan(v) else L.orc_f32_to_f16(float("nan"))
                    for v in x], dtype=np.uint16)
    nan = np.isnan(x)
    assert np.array_equal(got[~nan], ref[~nan])
    assert np.all(np.isnan(got[nan].view(np.float16)))
    # every fp16 value converts back to itself (round trip of exact values)
    bits = np.arange(65536, dtype=np.uint16)
    f = bits.view(np.float16).astype(np.float32)
    ok = ~np.isnan(f)
    back = np.array([L.orc_f32_to_f16(float(v)) for v in f[ok]], dtype=np.uint16)
    assert np.array_equal(back, bits[ok])


def test_f16_ties_hand_values():
    L = oracle.lib()
    # 2049 is halfway between 2048 and 2050 -> even mantissa 2048; 2051 -> 2052
    assert np.uint16(L.orc_f32_to_f16(2049.0)).view(np.float16) == 2048.0
    assert np.uint16(L.orc_f32_to_f16(2051.0)).view(np.float16) == 2052.0
    assert L.orc_f32_to_f16(65520.0) == 0x7C00 and L.orc_f32_to_f16(65519.0) == 0x7BFF
    assert L.orc_f32_to_f16(2.0 ** -25) == 0 and L.orc_f32_to_f16(2.0 ** -25 * 1.0001) == 1
    assert L.orc_f32_to_f16(-0.0) == 0x8000


def test_bf16_matches_torch_and_hand_values():
    L = oracle.lib()
    x = _interesting_floats(np.random.default_rng(12), 20000)
    ref = torch.from_numpy(x.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([L.orc_f32_to_bf16(float(v)) for v in x], dtype=np.uint16)
    nan = np.isnan(x)
    assert np.array_equal(got[~nan], ref[~nan])
    assert np.all(np.isnan(bf16_bits_to_f32(got[nan])))
    as_f = lambda u: np.array([u], dtype=np.uint32).view(np.float32)[0]
    assert L.orc_f32_to_bf16(float(as_f(0x3F808000))) == 0x3F80      # tie -> even (down)
    assert L.orc_f32_to_bf16(float(as_f(0x3F818000))) == 0x3F82      # tie -> even (up)
    assert L.orc_f32_to_bf16(float(as_f(0x3F808001))) == 0x3F81
    assert L.orc_f32_to_bf16(3.4e38) == 0x7F80                       # overflow -> inf
    bits = np.arange(65536, dtype=np.uint16)
    got = np.array([L.orc_bf16_to_f32(int(b)) for b in bits], dtype=np.float32).view(np.uint32)
    notnan = ~np.isnan(bf16_bits_to_f32(bits))       # signalling NaNs are quieted on the way through Python floats
    assert np.array_equal((got >> 16)[notnan], bits.astype(np.uint32)[notnan]) and np.all((got & 0xFFFF)[notnan] == 0)
    assert np.all(np.isnan(got.view(np.float32)[~notnan]))


# ---- hand-computed tiny cases ---------------------------------------------------
def test_add_1d_hand():
    a = np.array([1, 2, 3], np.float32); b = np.array([10, 20, 30], np.float32); o = np.zeros(3, np.float32)
    assert run1("ADD", o, [a, b]) == 0
    assert o.tolist() == [11.0, 22.0, 33.0]


def test_broadcast_row_and_column_hand():
    a = np.array([[1, 2, 3], [4, 5, 6]], np.float32)
    row = np.array([10, 20, 30], np.float32); col = np.array([100, 200], np.float32)
    o = np.zeros((2, 3), np.float32)
    run1("ADD", o, [a, np.broadcast_to(row, (2, 3))])
    assert o.tolist() == [[11, 22, 33], [14, 25, 36]]
    run1("ADD", o, [a, np.broadcast_to(col[:, None], (2, 3))])
    assert o.tolist() == [[101, 102, 103], [204, 205, 206]]


def test_broadcast_mask_bit_overrides_stride():
    """bcast_mask bit d forces stride 0 on dim d whatever the stride field says."""
    b = Builder()
    a = b.pool(np.array([[1, 2, 3], [4, 5, 6]], np.float32))
    v = b.pool(np.array([10, 20, 30], np.float32))
    o = b.pool(np.zeros((2, 3), np.float32))
    b.add("ADD", o, [a, np.broadcast_to(v, (2, 3))])
    s = b.stream()
    s.tasks["inp"]["stride"][0, 1, 0] = 7          # nonsense stride, masked out below
    s.tasks["inp"]["bcast_mask"][0, 1] = 0b01
    hp, st = run_oracle(s)
    assert st[0] == 0
    assert hp.arrays[2].view(np.float32).tolist() == [11, 22, 33, 14, 25, 36]


def test_transposed_and_stride2_views_hand():
    base = np.arange(6, dtype=np.float32).reshape(3, 2)      # [[0,1],[2,3],[4,5]]
    o = np.zeros((2, 3), np.float32)
    run1("COPY", o, [base.T])
    assert o.tolist() == [[0, 2, 4], [1, 3, 5]]
    long = np.arange(10, dtype=np.float32)
    o = np.zeros(4, np.float32)
    run1("SCALE", o, [long[1:9:2]], alpha=2.0)               # elements 1,3,5,7
    assert o.tolist() == [2, 6, 10, 14]


def test_unary_hand_values():
    o = np.zeros(3, np.float32)
    run1("RELU", o, [np.array([-1, 0, 2], np.float32)])
    assert o.tolist() == [0, 0, 2]
    run1("RELU", o, [np.array([-0.0, np.nan, -np.inf], np.float32)])
    assert o[0] == 0 and not np.signbit(o[0]) and np.isnan(o[1]) and o[2] == 0
    run1("EXP", o, [np.array([0, 1, -1], np.float32)])
    assert o[0] == 1.0 and o[1] == np.float32(math.e) and o[2] == np.float32(1 / math.e)
    run1("GELU_ERF", o, [np.array([0, 1, -1], np.float32)])
    phi1 = 0.5 * math.erfc(-1 / math.sqrt(2))
    assert o[0] == 0 and o[1] == np.float32(phi1) and o[2] == np.float32(-(1 - phi1))
    run1("GELU_TANH", o, [np.array([0, 1, -1], np.float32)])
    u = math.sqrt(2 / math.pi) * 1.044715
    g = 0.5 * (1 + math.tanh(u))
    assert o[0] == 0 and o[1] == np.float32(g) and abs(float(o[2]) + (1 - g)) < 1e-7


def test_golden_anchor_values():
    """tests/golden/gelu_anchors.txt: 6-digit anchors recomputed from the definitions."""
    L = oracle.lib()
    for line in open(os.path.join(GOLD, "gelu_anchors.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, x, want, tol = line.split()
        got = L.orc_scalar_op(S.IMPL[name], float(x), 0.0, 0.0, 0.0, 0)
        assert abs(got - float(want)) <= float(tol), (name, x, got, want)


def test_binary_scalar_hand_values():
    L = oracle.lib()
    op = lambda n, x, y=0.0, z=0.0, a=0.0: L.orc_scalar_op(S.IMPL[n], x, y, z, a, 0)
    assert op("SUB", 5.0, 7.0) == -2.0 and op("MUL", 3.0, -4.0) == -12.0 and op("DIV", 1.0, 4.0) == 0.25
    assert op("DIV", 1.0, 3.0) == np.float32(1.0) / np.float32(3.0)
    assert op("SCALE", 3.0, a=0.5) == 1.5
    # FMA rounds once: 1+2^-12 squared minus 1 keeps the 2^-24 term a separate multiply would lose
    x = 1.0 + 2.0 ** -12
    assert op("FMA", x, x, -1.0) == 2.0 ** -11 + 2.0 ** -24
    assert np.float32(np.float32(x) * np.float32(x)) - np.float32(1.0) == 2.0 ** -11   # the non-fused value differs
    assert op("SUB_EXP", 2.0, 2.0) == 1.0 and op("SUB_EXP", 1.0, 2.0) == np.float32(math.exp(-1.0))
    assert op("SUB_EXP", -np.inf, 0.0) == 0.0


def test_reductions_hand_values():
    a = np.array([[1, 2, 3], [4, 5, 6]], np.float32)
    o = np.zeros(2, np.float32)
    run1("SUM_LAST", o, [a]); assert o.tolist() == [6, 15]
    run1("MAX_LAST", o, [a]); assert o.tolist() == [3, 6]
    run1("MIN_LAST", o, [a]); assert o.tolist() == [1, 4]
    run1("MAX_LAST", o, [np.array([[1, np.nan, 3], [-np.inf, -5, -7]], np.float32)])
    assert np.isnan(o[0]) and o[1] == -5
    # MIN propagates NaN wherever it stands in the row, and -inf / +inf are ordinary values
    o4 = np.zeros(4, np.float32)
    run1("MIN_LAST", o4, [np.array([[np.nan, 1, 3], [2, 7, np.nan], [np.inf, -5, -np.inf], [np.inf, np.inf, np.inf]], np.float32)])
    assert np.isnan(o4[0]) and np.isnan(o4[1]) and o4[2] == -np.inf and o4[3] == np.inf
    run1("MAX_LAST", o4, [np.array([[3, 1, np.nan], [np.nan, 7, 2], [-np.inf, -5, np.inf], [-np.inf, -np.inf, -np.inf]], np.float32)])
    assert np.isnan(o4[0]) and np.isnan(o4[1]) and o4[2] == np.inf and o4[3] == -np.inf
    # reduce a transposed view: column sums of a
    o3 = np.zeros(3, np.float32)
    run1("SUM_LAST", o3, [a.T]); assert o3.tolist() == [5, 7, 9]
    # keepdim output [2,1]
    ok = np.zeros((2, 1), np.float32)
    b = Builder(); A = b.pool(a); O = b.pool(ok)
    b.add("SUM_LAST", O[:, 0], [A], flags=S.FLAG_KEEPDIM)
    hp, st = run_oracle(b.stream()); assert hp.arrays[1].view(np.float32).tolist() == [6, 15]


def test_sequential_fp32_accumulation_order():
    """SUM_LAST accumulates left to right in fp32: 2^24 + 1 + 1 ... stays 2^24, reversed it grows."""
    row = np.array([2.0 ** 24] + [1.0] * 8, np.float32)
    o = np.zeros(1, np.float32)
    run1("SUM_LAST", o, [row[None, :]]); assert o[0] == 2.0 ** 24
    run1("SUM_LAST", o, [row[::-1].copy()[None, :]]); assert o[0] == 2.0 ** 24 + 8


def test_int32_ops_wrap():
    a = np.array([2147483647, -5, 7], np.int32); b = np.array([1, 3, -2], np.int32); o = np.zeros(3, np.int32)
    run1("ADD", o, [a, b]); assert o.tolist() == [-2147483648, -2, 5]
    run1("SUB", o, [a, b]); assert o.tolist() == [2147483646, -8, 9]
    run1("MUL", o, [a, b]); assert o.tolist() == [2147483647, -15, -14]
    o1 = np.zeros(1, np.int32)
    run1("SUM_LAST", o1, [np.array([[2147483647, 1, 5]], np.int32)]); assert o1[0] == -2147483648 + 5
    run1("MAX_LAST", o1, [a[None, :]]); assert o1[0] == 2147483647
    run1("MIN_LAST", o1, [a[None, :]]); assert o1[0] == -5


def test_validation_rules():
    b = Builder()
    a = b.pool(np.zeros((2, 3), np.float32)); o = b.pool(np.zeros((2, 3), np.float32))
    i32 = b.pool(np.zeros((2, 3), np.int32))
    b.add("ADD", o, [a, a])
    s = b.stream(); hp = __import__("helpers").HostPools(s)
    T = hp.tasks
    v = lambda impl="ADD": oracle.validate(T, 0, S.IMPL[impl])
    assert v() == 0
    T["ndim"][0] = 7; assert v() == -1; T["ndim"][0] = 0; assert v() == -1; T["ndim"][0] = 2
    T["n_inputs"][0] = 1; assert v() == -1; T["n_inputs"][0] = 2
    T["out"]["bcast_mask"][0] = 1; assert v() == -1; T["out"]["bcast_mask"][0] = 0
    T["out"]["stride"][0, 1] = 0; assert v() == -1; T["out"]["stride"][0, 1] = 1
    T["inp"]["stride"][0, 0, 0] = -1; assert v() == -1; T["inp"]["stride"][0, 0, 0] = 3
    T["inp"]["ptr"][0, 1] = 0; assert v() == -1; T["inp"]["ptr"][0, 1] = T["inp"]["ptr"][0, 0]
    T["inp"]["ptr"][0, 1] += 2; assert v() == -1       # a 32-bit element at an address that is no multiple of 4
    T["out"]["ptr"][0] += 1; T["inp"]["ptr"][0, 1] -= 2; assert v() == -1
    T["out"]["ptr"][0] -= 1; assert v() == 0
    T["inp"]["dtype"][0, 0] = 9; assert v() == -1; T["inp"]["dtype"][0, 0] = S.I32
    assert v() == -1                                   # int and float tensors mixed
    T["inp"]["dtype"][0, 0] = S.F32
    T["size"][0, 0] = 1 << 31; assert v() == -1; T["size"][0, 0] = 2
    assert oracle.validate(T, 0, 99) == -3 and oracle.validate(T, 0, 0) == -3
    assert oracle.run_task(T, 0, S.IMPL["FAIL"]) == -3
    for k in ("inp",):
        T[k]["dtype"][0, :2] = S.I32
    T["out"]["dtype"][0] = S.I32
    assert v("ADD") == 0 and v("DIV") == -1           # DIV is not defined on I32


# ---- numpy as the independent index walker ----------------------------------------
def _random_view(rng, base, shape):
    """A random strided / broadcast view of `base` with the given shape (as_strided)."""
    nd = len(shape)
    perm = rng.permutation(nd)
    strides = [0] * nd
    acc = 1
    bc = [bool(rng.random() < 0.25) for _ in range(nd)]
    for d in perm:
        if bc[d] or shape[d] == 1:
            strides[d] = 0
            continue
        gap = int(rng.integers(1, 3))
        strides[d] = acc * gap
        acc = strides[d] * shape[d]
    start = int(rng.integers(0, 4))
    need = start + sum((shape[d] - 1) * strides[d] for d in range(nd)) + 1
    assert need <= base.size
    return np.lib.stride_tricks.as_strided(base[start:], shape=shape,
                                           strides=[s * base.itemsize for s in strides], writeable=False)


@pytest.mark.parametrize("seed", range(6))
def test_random_6d_views_against_numpy(seed):
    """Random <=6-D shapes, strides and broadcast dims: the oracle's div/mod walker against
    numpy's own strided iteration (fp32 add / mul / fma-free ops are exact, so bit equality)."""
    rng = np.random.default_rng(100 + seed)
    b = Builder()
    base = b.pool(rng.standard_normal(1 << 16).astype(np.float32))
    outs = []
    for _ in range(40):
        nd = int(rng.integers(1, 7))
        shape = [int(rng.integers(1, 5)) for _ in range(nd)]
        x = _random_view(rng, base, shape)
        y = _random_view(rng, base, shape)
        name = ["ADD", "SUB", "MUL", "DIV"][int(rng.integers(4))]
        # output: contiguous or a permuted-layout view of its own buffer
        obuf = b.pool(np.zeros(int(np.prod(shape)) * 2 + 8, np.float32))
        perm = rng.permutation(nd)
        st = [0] * nd; acc = 1
        for d in perm:
            st[d] = acc; acc *= shape[d]
        o = np.lib.stride_tricks.as_strided(obuf[int(rng.integers(0, 4)):], shape=shape,
                                            strides=[s * 4 for s in st])
        b.add(name, o, [x, y])
        with np.errstate(all="ignore"):
            ref = {"ADD": x + y, "SUB": x - y, "MUL": x * y, "DIV": x / y}[name]
        outs.append((len(b.bases) - 1, o, ref.astype(np.float32)))
    s = b.stream()
    hp, st = run_oracle(s)
    assert np.all(st == 0)
    for p, o, ref in outs:
        obuf = hp.arrays[p].view(np.float32)
        off = (o.ctypes.data - b.bases[p].ctypes.data) // 4
        got = np.lib.stride_tricks.as_strided(obuf[off:], shape=o.shape, strides=o.strides)
        assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))


def test_reduction_views_against_numpy_float64_and_int():
    rng = np.random.default_rng(7)
    b = Builder()
    base = b.pool(rng.standard_normal(1 << 14).astype(np.float32))
    ibase = b.pool(rng.integers(-1000, 1000, 1 << 12).astype(np.int32))
    checks = []
    for _ in range(30):
        nd = int(rng.integers(1, 6))
        shape = [int(rng.integers(1, 6)) for _ in range(nd)]
        x = _random_view(rng, base, shape)
        oshape = shape[:-1]
        o = b.pool(np.zeros(max(1, int(np.prod(oshape))), np.float32))
        ov = o[: int(np.prod(oshape))].reshape(oshape) if oshape else o[:1].reshape(())
        name = ["SUM_LAST", "MAX_LAST", "MIN_LAST"][int(rng.integers(3))]
        b.add(name, ov, [x], shape=shape)
        ref = {"SUM_LAST": x.astype(np.float64).sum(-1), "MAX_LAST": x.max(-1), "MIN_LAST": x.min(-1)}[name]
        checks.append((len(b.bases) - 1, name, np.asarray(ref).reshape(-1)))
    xi = ibase[:600].reshape(4, 5, 30)[:, :, ::2]
    oi = b.pool(np.zeros(20, np.int32))
    b.add("SUM_LAST", oi.reshape(4, 5), [xi], shape=[4, 5, 15])
    s = b.stream()
    hp, st = run_oracle(s)
    assert np.all(st == 0)
    for p, name, ref in checks:
        got = hp.arrays[p].view(np.float32)[: len(ref)]
        if name == "SUM_LAST":
            assert np.allclose(got, ref, rtol=1e-6, atol=1e-6)
        else:
            assert np.array_equal(got, ref.astype(np.float32))
    assert np.array_equal(hp.arrays[-1].view(np.int32), xi.sum(-1, dtype=np.int32).reshape(-1))


# ---- closed forms ------------------------------------------------------------------
def test_gelu_closed_forms_dense_sweep():
    """mode 0 equals the double-precision closed form rounded once; the tanh form and the
    sigmoid form agree in double to 1e-15 (the identity the oracle's formula relies on)."""
    L = oracle.lib()
    xs = np.linspace(-6, 6, 4001).astype(np.float32)
    for x in xs:
        xd = float(x)
        e = np.float32(0.5 * xd * math.erfc(-xd / math.sqrt(2.0)))
        assert L.orc_scalar_op(S.IMPL["GELU_ERF"], xd, 0, 0, 0, 0) == e
        u = math.sqrt(2 / math.pi) * (xd + 0.044715 * xd ** 3)
        t = 0.5 * xd * (1 + math.tanh(u))
        g = xd / (1 + math.exp(-2 * u))
        assert abs(t - g) <= 1e-15 * max(1.0, abs(t)) + 1e-16
        assert L.orc_scalar_op(S.IMPL["GELU_TANH"], xd, 0, 0, 0, 0) == np.float32(g)
        # the textbook 0.5 x (1 + erf) form agrees away from the cancellation region
        if xd > -1:
            assert abs(0.5 * xd * (1 + math.erf(xd / math.sqrt(2))) - float(e)) <= 2e-7 * max(1e-3, abs(xd))


def test_fp32_libm_mode_close_to_double_mode_for_exp():
    L = oracle.lib()
    xs = np.linspace(-20, 20, 2001).astype(np.float32)
    a = np.array([L.orc_scalar_op(S.IMPL["EXP"], float(x), 0, 0, 0, 0) for x in xs], np.float32)
    c = np.array([L.orc_scalar_op(S.IMPL["EXP"], float(x), 0, 0, 0, 1) for x in xs], np.float32)
    assert ulp_distance(a.view(np.uint32), c.view(np.uint32), S.F32).max() <= 1
    ref = np.exp(xs.astype(np.float64)).astype(np.float32)
    assert np.array_equal(a, ref)


@pytest.mark.parametrize("dt", [np.float16, np.uint16])
def test_all_16bit_patterns_through_unary_ops(dt):
    """Every fp16 / bf16 bit pattern through each unary op: COPY is the bit identity (NaN payloads
    and -0 included); RELU / SCALE / EXP against numpy computed from the exact fp32 value."""
    bits = np.arange(65536, dtype=np.uint16)
    src = bits.view(np.float16) if dt == np.float16 else bits
    code = S.F16 if dt == np.float16 else S.BF16
    f = src.astype(np.float32) if dt == np.float16 else bf16_bits_to_f32(bits)
    b = Builder()
    X = b.pool(src.copy())
    outs = {n: b.pool(np.zeros(65536, dt)) for n in ("COPY", "RELU", "SCALE", "EXP")}
    of32 = b.pool(np.zeros(65536, np.float32))
    for n, o in outs.items():
        b.add(n, o, [X], alpha=0.5)
    b.add("COPY", of32, [X])                        # widening copy = exact conversion
    hp, st = run_oracle(b.stream()); assert np.all(st == 0)
    get = lambda k: hp.arrays[1 + k].view(np.uint16)
    assert np.array_equal(get(0), bits)
    nan = np.isnan(f)
    wide = hp.arrays[5].view(np.float32)
    assert np.array_equal(wide[~nan].view(np.uint32), f[~nan].view(np.uint32)) and np.all(np.isnan(wide[nan]))
    def narrow(v):
        if dt == np.float16:
            with np.errstate(over="ignore"):
                return v.astype(np.float16).view(np.uint16)
        return torch.from_numpy(v.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    relu = np.where(f > 0, f, np.float32(0))
    assert np.array_equal(get(1)[~nan], narrow(relu)[~nan])
    with np.errstate(all="ignore"):
        assert np.array_equal(get(2)[~nan], narrow(f * np.float32(0.5))[~nan])
        ex = np.exp(f.astype(np.float64)).astype(np.float32)
    assert np.array_equal(get(3)[~nan], narrow(ex)[~nan])


# ---- invariants ----------------------------------------------------------------------
def test_broadcast_equals_explicit_expand_and_strided_equals_copy():
    rng = np.random.default_rng(5)
    b = Builder()
    a = b.pool(rng.standard_normal((7, 33)).astype(np.float32))
    v = b.pool(rng.standard_normal(33).astype(np.float32))
    vexp = b.pool(np.broadcast_to(v, (7, 33)).copy())
    big = b.pool(rng.standard_normal((33, 14)).astype(np.float32))
    tcopy = b.pool(big[:, ::2].T.copy())
    o = [b.pool(np.zeros((7, 33), np.float32)) for _ in range(4)]
    b.add("MUL", o[0], [a, np.broadcast_to(v, (7, 33))])
    b.add("MUL", o[1], [a, vexp])
    b.add("SUB", o[2], [a, big[:, ::2].T])
    b.add("SUB", o[3], [a, tcopy])
    hp, st = run_oracle(b.stream())
    r = [hp.arrays[5 + k] for k in range(4)]
    assert np.array_equal(r[0], r[1]) and np.array_equal(r[2], r[3])
    # commutativity and x - x
    b2 = Builder(); A = b2.pool(a); V = b2.pool(vexp); O = [b2.pool(np.zeros((7, 33), np.float32)) for _ in range(3)]
    b2.add("ADD", O[0], [A, V]); b2.add("ADD", O[1], [V, A]); b2.add("SUB", O[2], [A, A])
    hp, _ = run_oracle(b2.stream())
    assert np.array_equal(hp.arrays[2], hp.arrays[3]) and not hp.arrays[4].view(np.float32).any()


def test_sum_of_ones_is_n_and_max_is_an_element():
    b = Builder()
    for n in (1, 2, 1000, 4097):
        ones = b.pool(np.ones((3, n), np.float32)); o = b.pool(np.zeros(3, np.float32))
        b.add("SUM_LAST", o, [ones])
    rng = np.random.default_rng(3)
    x = b.pool(rng.standard_normal((16, 77)).astype(np.float16)); om = b.pool(np.zeros(16, np.float16))
    b.add("MAX_LAST", om, [x])
    hp, _ = run_oracle(b.stream())
    for k, n in enumerate((1, 2, 1000, 4097)):
        assert hp.arrays[2 * k + 1].view(np.float32).tolist() == [n] * 3
    got = hp.arrays[-1].view(np.float16)
    assert np.array_equal(got, x.max(-1))


def test_softmax_chain_properties():
    """Third configuration, tiny: rows sum to 1, zeros above the diagonal, and the chain matches a
    direct double-precision causal softmax of s/8 within fp16 rounding of each step."""
    s = S.config3(n_chains=3, seed=2, buffer_sets=1, heads=2, Bs=(1, 2), Ss=(64,))
    hp, st = run_oracle(s)
    assert np.all(st == 0)
    for c in range(3):
        b_, s_ = s.info["pairs"][s.info["chain_pair"][c]]
        lay = s.info["layout"][(b_, s_)][s.info["chain_set"][c]]
        n = b_ * 2 * s_ * s_
        if c != 2 and s.info["chain_pair"][c] == s.info["chain_pair"][2]:
            continue                                    # overwritten by the later chain on the same set
        sc = hp.view(lay["s"], 0, n, S.F16).astype(np.float64).reshape(b_, 2, s_, s_)
        p = hp.view(lay["w"], lay["p"], n, S.F16).astype(np.float64).reshape(b_, 2, s_, s_)
        z = sc / 8.0 + np.triu(np.full((s_, s_), -np.inf), 1)
        z = z - z.max(-1, keepdims=True)
        ref = np.exp(z); ref /= ref.sum(-1, keepdims=True)
        assert np.all(p[..., np.triu_indices(s_, 1)[0], np.triu_indices(s_, 1)[1]] == 0)
        assert np.abs(p.sum(-1) - 1).max() <= s_ * 2.0 ** -11
        assert np.abs(p - ref).max() <= 4 * 2.0 ** -11
        m = hp.view(lay["w"], lay["m"], b_ * 2 * s_, S.F32)
        t2 = hp.view(lay["w"], lay["t2"], n, S.F16).reshape(-1, s_)
        assert np.array_equal(m, t2.max(-1).astype(np.float32))


def test_sum_last_f64_helper_matches_numpy():
    rng = np.random.default_rng(9)
    b = Builder()
    x = b.pool(rng.uniform(-1, 1, (5, 1000)).astype(np.float32)); o = b.pool(np.zeros(5, np.float32))
    b.add("SUM_LAST", o, [x])
    s = b.stream(); hp, _ = run_oracle(s)
    sm, l1 = oracle.sum_last_f64(hp.tasks, 0, 5)
    assert np.allclose(sm, x.astype(np.float64).sum(-1), rtol=1e-14)
    assert np.allclose(l1, np.abs(x.astype(np.float64)).sum(-1), rtol=1e-14)
    got = hp.arrays[1].view(np.float32)
    assert np.all(np.abs(got - sm) <= 1e-5 * np.maximum(np.abs(sm), l1 / math.sqrt(1000)))


# ---- planted mistakes: a wrong oracle would be caught ------------------------------------
def test_pins_detect_transposed_operand_and_dropped_broadcast():
    """Sanity of the pins themselves: the numpy reference differs when an operand is transposed or a
    broadcast dim is ignored, so an oracle with that mistake could not pass the tests above."""
    a = np.arange(6, dtype=np.float32).reshape(2, 3)
    assert not np.array_equal(a + a, a + a.T.reshape(2, 3))
    v = np.array([1, 2, 3], np.float32)
    assert not np.array_equal(a + v, a + np.arange(6, dtype=np.float32).reshape(2, 3))
