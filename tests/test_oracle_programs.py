"""Pins for the oracle's operator programs (elementwise operators given as instruction lists):
every opcode against numpy's own float32 arithmetic (an independent IEEE implementation), the
fused multiply-add against exact rational arithmetic, programs against the already pinned built-in
operators run as separate tasks, register conventions, strided / broadcast / mixed-dtype operands,
and validation."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2604_17861_amd import streams as S
from helpers import Builder, HostPools, run_oracle, bf16_bits_to_f32

OP_P = 200                       # logical op ids the tests bind programs to
P = S.program


def _run_program(code, n_inputs, ins, out, alpha=0.0, extra=None):
    """One task with `code` as its operator; returns the output as the oracle left it."""
    b = Builder()
    views = [b.pool(a) for a in ins]
    o = b.pool(out)
    b.define_program(OP_P, code, n_inputs)
    b.add("COPY", o, views, op_id=OP_P, alpha=alpha)
    if extra:
        extra(b)
    s = b.stream()
    hp, st = run_oracle(s)
    assert np.all(st == 0), st
    p, off = b._locate(o)
    return hp.arrays[p][off: off + o.nbytes].view(o.dtype).reshape(o.shape), s, hp


def _vals(n=4096, seed=0):
    rng = np.random.default_rng(seed)
    v = (rng.standard_normal(n) * np.exp(rng.uniform(-20, 20, n))).astype(np.float32)
    v[:12] = [0.0, -0.0, np.inf, -np.inf, np.nan, 1.0, -1.0, 1e-45, -1e-45, 3.4e38, 88.7, -104.0]
    return v


@pytest.mark.parametrize("name", ["ADD", "SUB", "MUL", "DIV", "MAX", "MIN"])
def test_binary_opcodes_match_numpy_float32(name):
    x, y = _vals(seed=1), np.roll(_vals(seed=2), 5)
    got, _, _ = _run_program(P((name, 0, 0, 1)), 2, [x, y], np.zeros_like(x))
    with np.errstate(all="ignore"):
        want = {"ADD": x + y, "SUB": x - y, "MUL": x * y, "DIV": x / y}.get(name)
    if want is None:
        cmp = (x > y) if name == "MAX" else (x < y)
        want = np.where(np.isnan(x), x, np.where(np.isnan(y), y, np.where(cmp, x, y)))
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))


@pytest.mark.parametrize("name", ["NEG", "ABS", "RELU", "SQRT", "MOV"])
def test_unary_opcodes_match_numpy_float32(name):
    x = _vals(seed=3)
    got, _, _ = _run_program(P((name, 0, 0)), 1, [x], np.zeros_like(x))
    with np.errstate(all="ignore"):
        want = {"NEG": -x, "ABS": np.abs(x), "SQRT": np.sqrt(x), "MOV": x,
                "RELU": np.where(np.isnan(x), x, np.where(x > 0, x, np.float32(0.0)))}[name]
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))


def test_fma_rounds_once_checked_with_exact_rationals():
    rng = np.random.default_rng(4)
    x = rng.standard_normal(300).astype(np.float32)
    y = rng.standard_normal(300).astype(np.float32)
    z = (-(x.astype(np.float64) * y.astype(np.float64))).astype(np.float32)     # cancels: a second rounding would show
    z[::3] = rng.standard_normal(100).astype(np.float32)
    got, _, _ = _run_program(P(("MOV", 4, 2), ("FMA", 4, 0, 1), ("MOV", 0, 4)), 3, [x, y, z], np.zeros_like(x))
    for i in range(300):
        exact = Fraction(float(x[i])) * Fraction(float(y[i])) + Fraction(float(z[i]))
        f = np.float32(float(exact))              # float(Fraction) and float64 -> float32: two correct roundings ...
        # ... which can differ from one rounding only at a float32 tie of the float64 value: rule those out exactly
        lo, hi = np.nextafter(f, np.float32(-np.inf)), np.nextafter(f, np.float32(np.inf))
        best = min((lo, f, hi), key=lambda c: abs(Fraction(float(c)) - exact))
        assert got[i] == best, (i, got[i], best)
    sep = x * y
    assert np.any(got != (sep + z))               # the separately rounded product differs somewhere: FMA really fuses


def test_exp_opcode_is_the_pinned_exp_operator():
    x = np.linspace(-104, 89, 5000).astype(np.float32)
    got, _, _ = _run_program(P(("EXP", 0, 0)), 1, [x], np.zeros_like(x))
    L = oracle.lib()
    want = np.array([L.orc_scalar_op(S.IMPL["EXP"], float(v), 0.0, 0.0, 0.0, 0) for v in x], np.float32)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


def test_registers_alpha_immediates_and_result_convention():
    """r3 = alpha, r4..r7 start at zero, IMM loads a constant, the result is r0 after the last
    instruction (not the last destination), unused inputs read as zero."""
    x = np.arange(1, 9, dtype=np.float32)
    code = P(("ADD", 5, 4, 6),            # r5 = 0 + 0
             ("IMM", 6, 2.5),             # r6 = 2.5
             ("MUL", 7, 0, 3),            # r7 = x * alpha
             ("ADD", 7, 7, 6),            # r7 = x * alpha + 2.5
             ("ADD", 0, 7, 5),            # r0 = r7 + 0
             ("IMM", 7, 99.0))            # a later write to another register does not change the result
    got, _, _ = _run_program(code, 1, [x], np.zeros_like(x), alpha=-3.0)
    assert np.array_equal(got, x * np.float32(-3.0) + np.float32(2.5))
    got, _, _ = _run_program(P(("ADD", 0, 1, 2)), 1, [x], np.zeros_like(x))      # r1, r2: inputs the task does not have
    assert not got.any()


def test_program_equals_the_same_steps_as_separate_built_in_tasks():
    """sigmoid-like chain y = a / (1 + exp(-(x * a))) ... built two ways: one program, and five
    tasks of the pinned built-in operators with fp32 intermediates.  Bit-identical."""
    rng = np.random.default_rng(6)
    x = (rng.standard_normal((37, 50)) * 4).astype(np.float32)
    a = np.float32(0.75)
    code = P(("MUL", 4, 0, 3), ("NEG", 4, 4), ("EXP", 4, 4), ("IMM", 5, 1.0), ("ADD", 4, 4, 5), ("DIV", 0, 3, 4))
    def chain(b):
        xs = b.pool(x.copy())
        t1, t2, t3, t4, y = (b.pool(np.zeros_like(x)) for _ in range(5))
        ones = b.pool(np.ones(1, np.float32))
        al = b.pool(np.full(1, a, np.float32))
        b.add("SCALE", t1, [xs], alpha=float(a))
        b.add("SCALE", t2, [t1], alpha=-1.0)
        b.add("EXP", t3, [t2])
        b.add("ADD", t4, [t3, np.broadcast_to(ones, x.shape)])
        b.add("DIV", y, [np.broadcast_to(al, x.shape), t4])
        chain.y = y
    got, s, hp = _run_program(code, 1, [x], np.zeros_like(x), alpha=float(a), extra=chain)
    b_y = chain.y
    # locate the chain's result in the oracle's pools: it is the last pool but two (ones, alpha follow it)
    arrays = [arr.view(np.float32) for arr in hp.arrays if arr.nbytes == x.nbytes]
    want = arrays[-1].reshape(x.shape)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


@pytest.mark.parametrize("code_dt", [S.F16, S.BF16])
def test_program_on_strided_broadcast_mixed_dtype_operands(code_dt):
    rng = np.random.default_rng(7)
    raw = (rng.standard_normal((6, 40, 24)) * 2).astype(np.float32)
    if code_dt == S.F16:
        xs = raw.astype(np.float16); x32 = xs.astype(np.float32)
    else:
        xs = (raw.view(np.uint32) >> 16).astype(np.uint16); x32 = bf16_bits_to_f32(xs)
    row = rng.standard_normal(40).astype(np.float32)
    b = Builder()
    x = b.pool(xs)
    r = b.pool(row)
    o = b.pool(np.zeros((6, 24, 40), np.float32))
    b.define_program(OP_P, P(("MUL", 0, 0, 1), ("ABS", 0, 0), ("SQRT", 0, 0), ("SUB", 0, 0, 3)), 2)
    b.add("COPY", o, [x.transpose(0, 2, 1), np.broadcast_to(r, (6, 24, 40))], op_id=OP_P, alpha=0.5)
    s = b.stream()
    hp, st = run_oracle(s)
    assert np.all(st == 0)
    p, off = b._locate(o)
    got = hp.arrays[p][off: off + o.nbytes].view(np.float32).reshape(o.shape)
    want = np.sqrt(np.abs(x32.transpose(0, 2, 1) * row[None, None, :])) - np.float32(0.5)
    assert np.array_equal(got.view(np.uint32), want.astype(np.float32).view(np.uint32))


def test_program_validation():
    ok = P(("ADD", 0, 0, 1))
    assert oracle.validate_program(ok, 2) == 0
    assert oracle.validate_program(ok, 0) == -1 and oracle.validate_program(ok, 4) == -1
    assert oracle.validate_program(ok[:0], 1) == -1
    assert oracle.validate_program(np.concatenate([ok] * 33), 2) == -1
    for field, bad in (("op", 14), ("dst", 8), ("a", 8), ("b", 200)):
        c = ok.copy()
        c[field] = bad
        assert oracle.validate_program(c, 2) == -1, field
    # the task must have the program's arity and float tensors
    b = Builder()
    xi = b.pool(np.zeros(8, np.int32))
    xf = b.pool(np.zeros(8, np.float32))
    of = b.pool(np.zeros(8, np.float32))
    oi = b.pool(np.zeros(8, np.int32))
    b.add("COPY", of, [xf], op_id=OP_P)
    b.add("COPY", oi, [xi, xi], op_id=OP_P)
    b.add("COPY", of, [xf, xf], op_id=OP_P)
    s = b.stream()
    hp = HostPools(s)
    assert oracle.run_task_program(hp.tasks, 0, ok, 2) == -1          # one input, program wants two
    assert oracle.run_task_program(hp.tasks, 1, ok, 2) == -1          # integers
    assert oracle.run_task_program(hp.tasks, 2, ok, 2) == 0
