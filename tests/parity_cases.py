"""Stream builders for the parity tests.  Each returns a Stream; the CPU suite checks that every
tensor a case names lies inside its pool and that the oracle accepts and runs it, the GPU suite
runs it through the library and compares with the oracle."""
import numpy as np

from paper_2604_17861_amd import streams as S
from helpers import Builder, np_dtype

ELEMENTWISE = ["ADD", "SUB", "MUL", "DIV", "RELU", "EXP", "GELU_ERF", "GELU_TANH", "SCALE", "FMA", "SUB_EXP", "COPY"]


def to_dtype(v32, code):
    if code == S.F32:
        return v32.astype(np.float32)
    if code == S.F16:
        with np.errstate(over="ignore"):
            return v32.astype(np.float16)
    return (v32.astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)


def special_values():
    return np.array([0.0, -0.0, 1.0, -1.0, 0.5, 3.0, -3.0, 6.0, -6.0, 10.0, -10.0, 65504.0, -65504.0, 1e-8, -1e-8,
                     6e-5, 88.0, -88.0, 100.0, -100.0, np.inf, -np.inf, np.nan, 2049.0, 1.0009766], dtype=np.float32)


def stream_extent_violations(stream):
    """Indices of tasks naming memory outside their pool (host-side bounds check)."""
    bad = []
    T = stream.tasks
    red_ops = {S.OP["SUM_LAST"], S.OP["MAX_LAST"], S.OP["MIN_LAST"]}
    for i in range(len(T)):
        nd = int(T["ndim"][i])
        size = [int(x) for x in T["size"][i][:nd]]
        if any(s == 0 for s in size):
            continue
        for k in range(4):
            p = int(stream.pool_of[i, k])
            if p < 0:
                continue
            rec = T["inp"][i, k] if k < 3 else T["out"][i]
            dims = nd - 1 if (k == 3 and int(T["op_id"][i]) in red_ops) else nd
            es = S.ELEM_SIZE[int(rec["dtype"])]
            span = 0
            for d in range(dims):
                st = 0 if (int(rec["bcast_mask"]) >> d) & 1 else int(rec["stride"][d])
                span += (size[d] - 1) * st
            lo = int(rec["ptr"])
            if lo < 0 or lo + (span + 1) * es > stream.pools[p].nbytes:
                bad.append(i)
                break
    return bad


def elementwise_contiguous(code):
    """All elementwise implementations on contiguous tensors: sizes 1, 7 (scalar tail only), 1000,
    16384 (exactly one chunk), 40003 (three chunks, ragged vector tail), special values, and an
    unaligned base pointer (scalar fallback)."""
    rng = np.random.default_rng(21 + code)
    b = Builder()
    for n in (1, 7, 1000, 16384, 40003):
        vals = rng.standard_normal(n).astype(np.float32) * 2
        if n > 30:
            vals[: len(special_values())] = special_values()
        x = b.pool(to_dtype(vals, code))
        y = b.pool(to_dtype(rng.standard_normal(n).astype(np.float32), code))
        z = b.pool(to_dtype(rng.standard_normal(n).astype(np.float32), code))
        for name in ELEMENTWISE:
            o = b.pool(np.zeros(n, x.dtype))
            b.add(name, o, [x, y, z][: S.ARITY[S.IMPL[name]]], alpha=0.37)
    big = b.pool(to_dtype(rng.standard_normal(5001).astype(np.float32), code))
    o = b.pool(np.zeros(5001, big.dtype))
    b.add("MUL", o[1:], [big[1:], big[:-1]])
    return b.stream("elementwise_contiguous_%d" % code)


def all_16bit_patterns(code):
    """Every 16-bit pattern through each unary implementation, same-dtype and fp32 outputs."""
    bits = np.arange(65536, dtype=np.uint16)
    src = bits.view(np.float16) if code == S.F16 else bits
    b = Builder()
    X = b.pool(src.copy())
    for name in ("COPY", "RELU", "SCALE", "EXP", "GELU_ERF", "GELU_TANH"):
        o = b.pool(np.zeros(65536, src.dtype))
        b.add(name, o, [X], alpha=-1.7)
        o32 = b.pool(np.zeros(65536, np.float32))
        b.add(name, o32, [X], alpha=-1.7)
    return b.stream("all_16bit_%d" % code)


def sub_exp_16bit_patterns(code):
    """exp(x - y) with a 16-bit output for every 16-bit pattern x against sixteen subtrahends y, as a
    per-row scalar (the attention chain's x - rowmax) and as a full operand: the exponential that is
    evaluated for 16-bit outputs must stay within 2 units of the output format of the defined result
    over the whole range (overflow, results below the normal range, NaN, infinities)."""
    bits = np.arange(65536, dtype=np.uint16)
    src = bits.view(np.float16) if code == S.F16 else bits
    ys = np.array([0.0, 1.5, -3.25, 11.0, -11.0, 88.0, -88.0, 0.001, 5.5, -0.75, 20.0, -20.0, 60.0, -60.0, 100.0, -100.0], np.float32)
    b = Builder()
    X = b.pool(np.tile(src, 16).reshape(16, 65536))
    ycol = b.pool(ys)
    o = b.pool(np.zeros((16, 65536), src.dtype))
    b.add("SUB_EXP", o, [X, np.broadcast_to(ycol[:, None], (16, 65536))])            # per-row scalar, fp32
    yfull = b.pool(to_dtype(np.repeat(ys, 65536).reshape(16, 65536), code))
    o = b.pool(np.zeros((16, 65536), src.dtype))
    b.add("SUB_EXP", o, [X, yfull])                                                  # contiguous, same dtype
    o = b.pool(np.zeros(16 * 65536, src.dtype))
    b.add("EXP", o, [X.reshape(-1)])
    return b.stream("sub_exp_16bit_%d" % code)


def fp32_transcendental_sweep():
    rng = np.random.default_rng(5)
    grids = [np.linspace(-6, 6, 200001), np.linspace(-104, 89, 200001), rng.uniform(-3, 3, 200000),
             rng.standard_normal(200000), np.linspace(-20, 20, 100001)]
    b = Builder()
    for g in grids:
        x = b.pool(g.astype(np.float32))
        y = b.pool(rng.standard_normal(len(g)).astype(np.float32))
        for name in ("EXP", "GELU_ERF", "GELU_TANH", "SUB_EXP"):
            o = b.pool(np.zeros(len(g), np.float32))
            b.add(name, o, [x, y][: S.ARITY[S.IMPL[name]]])
    return b.stream("fp32_transcendental")


def random_view(rng, base, shape, p_bcast=0.25):
    """A random strided / broadcast view of `base` (as_strided), checked to stay inside it."""
    nd = len(shape)
    perm = rng.permutation(nd)
    strides = [0] * nd
    acc = 1
    for d in perm:
        if shape[d] == 1 or rng.random() < p_bcast:
            continue
        strides[d] = acc * int(rng.integers(1, 3))
        acc = strides[d] * shape[d]
    start = int(rng.integers(0, 4))
    need = start + sum((shape[d] - 1) * strides[d] for d in range(nd)) + 1
    assert need <= base.size, (need, base.size)
    return np.lib.stride_tricks.as_strided(base[start:], shape=shape, strides=[s * base.itemsize for s in strides],
                                           writeable=False)


def random_strided_views(seed):
    """Random <= 6-D shapes (at most 2^15 elements) with permuted / gapped / broadcast input strides,
    permuted output layouts and mixed dtypes."""
    rng = np.random.default_rng(300 + seed)
    b = Builder()
    bases = {c: b.pool(to_dtype(rng.standard_normal(1 << 21).astype(np.float32), c)) for c in (S.F32, S.F16, S.BF16)}
    names = ["ADD", "SUB", "MUL", "DIV", "FMA", "RELU", "SCALE", "COPY", "SUB_EXP", "GELU_TANH"]
    for _ in range(120):
        nd = int(rng.integers(1, 7))
        shape = [int(rng.integers(1, 9)) for _ in range(nd)]
        while int(np.prod(shape)) > (1 << 15):
            shape[int(np.argmax(shape))] //= 2
        name = names[int(rng.integers(len(names)))]
        ar = S.ARITY[S.IMPL[name]]
        ins = [random_view(rng, bases[int(rng.integers(3))], shape) for _ in range(ar)]
        ocode = int(rng.integers(3))
        obuf = b.pool(np.zeros(int(np.prod(shape)) + 8, bases[ocode].dtype))
        perm = rng.permutation(nd)
        st = [0] * nd
        acc = 1
        for d in perm:
            st[d] = acc
            acc *= shape[d]
        o = np.lib.stride_tricks.as_strided(obuf[int(rng.integers(0, 4)):], shape=shape,
                                            strides=[s * obuf.itemsize for s in st])
        b.add(name, o, ins, alpha=1.25)
    return b.stream("random_views_%d" % seed)


def broadcast_2d():
    """[R, C] op row vector / column vector / per-row scalar of another dtype, C a multiple of the
    vector width and not; several chunks."""
    rng = np.random.default_rng(8)
    b = Builder()
    for code in (S.F32, S.F16, S.BF16):
        for (R_, C_) in ((5, 64), (300, 256), (33, 1000), (130, 520), (7, 77)):
            a = b.pool(to_dtype(rng.standard_normal((R_, C_)).astype(np.float32), code))
            row = b.pool(to_dtype(rng.standard_normal(C_).astype(np.float32), code))
            col = b.pool(to_dtype(rng.standard_normal(R_).astype(np.float32), code))
            col32 = b.pool(rng.standard_normal(R_).astype(np.float32))
            for name, ins in (("ADD", [a, np.broadcast_to(row, (R_, C_))]),
                              ("SUB", [np.broadcast_to(row, (R_, C_)), a]),
                              ("MUL", [a, np.broadcast_to(col[:, None], (R_, C_))]),
                              ("SUB_EXP", [a, np.broadcast_to(col32[:, None], (R_, C_))]),
                              ("DIV", [a, np.broadcast_to(col32[:, None], (R_, C_))]),
                              ("FMA", [a, np.broadcast_to(row, (R_, C_)), np.broadcast_to(col[:, None], (R_, C_))])):
                o = b.pool(np.zeros((R_, C_), a.dtype))
                b.add(name, o, ins)
    return b.stream("broadcast_2d")


def transposed_2d():
    """Contiguous [B, R, C] outputs whose inputs mix transposed views (unit stride along R, column
    pitch >= R), row-major views with a row pitch, broadcast rows and broadcast columns: the
    LDS-tiled gather.  Sizes below, at and across the 32 x 32 tile with ragged edges, several
    chunks, every float dtype pair."""
    rng = np.random.default_rng(9)
    b = Builder()
    shapes = ((1, 8, 8), (1, 33, 65), (3, 40, 31), (2, 100, 260), (1, 257, 1030), (5, 64, 64), (1, 9, 3000))
    for n, (B_, R_, C_) in enumerate(shapes):
        for code in (S.F32, S.F16, S.BF16):
            ocode = (S.F32, S.F16, S.BF16)[(n + code) % 3]
            pad = int(rng.integers(0, 5))
            # stored [B, C, R + pad]: viewed as [B, R, C] its unit stride runs along R
            at = b.pool(to_dtype(rng.standard_normal((B_, C_, R_ + pad)).astype(np.float32), code))
            a_t = at[:, :, :R_].transpose(0, 2, 1)
            bt = b.pool(rng.standard_normal((B_, C_, R_)).astype(np.float32))
            b_t = bt.transpose(0, 2, 1)
            full = b.pool(to_dtype(rng.standard_normal((B_, R_, C_ + 3)).astype(np.float32), code))[:, :, :C_]
            row = np.broadcast_to(b.pool(to_dtype(rng.standard_normal(C_).astype(np.float32), code)), (B_, R_, C_))
            col = np.broadcast_to(b.pool(rng.standard_normal(R_).astype(np.float32))[None, :, None], (B_, R_, C_))
            bsame = np.broadcast_to(b_t[:1], (B_, R_, C_))          # batch stride 0 on a transposed operand
            for name, ins in (("COPY", [a_t]), ("GELU_TANH", [a_t]), ("ADD", [a_t, full]), ("SUB", [full, a_t]),
                              ("MUL", [a_t, b_t]), ("DIV", [a_t, row]), ("SUB_EXP", [a_t, col]),
                              ("FMA", [a_t, b_t, full]), ("FMA", [row, bsame, a_t]), ("SCALE", [b_t])):
                o = b.pool(np.zeros((B_, R_, C_), np_dtype(ocode)))
                if B_ == 1 and name in ("ADD", "MUL"):
                    b.add(name, o[0], [v[0] for v in ins], alpha=0.75)      # rank 2
                else:
                    b.add(name, o, ins, alpha=0.75)
    return b.stream("transposed_2d")


def row_operations():
    """Softmax, scaled + masked softmax and layer norm over the last dim: rows in registers (row
    lengths from one vector to 1024 vectors: sub-wave, whole-wave and whole-workgroup ownership,
    several chunks and ragged last chunks), streamed rows beyond that, and the generic path (odd
    lengths, strided rows, mixed dtypes);
    masks laid out like x, repeated every S rows, or one row; special values."""
    rng = np.random.default_rng(12)
    b = Builder()
    for code in (S.F32, S.F16, S.BF16):
        V = 4 if code == S.F32 else 8
        dt = np_dtype(code)
        for rows, n in ((1, V), (7, 8 * V), (300, 24 * V), (1000, 64 * V), (130, 65 * V), (90, 128 * V),
                        (50, 200 * V), (40, 256 * V), (12, 257 * V), (9, 512 * V), (7, 1000 * V), (5, 1024 * V),
                        (3, 1500 * V), (2, 4096 * V), (33, 5), (65, 1001), (3, 20000)):
            x = b.pool(to_dtype((rng.standard_normal((rows, n)) * 3).astype(np.float32), code))
            o1, o2, o3 = (b.pool(np.zeros((rows, n), dt)) for _ in range(3))
            b.add("SOFTMAX_LAST", o1, [x])
            mrow = b.pool(to_dtype(rng.standard_normal(n).astype(np.float32), code))
            b.add("MASKED_SOFTMAX_LAST", o2, [x, np.broadcast_to(mrow, (rows, n))], alpha=0.3)
            g = b.pool(to_dtype((1 + 0.2 * rng.standard_normal(n)).astype(np.float32), code))
            be = b.pool(to_dtype(rng.standard_normal(n).astype(np.float32), code))
            b.add("LAYERNORM_LAST", o3, [x, np.broadcast_to(g, (rows, n)), np.broadcast_to(be, (rows, n))], alpha=1e-5)
        # attention-shaped: [B, H, S, S] scores, causal mask [S, S] repeated every S rows, and a full-size bias
        for (B_, H_, S_) in ((2, 3, 64), (1, 5, 128), (3, 2, 24)):
            x = b.pool(to_dtype((rng.standard_normal((B_, H_, S_, S_)) * 2).astype(np.float32), code))
            causal = np.where(np.tril(np.ones((S_, S_), bool)), 0.0, -np.inf).astype(np.float32)
            m = b.pool(to_dtype(causal, code))
            o = b.pool(np.zeros((B_, H_, S_, S_), dt))
            b.add("MASKED_SOFTMAX_LAST", o, [x, np.broadcast_to(m, (B_, H_, S_, S_))], alpha=0.125)
            bias = b.pool(to_dtype(rng.standard_normal((B_, H_, S_, S_)).astype(np.float32), code))
            o = b.pool(np.zeros((B_, H_, S_, S_), dt))
            b.add("MASKED_SOFTMAX_LAST", o, [x, bias], alpha=1.0)
            mh = b.pool(to_dtype(rng.standard_normal((H_, 1, S_)).astype(np.float32), code))     # per head, one row
            o = b.pool(np.zeros((B_, H_, S_, S_), dt))
            b.add("MASKED_SOFTMAX_LAST", o, [x, np.broadcast_to(mh[None], (B_, H_, S_, S_))], alpha=0.5)
    # layer norm with fp32 gamma / beta under 16-bit x and y (how frameworks keep the parameters): vector paths
    for code in (S.F16, S.BF16):
        for rows, n in ((9, 64), (40, 768), (33, 1024), (17, 2048), (6, 4096), (5, 8192), (3, 12288)):
            x = b.pool(to_dtype((rng.standard_normal((rows, n)) * 2 + 0.5).astype(np.float32), code))
            g = b.pool((1 + 0.2 * rng.standard_normal(n)).astype(np.float32))
            be = b.pool(rng.standard_normal(n).astype(np.float32))
            o = b.pool(np.zeros((rows, n), np_dtype(code)))
            b.add("LAYERNORM_LAST", o, [x, np.broadcast_to(g, (rows, n)), np.broadcast_to(be, (rows, n))], alpha=1e-5)
    # generic path: strided rows, transposed views, mixed dtypes, fp32 output of 16-bit input
    x16 = b.pool(to_dtype((rng.standard_normal((64, 96)) * 2).astype(np.float32), S.F16))
    x32 = b.pool((rng.standard_normal((96, 64)) * 2).astype(np.float32))
    g32 = b.pool((1 + 0.1 * rng.standard_normal(96)).astype(np.float32))
    be16 = b.pool(to_dtype(rng.standard_normal(96).astype(np.float32), S.BF16))
    o = b.pool(np.zeros((64, 96), np.float32))
    b.add("SOFTMAX_LAST", o, [x16])
    o = b.pool(np.zeros((64, 96), np.float16))
    b.add("SOFTMAX_LAST", o, [x32.T])
    o = b.pool(np.zeros((64, 48), np.float32))
    b.add("MASKED_SOFTMAX_LAST", o, [x16[:, ::2], x32.T[:, 1::2]], alpha=-0.7)
    o = b.pool(np.zeros((64, 96), np.uint16))
    b.add("LAYERNORM_LAST", o, [x16, np.broadcast_to(g32, (64, 96)), np.broadcast_to(be16, (64, 96))], alpha=1e-3)
    o = b.pool(np.zeros((64, 96), np.float32))
    b.add("LAYERNORM_LAST", o, [x32.T, x32.T, x32.T], alpha=0.25)              # per-element gamma and beta
    x4 = b.pool(rng.standard_normal((2, 3, 4, 5, 6, 32)).astype(np.float32))     # six dims, outer dims permuted
    o = b.pool(np.zeros((4, 2, 3, 5, 6, 32), np.float32))
    b.add("SOFTMAX_LAST", o, [x4.transpose(2, 0, 1, 3, 4, 5)])
    # special values
    inf, nan = np.inf, np.nan
    sp = np.zeros((8, 16), np.float32)
    sp[0, 3] = nan
    sp[1, :] = -inf
    sp[2, 5] = inf
    sp[3, ::2] = -inf
    sp[4, :] = 88.0
    sp[5, :] = np.linspace(-120, 0, 16)                 # results far below fp32's normal range
    sp[6, :] = 1e30
    xs = b.pool(sp)
    o = b.pool(np.zeros((8, 16), np.float32))
    b.add("SOFTMAX_LAST", o, [xs])
    o = b.pool(np.zeros((8, 15), np.float32))
    b.add("SOFTMAX_LAST", o, [xs[:, :15]])               # the same through the generic path
    const = b.pool(np.full((4, 64), 3.0, np.float32))   # zero variance: eps alone under the root
    one, zero = b.pool(np.ones(64, np.float32)), b.pool(np.zeros(64, np.float32))
    o = b.pool(np.zeros((4, 64), np.float32))
    b.add("LAYERNORM_LAST", o, [const, np.broadcast_to(one, (4, 64)), np.broadcast_to(zero, (4, 64))], alpha=1e-5)
    return b.stream("row_operations")


def operator_programs():
    """Operators defined as programs: an exactly rounded mix (bit-exact), a leaky-relu-like select by
    max / min, a three-input fma chain, sqrt / abs / neg / div, and two with an exponential inside
    (sigmoid, softplus-like) whose error bound is derived below.  Layouts: contiguous (several
    chunks), row vector and per-row scalar operands, transposed inputs, stride-2 slices, mixed
    dtypes, all float output dtypes."""
    rng = np.random.default_rng(21)
    b = Builder()
    P = S.program
    progs = {
        210: (P(("MUL", 4, 0, 1), ("ADD", 4, 4, 3), ("SUB", 0, 4, 0)), 2),                      # x*y + alpha - x
        211: (P(("IMM", 4, 0.0), ("MAX", 5, 0, 4), ("MIN", 6, 0, 4), ("MUL", 6, 6, 3), ("ADD", 0, 5, 6)), 1),   # leaky relu, slope alpha
        212: (P(("MOV", 4, 2), ("FMA", 4, 0, 1), ("FMA", 4, 4, 3), ("NEG", 0, 4)), 3),          # -(fma(fma(x,y,z), alpha, ...)) chain
        213: (P(("ABS", 4, 0), ("SQRT", 4, 4), ("IMM", 5, 1.0), ("ADD", 5, 5, 4), ("DIV", 0, 0, 5), ("RELU", 0, 0)), 1),   # relu(x / (1 + sqrt|x|))
        214: (P(("NEG", 4, 0), ("EXP", 4, 4), ("IMM", 5, 1.0), ("ADD", 4, 4, 5), ("DIV", 0, 5, 4)), 1),   # sigmoid
        215: (P(("SUB", 4, 0, 1), ("MUL", 4, 4, 3), ("EXP", 4, 4), ("MUL", 0, 4, 1)), 2),       # exp(alpha (x - y)) * y
    }
    impl_of = {op: b.define_program(op, code, nin) for op, (code, nin) in sorted(progs.items())}
    codes = (S.F32, S.F16, S.BF16)
    def T(shape, code, scale=2.0):
        return b.pool(to_dtype((rng.standard_normal(shape) * scale).astype(np.float32), code))
    n = 0
    for code in codes:
        dt = np_dtype(code)
        ocode = codes[(code + 1) % 3]
        for numel in (1000, 16384, 70001):
            x, y, z = T(numel, code), T(numel, code), T(numel, code)
            for op in (210, 211, 212, 213, 214, 215):
                nin = progs[op][1]
                o = b.pool(np.zeros(numel, np_dtype(ocode if op in (211, 214) else code)))
                b.add("COPY", o, [x, y, z][:nin], op_id=op, alpha=0.3)
        R_, C_ = 130, 264
        m = T((R_, C_), code)
        row, col = T(C_, code), b.pool(rng.standard_normal(R_).astype(np.float32))
        mt = T((C_, R_ + 3), code)[:, :R_].T                 # unit stride along R
        wide = T((R_, 2 * C_), code)
        for op, ins in ((210, [m, np.broadcast_to(row, (R_, C_))]), (215, [m, np.broadcast_to(col[:, None], (R_, C_))]),
                        (210, [mt, m]), (212, [mt, np.broadcast_to(row, (R_, C_)), wide[:, ::2]]),
                        (214, [mt]), (213, [wide[:, 1::2]]), (211, [m[::2]])):
            shape = ins[0].shape
            o = b.pool(np.zeros(shape, dt if op != 215 else np.float32))
            b.add("COPY", o, ins, op_id=op, alpha=-0.7)
    s = b.stream("operator_programs")
    # sigmoid: e = exp(-x) within 2 ulp (relative 2^-22); 1 + e inherits at most that (relative to a
    # value >= 1, half an ulp more for the add); the division adds half an ulp: 3 ulp of fp32, and a
    # 16-bit output format absorbs all of it but one step.  exp(alpha (x - y)) * y: 2 ulp then half.
    s.info["program_ulp"] = {impl_of[214]: 4, impl_of[215]: 3}
    return s


def reductions():
    """SUM / MAX / MIN over the last dim: row lengths from 1 to 20000 (sub-wave rows, one workgroup
    per row, scalar fallback for odd lengths), all float dtypes, fp32 and same-dtype outputs,
    strided / transposed inputs, keepdim, NaN and -inf rows."""
    rng = np.random.default_rng(9)
    b = Builder()
    for code in (S.F32, S.F16, S.BF16):
        for rows, n in ((3, 1), (700, 8), (513, 64), (300, 128), (77, 256), (50, 100), (9, 1000), (5, 4096), (3, 20000),
                        (2, 16388), (1100, 32)):
            x32 = rng.uniform(-1, 1, (rows, n)).astype(np.float32)
            if n >= 64:
                x32[0, 3] = np.nan
                x32[1 % rows, :] = -np.inf
            x = b.pool(to_dtype(x32, code))
            for name in ("SUM_LAST", "MAX_LAST", "MIN_LAST"):
                o = b.pool(np.zeros(rows, np.float32)); b.add(name, o, [x])
                o2 = b.pool(np.zeros(rows, x.dtype)); b.add(name, o2, [x])
    t = b.pool(rng.standard_normal((37, 50)).astype(np.float32))
    o = b.pool(np.zeros(50, np.float32)); b.add("SUM_LAST", o, [t.T])
    g = b.pool(rng.standard_normal((6, 5, 4, 66)).astype(np.float16))
    o = b.pool(np.zeros((4, 5, 6), np.float32))
    b.add("MAX_LAST", o.transpose(2, 1, 0), [g[..., ::2]], shape=[6, 5, 4, 33])
    k = b.pool(np.zeros((9, 1), np.float32))
    x = b.pool(rng.standard_normal((9, 300)).astype(np.float32))
    b.add("SUM_LAST", k[:, 0], [x], flags=S.FLAG_KEEPDIM)
    one = b.pool(np.ones((3, 4097), np.float32)); o1 = b.pool(np.zeros(3, np.float32)); b.add("SUM_LAST", o1, [one])
    return b.stream("reductions")


def degenerate():
    """The degenerate cases: empty tensors (nothing may be touched), one-element tensors, six dims of
    size 1, six real dims, rows of one element, in-place updates, an input used twice, an all-broadcast
    operand, NaN payloads and -0 through COPY, outputs that are interior slices of their buffers
    (the bytes around them must survive).  Only exactly rounded operations: the test compares whole
    buffers byte by byte."""
    rng = np.random.default_rng(21)
    b = Builder()
    f = lambda *sh: b.pool(rng.integers(-8, 9, sh).astype(np.float32))
    x, y, o = f(40), f(40), f(40)
    b.add("ADD", o[:0], [x[:0], y[:0]])                                   # empty 1-D
    e3 = f(4, 6, 5)
    b.add("MUL", e3[:, :0, :], [e3[:, :0, :], e3[:, :0, :]])              # empty in the middle dim
    z = f(3, 8); zo = f(3)
    b.add("SUM_LAST", zo[:0], [z[:0]])                                    # no rows
    b.add("SOFTMAX_LAST", z[:0], [z[:0]])                                 # no rows (a row operation)
    b.add("ADD", o[5:6], [x[7:8], y[9:10]])                               # one element, interior output
    s6 = f(1, 1, 1, 1, 1, 1); t6 = f(1, 1, 1, 1, 1, 1); o6 = f(1, 1, 1, 1, 1, 1)
    b.add("SUB", o6, [s6, t6])
    r6 = f(2, 3, 2, 3, 2, 3); q6 = f(3, 2, 3, 2, 3, 2); w6 = f(2, 3, 2, 3, 2, 3)
    b.add("ADD", w6, [r6, q6.transpose(5, 4, 3, 2, 1, 0)])                # six real dims, one operand reversed
    one = f(1, 1); oo = f(1)
    b.add("MAX_LAST", oo, [one])                                          # a row of one element
    col = f(9, 1); co = f(9)
    b.add("SUM_LAST", co, [col])                                          # nine rows of one element
    ip, iq = f(5, 33), f(5, 33)
    b.add("ADD", ip, [ip, iq])                                            # in place
    ir = b.pool(rng.standard_normal((7, 19)).astype(np.float32))
    b.add("RELU", ir[1:6, 2:17], [ir[1:6, 2:17]])                         # in place on an interior block
    tw = f(64); to = f(64)
    b.add("MUL", to, [tw, tw])                                            # the same tensor twice
    sc = f(1, 1); bb = f(3, 4); bo = f(3, 4)
    b.add("ADD", bo, [np.broadcast_to(sc, (3, 4)), bb])                   # an operand broadcast along every dim
    pay = np.array([0x7fc00001, 0xffc12345, 0x80000000, 0x00000001, 0x7f800000, 0xff800000, 0x7f812345, 0], np.uint32)
    cp = b.pool(pay.view(np.float32).copy()); cq = b.pool(np.zeros(10, np.float32))
    b.add("COPY", cq[1:9], [cp])                                          # NaN payloads, -0, a subnormal, infinities
    h = b.pool(np.array([0x7e01, 0xfe02, 0x8000, 0x0001, 0x7c00], np.uint16).view(np.float16).copy()); ho = b.pool(np.zeros(7, np.float16))
    b.add("COPY", ho[1:6], [h])
    mid = f(6, 1, 7); mo = f(6, 1, 7)
    b.add("SUB", mo, [mid, np.broadcast_to(mid[:, :, 3:4], (6, 1, 7))])   # a size-1 dim and a broadcast column
    i32 = b.pool(np.array([2147483647, -2147483648, -1, 0, 5], np.int32)); io = b.pool(np.zeros(7, np.int32))
    b.add("ADD", io[1:6], [i32, i32])                                     # int32 wrap-around, interior output
    return b.stream("degenerate")


def dependency_dag(seed, n_tasks=2500, n_buffers=10, max_dist=48):
    """A random stream of exactly rounded operations over a FEW buffers, so that almost every task
    reads or overwrites what an earlier, possibly still running, task wrote or reads: read-after-write,
    write-after-write and write-after-read hazards, each declared the way a caller must (back-distances
    to the tickets involved; FENCE when there are more than three).  Task sizes from 256 elements to
    256K (many chunks) make completions overtake each other.  The result of the whole stream is
    unique: the test compares every buffer with sequential execution byte for byte."""
    rng = np.random.default_rng(100 + seed)
    b = Builder()
    side = 512
    bufs = [b.pool(rng.integers(-4, 5, (side, side)).astype(np.float32)) for _ in range(n_buffers)]
    last_writer = [None] * n_buffers                 # ticket of the newest task that wrote the buffer
    readers = [[] for _ in range(n_buffers)]         # tickets that read it since
    for t in range(n_tasks):
        rows = int(rng.choice([1, 4, 32, 128, 512]))
        cols = int(rng.choice([256, 512])) if rows > 1 else 256
        r0 = int(rng.integers(0, side - rows + 1))
        c0 = int(rng.integers(0, side - cols + 1))
        view = lambda k: bufs[k][r0: r0 + rows, c0: c0 + cols]
        o = int(rng.integers(2, n_buffers))            # buffers 0 and 1 are never written: the second operands of ADD / SUB,
        name = str(rng.choice(["ADD", "SUB", "RELU", "COPY", "SCALE", "MAX_ROWS"]))   # so magnitudes grow by at most 4 per task
        if name == "MAX_ROWS":                        # a reduction: [rows, cols] -> column r0.. of the output buffer
            i0 = int(rng.integers(n_buffers))
            while i0 == o:
                i0 = int(rng.integers(n_buffers))
            ins, out, impl = [view(i0)], bufs[o][r0: r0 + rows, c0], "MAX_LAST"
        else:
            nin = 2 if name in ("ADD", "SUB") else 1
            ids = [int(rng.integers(n_buffers))] + ([int(rng.integers(2))] if nin == 2 else [])
            ins, out, impl = [view(k) for k in ids], view(o), name       # an input from the output buffer is the same view: in place
        used = [i0] if name == "MAX_ROWS" else ids
        need = set()
        for k in used:
            if last_writer[k] is not None:
                need.add(last_writer[k])             # read after write
        if last_writer[o] is not None:
            need.add(last_writer[o])                 # write after write
        need.update(readers[o])                      # write after read
        need.discard(t)
        dist = sorted(t - w for w in need)
        if len(dist) <= 3 and (not dist or dist[-1] <= max_dist):   # a back-distance must stay inside the ring
            dep, flags = tuple(dist + [0] * (3 - len(dist))), 0
        else:
            dep, flags = (0, 0, 0), S.FLAG_FENCE
        b.add(impl, out, ins, alpha=-1.0 if name == "SCALE" else 0.0, dep=dep, flags=flags)
        for k in used:
            if k != o:
                readers[k].append(t)
        last_writer[o] = t
        readers[o] = []
    return b.stream("dependency_dag_%d" % seed, batch=64)


def producer_with_dependants(n_consumers=1200, n_links=300):
    """The stream shape that needs publication in dependency order: a large task, a large task that
    depends on it (held back by the dispatcher while the first one runs), then more small tasks than
    there are workgroups (with n_consumers = 6400: more than the workgroups can hold between them at
    eight units each) that each read one row of the held task's output, and a chain of four-chunk
    links whose first link reads it too.  Exactly rounded operations on small integers: the buffers at
    the end equal sequential execution byte for byte."""
    rng = np.random.default_rng(77)
    rows, cols = (2048, 1024) if n_consumers <= 2048 else (8192, 256)
    assert n_consumers <= rows
    f = lambda *shape: b.pool(rng.integers(-3, 4, shape).astype(np.float32))
    b = Builder()
    A, B, Cc, D = f(rows, cols), f(rows, cols), f(rows, cols), f(rows, cols)
    X, Y, Z = b.pool(np.zeros((rows, cols), np.float32)), b.pool(np.zeros((rows, cols), np.float32)), b.pool(np.zeros((rows, cols), np.float32))
    b.add("ADD", X, [A, B])                                    # 2M elements: 128 chunks
    b.add("MUL", Y, [X, Cc], dep=(1, 0, 0))                    # large and dependent: held until the ADD is done
    for k in range(n_consumers):                               # one row each, all naming the held task
        b.add("SUB", Z[k], [Y[k], D[k]], dep=(k + 1, 0, 0))
    W, E = b.pool(np.zeros(4 * 8192, np.float32)), f(4 * 8192)
    b.add("ADD", W, [Y.reshape(-1)[: 4 * 8192], E], dep=(n_consumers + 1, 0, 0))     # four chunks, reads the held task's output
    for _ in range(n_links - 1):
        b.add("ADD", W, [W, E], dep=(1, 0, 0))                 # in place, each link after the previous one
    return b.stream("producer_with_dependants", batch=64)


def staged_gathers():
    """Contiguous outputs whose inputs are stride-2 / 3 / 4 / 9 slices at every phase of a 16-byte
    vector, row vectors of odd lengths, column vectors over few rows, batches of small transposes,
    operands of other dtypes, three gathered operands at once, spans too large for the staging
    memory (read element by element instead), also in turn with spans that fit, several chunks with
    a ragged end, special values: the
    layouts the LDS-staged gather path takes, all float dtypes in and out."""
    rng = np.random.default_rng(31)
    b = Builder()
    codes = (S.F32, S.F16, S.BF16)
    def T(shape, code, scale=2.0):
        v = (rng.standard_normal(shape) * scale).astype(np.float32)
        flat = v.reshape(-1)
        if flat.size > 40:
            flat[: len(special_values())] = special_values()
        return b.pool(to_dtype(v, code))
    for code in codes:
        ocode = codes[(code + 1) % 3]
        for numel in (5, 1000, 4096, 70001):
            for stride in (2, 3, 4, 9):
                src = T(numel * stride + 8, code)
                for phase in (0, 1, 3, 7):
                    x = src[phase: phase + numel * stride: stride]
                    o = b.pool(np.zeros(numel, np_dtype(code if phase != 3 else ocode)))
                    b.add("RELU" if phase % 2 else "SCALE", o, [x], alpha=-1.5)
            y2, y3 = T(2 * numel + 3, code), T(3 * numel + 3, ocode)
            o = b.pool(np.zeros(numel, np_dtype(code)))
            b.add("FMA", o, [y2[1::2][:numel], y3[2::3][:numel], T(numel, code)])       # two gathered operands and a contiguous one
            o = b.pool(np.zeros(numel, np_dtype(ocode)))
            b.add("SUB", o, [T(numel, S.F32), np.broadcast_to(T(1, code), (numel,))])   # a scalar operand, mixed dtypes
        for R_, C_ in ((1, 77), (33, 77), (5, 1), (700, 3), (64, 333), (3, 5000), (2, 40000)):
            m = T((R_, C_), code)
            row, col = T(C_, code), T(R_, code)
            o = b.pool(np.zeros((R_, C_), np_dtype(code)))
            b.add("ADD", o, [m, np.broadcast_to(row, (R_, C_))])
            o = b.pool(np.zeros((R_, C_), np_dtype(ocode)))
            b.add("DIV", o, [np.broadcast_to(col[:, None], (R_, C_)), m])
            o = b.pool(np.zeros((R_, C_), np_dtype(code)))
            b.add("MUL", o, [np.broadcast_to(row, (R_, C_)), np.broadcast_to(col[:, None], (R_, C_))])   # outer product: no full operand
        for B_, R_, C_ in ((9, 13, 3), (40, 5, 7), (3, 300, 2), (2, 7, 99)):
            t = T((B_, C_, R_), code).transpose(0, 2, 1)                 # batches of small transposes
            m = T((B_, R_, C_), ocode)
            o = b.pool(np.zeros((B_, R_, C_), np_dtype(code)))
            b.add("SUB", o, [t, m])
            o = b.pool(np.zeros((B_, R_, C_), np_dtype(code)))
            b.add("GELU_TANH", o, [t])
        wide = T((130, 2 * 264), code)
        o = b.pool(np.zeros((130, 264), np_dtype(code)))
        b.add("SUB_EXP", o, [wide[:, ::2], wide[:, 1::2]])               # two column-strided matrices (rows do not merge)
        # rows far apart: a round inside a row stages its window, a round that crosses into the next
        # row has a window too wide for the staging memory, so both kinds alternate within the chunks
        far = T((6, 20000), code)[:, :3000:2]
        o = b.pool(np.zeros((6, 1500), np_dtype(ocode)))
        b.add("ADD", o, [far, T((6, 1500), code)])
        o = b.pool(np.zeros((6, 1500), np_dtype(code)))
        b.add("GELU_TANH", o, [far])
    return b.stream("staged_gathers")


def int32_ops():
    rng = np.random.default_rng(10)
    b = Builder()
    a = b.pool(rng.integers(-2 ** 31, 2 ** 31 - 1, 50000, dtype=np.int64).astype(np.int32))
    c = b.pool(rng.integers(-2 ** 31, 2 ** 31 - 1, 50000, dtype=np.int64).astype(np.int32))
    for name in ("ADD", "SUB", "MUL", "COPY"):
        ar = S.ARITY[S.IMPL[name]]
        o = b.pool(np.zeros(50000, np.int32)); b.add(name, o, [a, c][:ar])
        o = b.pool(np.zeros((100, 250), np.int32))
        b.add(name, o, [a.reshape(250, 200)[:, ::2].T, np.broadcast_to(c[:250], (100, 250))][:ar])
    m = a.reshape(100, 500)
    for name in ("SUM_LAST", "MAX_LAST", "MIN_LAST"):
        o = b.pool(np.zeros(100, np.int32)); b.add(name, o, [m])
        o = b.pool(np.zeros(500, np.int32)); b.add(name, o, [m.T])
    return b.stream("int32")


def config2_reduced():
    return S.config2(n_tasks=2000, in_pool_elems=1 << 21)


def config3_reduced():
    return S.config3(n_chains=12, buffer_sets=1)


def config3_fused_reduced():
    return S.config3_fused(n_chains=12, buffer_sets=1)


def config4_reduced():
    return S.config4(n_tasks=30000, swap_every=2000, window=15000, in_pool_elems=1 << 20)


def config5_reduced():
    return S.config5(n_tasks=300, rows_range=(64, 1024), cols_range=(256, 4096), max_numel=1 << 20,
                     in_pool_bytes=1 << 28, out_slots=300, tile_elems=1 << 22)


CPU_CHECKED = {
    "elementwise_f32": lambda: elementwise_contiguous(S.F32),
    "elementwise_f16": lambda: elementwise_contiguous(S.F16),
    "elementwise_bf16": lambda: elementwise_contiguous(S.BF16),
    "all_16bit_f16": lambda: all_16bit_patterns(S.F16),
    "all_16bit_bf16": lambda: all_16bit_patterns(S.BF16),
    "fp32_transcendental": fp32_transcendental_sweep,
    "sub_exp_16bit_f16": lambda: sub_exp_16bit_patterns(S.F16),
    "sub_exp_16bit_bf16": lambda: sub_exp_16bit_patterns(S.BF16),
    "random_views_0": lambda: random_strided_views(0),
    "random_views_1": lambda: random_strided_views(1),
    "random_views_2": lambda: random_strided_views(2),
    "broadcast_2d": broadcast_2d,
    "staged_gathers": staged_gathers,
    "transposed_2d": transposed_2d,
    "reductions": reductions,
    "operator_programs": operator_programs,
    "row_operations": row_operations,
    "int32": int32_ops,
    "degenerate": degenerate,
    "sequences": lambda: S.sequences(n_seq=40, length=12, interleave=4),
    "dependency_dag": lambda: dependency_dag(0, n_tasks=300),
    "producer_with_dependants": producer_with_dependants,
    "config2_reduced": config2_reduced,
    "config3_reduced": config3_reduced,
    "config3_fused_reduced": config3_fused_reduced,
    "config4_reduced": config4_reduced,
    "config5_reduced": config5_reduced,
}
