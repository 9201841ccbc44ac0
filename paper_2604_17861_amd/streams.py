"""Seeded synthetic task streams (the five benchmark configurations).

This module only LAYS OUT work: it draws shapes, strides, dtypes, operator ids
and input values with numpy's seeded generator and writes task descriptors in
the C ABI layout.  It contains none of the method's arithmetic (no operator is
evaluated here, no dtype rounding is implemented: 16-bit inputs are produced by
numpy's own float16 cast or by keeping the upper half of a float32), so the
same arrays can drive both the GPU library and the CPU oracle.

The streams stand in for the paper's workloads, which Section 6.1 describes
only by shape: sequences of elementwise operations on 1K-16K-element tensors,
attention decoding, mixed pipelines.  No dataset or benchmark suite is involved.

A stream keeps tensor addresses as (pool index, byte offset); `materialize`
turns them into absolute pointers for a given set of pool base addresses
(device memory for the library, host arrays for the oracle).
"""
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np

MAX_DIMS = 6

# ---- C ABI mirrors (include/gpuos.h) ---------------------------------------
TENSOR_DT = np.dtype([("ptr", "<u8"), ("stride", "<i8", (MAX_DIMS,)), ("dtype", "u1"),
                      ("bcast_mask", "u1"), ("reserved", "u1", (6,))])
TASK_DT = np.dtype([("op_id", "<u2"), ("ndim", "u1"), ("n_inputs", "u1"), ("flags", "<u4"),
                    ("size", "<i8", (MAX_DIMS,)), ("inp", TENSOR_DT, (3,)), ("out", TENSOR_DT),
                    ("alpha", "<f4"), ("dep", "<u2", (3,)), ("reserved", "<u2", (3,))])
COMPLETION_DT = np.dtype([("ticket", "<u8"), ("status", "<i4"), ("op_version", "<u4"),
                          ("t_submit_ns", "<u8"), ("t_done_ns", "<u8")])
assert TENSOR_DT.itemsize == 64 and TASK_DT.itemsize == 328 and COMPLETION_DT.itemsize == 32

F32, F16, BF16, I32 = 0, 1, 2, 3
ELEM_SIZE = {F32: 4, F16: 2, BF16: 2, I32: 4}

IMPL = dict(NONE=0, ADD=1, SUB=2, MUL=3, DIV=4, RELU=5, EXP=6, GELU_ERF=7, GELU_TANH=8, SCALE=9,
            FMA=10, SUB_EXP=11, COPY=12, SUM_LAST=13, MAX_LAST=14, MIN_LAST=15, FAIL=16,
            SOFTMAX_LAST=17, MASKED_SOFTMAX_LAST=18, LAYERNORM_LAST=19)
IMPL_NAME = {v: k for k, v in IMPL.items()}
ARITY = {1: 2, 2: 2, 3: 2, 4: 2, 5: 1, 6: 1, 7: 1, 8: 1, 9: 1, 10: 3, 11: 2, 12: 1, 13: 1, 14: 1,
         15: 1, 16: 1, 17: 1, 18: 2, 19: 3}
REDUCTIONS = (13, 14, 15)
ROWOPS = (17, 18, 19)          # fused row operations: the output has the input's full shape

# Logical operator ids the streams use.  They differ from the impl ids on
# purpose (id = impl + 32) so that a mix-up of the two shows; OP_GELU is the
# hot-swapped entry of the fourth configuration.
OP = {name: code + 32 for name, code in IMPL.items() if name not in ("NONE",)}
OP_GELU = 80

FLAG_FENCE, FLAG_KEEPDIM = 1, 2

# Operator programs (elementwise operators defined at run time as instruction lists): impl ids from
# PROGRAM_BASE name the programs a context (or a test) has defined.  Eight fp32 registers: r0..r2 the
# inputs, r3 alpha, r4..r7 zero; each instruction dst = op(a, b); the result is r0.
PROGRAM_BASE = 64
INSTR_DT = np.dtype([("op", "u1"), ("dst", "u1"), ("a", "u1"), ("b", "u1"), ("imm", "<f4")])
PC = dict(MOV=0, IMM=1, ADD=2, SUB=3, MUL=4, DIV=5, FMA=6, MAX=7, MIN=8, NEG=9, ABS=10, RELU=11, EXP=12, SQRT=13)
PC_INEXACT = (PC["EXP"],)


def program(*instrs):
    """Assemble ('ADD', dst, a, b) / ('IMM', dst, value) / ('NEG', dst, a) ... tuples."""
    code = np.zeros(len(instrs), dtype=INSTR_DT)
    for i, ins in enumerate(instrs):
        name = ins[0]
        code[i]["op"] = PC[name]
        code[i]["dst"] = ins[1]
        if name == "IMM":
            code[i]["imm"] = ins[2]
        else:
            code[i]["a"] = ins[2]
            code[i]["b"] = ins[3] if len(ins) > 3 else 0
    return code


def default_table() -> Dict[int, int]:
    """logical op id -> impl id as registered before any stream starts."""
    t = {OP[name]: IMPL[name] for name in OP}
    t[OP_GELU] = IMPL["GELU_ERF"]
    return t


@dataclass
class Pool:
    name: str
    nbytes: int
    data: Optional[np.ndarray] = None       # uint8 host image (None: output-only, starts zeroed)
    tile: Optional[np.ndarray] = None       # uint8 block repeated to fill the pool (large pools)

    def host_image(self) -> np.ndarray:
        if self.data is not None:
            return self.data
        if self.tile is not None:
            reps = -(-self.nbytes // self.tile.nbytes)
            return np.tile(self.tile, reps)[: self.nbytes]
        return np.zeros(self.nbytes, dtype=np.uint8)


@dataclass
class Stream:
    name: str
    tasks: np.ndarray                        # TASK_DT, ptr fields = byte offsets inside pools
    pool_of: np.ndarray                      # int16 [n, 4] pool index of in0, in1, in2, out (-1 unused)
    pools: List[Pool]
    table: Dict[int, int] = field(default_factory=default_table)
    swaps: List[Tuple[int, int, int]] = field(default_factory=list)  # (before task index, op id, impl)
    batch: int = 0                           # submit batch size (0 = one batch)
    info: dict = field(default_factory=dict)
    programs: Dict[int, Tuple[np.ndarray, int]] = field(default_factory=dict)   # impl id >= PROGRAM_BASE -> (INSTR_DT code, n_inputs)

    def __len__(self):
        return len(self.tasks)

    def materialize(self, bases, out_bases=None) -> np.ndarray:
        """Copy of the task array with absolute pointers: ptr = bases[pool] + offset.
        out_bases (optional) gives different base addresses for the output tensors."""
        out = self.tasks.copy()
        bases = np.asarray(bases, dtype=np.uint64)
        obases = bases if out_bases is None else np.asarray(out_bases, dtype=np.uint64)
        for k in range(3):
            used = self.pool_of[:, k] >= 0
            idx = np.where(used, self.pool_of[:, k], 0)
            out["inp"]["ptr"][:, k] = np.where(used, bases[idx] + self.tasks["inp"]["ptr"][:, k], 0)
        idx = self.pool_of[:, 3]
        out["out"]["ptr"] = obases[idx] + self.tasks["out"]["ptr"]
        return out

    def impl_for(self, versions=None) -> np.ndarray:
        """impl id of every task.  Without hot swaps this is the table lookup; with swaps the
        recorded per-task versions decide (version v of an op is its v-th binding)."""
        n = len(self.tasks)
        hist = {op: [impl] for op, impl in self.table.items()}
        for _, op, impl in self.swaps:
            hist[op].append(impl)
        ops = self.tasks["op_id"]
        out = np.zeros(n, dtype=np.int32)
        for op, h in hist.items():
            sel = ops == op
            if not sel.any():
                continue
            if versions is None or len(h) == 1:
                out[sel] = h[0]
            else:
                v = np.asarray(versions)[sel].astype(np.int64)
                harr = np.asarray(h, dtype=np.int32)
                out[sel] = harr[np.clip(v - 1, 0, len(h) - 1)]
        return out


# ---- helpers ----------------------------------------------------------------

def contiguous_strides(shape):
    st = [0] * len(shape)
    acc = 1
    for d in range(len(shape) - 1, -1, -1):
        st[d] = acc
        acc *= int(shape[d])
    return st


def _align(x, a=256):
    return (int(x) + a - 1) // a * a


def new_tasks(n):
    return np.zeros(n, dtype=TASK_DT), np.full((n, 4), -1, dtype=np.int16)


def set_tensor(tasks, pool_of, i, slot, pool, byte_off, strides, dtype, bcast_mask=0):
    """slot 0..2 = inputs, 3 = output."""
    rec = tasks["inp"][i, slot] if slot < 3 else tasks["out"][i]
    rec["ptr"] = byte_off
    st = np.zeros(MAX_DIMS, dtype=np.int64)
    st[: len(strides)] = strides
    rec["stride"] = st
    rec["dtype"] = dtype
    rec["bcast_mask"] = bcast_mask
    if slot < 3:
        tasks["inp"][i, slot] = rec
    else:
        tasks["out"][i] = rec
    pool_of[i, slot] = pool


def set_head(tasks, i, op_id, shape, n_inputs, alpha=0.0, dep=(0, 0, 0), flags=0):
    tasks["op_id"][i] = op_id
    tasks["ndim"][i] = len(shape)
    tasks["n_inputs"][i] = n_inputs
    tasks["flags"][i] = flags
    sz = np.zeros(MAX_DIMS, dtype=np.int64)
    sz[: len(shape)] = shape
    tasks["size"][i] = sz
    tasks["alpha"][i] = alpha
    tasks["dep"][i] = dep


def random_values(rng, n, dist, dtype):
    """n seeded input values as raw bytes (uint8 view) in the given element type."""
    if dist == "uniform1":
        v = rng.uniform(-1.0, 1.0, n).astype(np.float32)
    elif dist == "uniform3":
        v = rng.uniform(-3.0, 3.0, n).astype(np.float32)
    elif dist == "normal1":
        v = rng.standard_normal(n, dtype=np.float32)
    elif dist == "normal2":
        v = (2.0 * rng.standard_normal(n, dtype=np.float32)).astype(np.float32)
    else:
        raise ValueError(dist)
    if dtype == F32:
        return v.view(np.uint8)
    if dtype == F16:
        return v.astype(np.float16).view(np.uint8)
    if dtype == BF16:                       # keep the upper half of the float32 pattern
        return (v.view(np.uint32) >> 16).astype(np.uint16).view(np.uint8)
    raise ValueError(dtype)


# ---- configuration 1 ---------------------------------------------------------

def config1(n_tasks=1000, numel=1024, seed=0) -> Stream:
    """n_tasks x fp32 ADD on contiguous 1-D tensors, uniform[-1,1], one submit batch."""
    rng = np.random.default_rng(seed)
    tasks, pool_of = new_tasks(n_tasks)
    nb = numel * 4
    a = Pool("a", n_tasks * nb, random_values(rng, n_tasks * numel, "uniform1", F32))
    b = Pool("b", n_tasks * nb, random_values(rng, n_tasks * numel, "uniform1", F32))
    o = Pool("out", n_tasks * nb)
    tasks["op_id"] = OP["ADD"]
    tasks["ndim"] = 1
    tasks["n_inputs"] = 2
    tasks["size"][:, 0] = numel
    offs = np.arange(n_tasks, dtype=np.uint64) * nb
    for k, p in ((0, 0), (1, 1)):
        tasks["inp"]["ptr"][:, k] = offs
        tasks["inp"]["stride"][:, k, 0] = 1
        tasks["inp"]["dtype"][:, k] = F32
        pool_of[:, k] = p
    tasks["out"]["ptr"] = offs
    tasks["out"]["stride"][:, 0] = 1
    tasks["out"]["dtype"] = F32
    pool_of[:, 3] = 2
    return Stream("config1", tasks, pool_of, [a, b, o], batch=0,
                  info=dict(seed=seed, numel=numel))


def sequences(n_seq=1000, length=100, interleave=1, seed=5) -> Stream:
    """The shape of the paper's elementwise micro-benchmark (Section 6.1): n_seq sequences of `length`
    dependent elementwise operations on an fp32 tensor of 1K-16K elements (numel log-uniform per
    sequence).  Step t of a sequence reads what step t-1 wrote (two buffers per sequence, used in
    turn) and names it as its dependency.  Sequences are independent; `interleave` of them are
    issued round-robin (1: one sequence after the other, the order an eager framework produces;
    more: what a caller with several requests in flight produces).  Operations cycle through
    x + c, x * c, relu(x), 0.99 x, x - c with a per-sequence operand c in [-1, 1]: all exactly
    rounded, values stay bounded."""
    rng = np.random.default_rng(seed)
    n = n_seq * length
    tasks, pool_of = new_tasks(n)
    numel = np.round(np.exp(rng.uniform(np.log(1024), np.log(16384), n_seq))).astype(np.int64)
    off = np.concatenate([[0], np.cumsum(numel)])[:-1] * 4                 # byte offset of sequence s in every pool
    total = int(numel.sum())
    x0 = Pool("x0", total * 4, random_values(rng, total, "uniform1", F32))
    c = Pool("c", total * 4, random_values(rng, total, "uniform1", F32))
    bufs = [Pool("ping", total * 4), Pool("pong", total * 4)]
    ops = [("ADD", 2), ("MUL", 2), ("RELU", 1), ("SCALE", 1), ("SUB", 2)]
    i = 0
    for s0 in range(0, n_seq, interleave):
        group = range(s0, min(n_seq, s0 + interleave))
        for t in range(length):
            for sq in group:
                name, nin = ops[t % len(ops)]
                # the previous step of this sequence was issued len(group) tasks ago
                set_head(tasks, i, OP[name], [int(numel[sq])], nin, alpha=0.99 if name == "SCALE" else 0.0,
                         dep=(len(group) if t else 0, 0, 0))
                src = 0 if t == 0 else 2 + (t - 1) % 2                     # pool of the input: x0, then ping / pong in turn
                set_tensor(tasks, pool_of, i, 0, src, int(off[sq]), [1], F32)
                if nin == 2:
                    set_tensor(tasks, pool_of, i, 1, 1, int(off[sq]), [1], F32)
                set_tensor(tasks, pool_of, i, 3, 2 + t % 2, int(off[sq]), [1], F32)
                i += 1
    return Stream("sequences_%d" % interleave, tasks, pool_of, [x0, c] + bufs, batch=64,
                  info=dict(seed=seed, n_seq=n_seq, length=length, interleave=interleave))


# ---- configuration 2 ---------------------------------------------------------

def _draw_shape(rng, numel, rank):
    """A rank-`rank` shape whose product is close to numel (not only powers of two)."""
    if rank == 1:
        return [int(numel)]
    dims = []
    rest = float(numel)
    for r in range(rank - 1):
        hi = max(2.0, rest ** (1.0 / (rank - r)) * 2.0)
        d = int(round(np.exp(rng.uniform(0.0, np.log(hi)))))
        d = max(1, min(d, int(rest)))
        dims.append(d)
        rest = max(1.0, rest / d)
    dims.append(max(1, int(round(rest))))
    rng.shuffle(dims)
    return [int(d) for d in dims]


def config2(n_tasks=10000, seed=1, batch=64, numel_lo=256, numel_hi=65536,
            in_pool_elems=1 << 22) -> Stream:
    """Mixed elementwise stream: op uniform over {ADD, MUL, SUB, RELU, EXP, GELU_TANH, SCALE};
    dtype fp32/fp16/bf16 = 50/25/25 (one per task); numel log-uniform; rank 1-4; 30 % of the
    inputs are non-contiguous views (transposed last two dims, or a stride-2 slice that may
    start at element 1); 20 % of the binary ops broadcast a row or a column vector; N(0,1)."""
    rng = np.random.default_rng(seed)
    tasks, pool_of = new_tasks(n_tasks)
    op_names = ["ADD", "MUL", "SUB", "RELU", "EXP", "GELU_TANH", "SCALE"]
    dts = [F32, F16, BF16]
    in_pools = [Pool("in_" + n, in_pool_elems * ELEM_SIZE[d],
                     random_values(rng, in_pool_elems, "normal1", d))
                for n, d in (("f32", F32), ("f16", F16), ("bf16", BF16))]
    out_off = [0, 0, 0]
    n_noncontig = n_bcast = n_binary = 0
    for i in range(n_tasks):
        name = op_names[int(rng.integers(len(op_names)))]
        impl = IMPL[name]
        ar = ARITY[impl]
        dsel = int(rng.choice(3, p=[0.5, 0.25, 0.25]))
        dt = dts[dsel]
        es = ELEM_SIZE[dt]
        numel = int(round(np.exp(rng.uniform(np.log(numel_lo), np.log(numel_hi)))))
        rank = int(rng.integers(1, 5))
        bcast_kind = None
        if ar == 2:
            n_binary += 1
            if rng.random() < 0.2:
                bcast_kind = "row" if rng.random() < 0.5 else "col"
                rank = max(rank, 2)
                n_bcast += 1
        shape = _draw_shape(rng, numel, rank)
        numel = int(np.prod(shape))
        alpha = float(rng.standard_normal()) if name == "SCALE" else 0.0
        set_head(tasks, i, OP[name], shape, ar, alpha=alpha)
        for k in range(ar):
            if k == 1 and bcast_kind is not None:
                if bcast_kind == "row":       # [1,..,1,C]: every dim but the last is broadcast
                    need = shape[-1]
                    strides = [0] * (rank - 1) + [1]
                    mask = (1 << (rank - 1)) - 1
                else:                         # [1,..,R,1]: a column along dim -2
                    need = shape[-2]
                    strides = [0] * (rank - 2) + [1, 0]
                    mask = ((1 << rank) - 1) & ~(1 << (rank - 2))
                off = int(rng.integers(0, in_pool_elems - need)) // 64 * 64
                set_tensor(tasks, pool_of, i, k, dsel, off * es, strides, dt, mask)
                continue
            kind = "contig"
            if rng.random() < 0.3:
                kind = "transposed" if (rank >= 2 and rng.random() < 0.5) else "slice2"
                n_noncontig += 1
            if kind == "contig":
                strides = contiguous_strides(shape)
                extent = numel
                start = 0
            elif kind == "transposed":        # stored with the last two dims swapped
                stored = shape[:-2] + [shape[-1], shape[-2]]
                st = contiguous_strides(stored)
                strides = st[:-2] + [st[-1], st[-2]]
                extent = numel
                start = 0
            else:                             # every second element of a buffer twice as long
                stored = shape[:-1] + [2 * shape[-1]]
                st = contiguous_strides(stored)
                strides = st[:-1] + [2]
                extent = 2 * numel
                start = int(rng.integers(0, 2))
            off = int(rng.integers(0, in_pool_elems - extent - 1)) // 64 * 64 + start
            set_tensor(tasks, pool_of, i, k, dsel, off * es, strides, dt)
        set_tensor(tasks, pool_of, i, 3, 3 + dsel, out_off[dsel], contiguous_strides(shape), dt)
        out_off[dsel] = _align(out_off[dsel] + numel * es)
    out_pools = [Pool("out_" + n, max(256, out_off[j])) for j, n in enumerate(("f32", "f16", "bf16"))]
    return Stream("config2", tasks, pool_of, in_pools + out_pools, batch=batch,
                  info=dict(seed=seed, noncontig_inputs=n_noncontig, broadcast_ops=n_bcast,
                            binary_ops=n_binary))


# ---- configuration 3 ---------------------------------------------------------

CHAIN_LEN = 6


def config3(n_chains=2000, seed=2, buffer_sets=2, heads=16, Bs=(1, 2, 4, 8), Ss=(64, 128, 256),
            batch=CHAIN_LEN) -> Stream:
    """Attention-softmax chains.  Scores fp16 [B, H, S, S] ~ N(0, sigma=2).  Per chain six tasks,
    each depending on the one before: SCALE by 1/sqrt(64); ADD the causal mask [S, S] (0 on and
    below the diagonal, -inf above) broadcast over B and H; MAX_LAST -> m (fp32); SUB_EXP(t2, m);
    SUM_LAST -> l (fp32); DIV(e, l).  Chains go round-robin over the (B, S) pairs in a seeded
    shuffled order; each pair owns `buffer_sets` sets of buffers that its chains reuse in turn,
    and a chain's first task depends on the last task of the chain that used its set before."""
    rng = np.random.default_rng(seed)
    pairs = [(b, s) for b in Bs for s in Ss]
    order = rng.permutation(len(pairs))
    pools: List[Pool] = []
    layout = {}
    for (b, s) in pairs:
        n = b * heads * s * s
        rows = b * heads * s
        mask = np.zeros((s, s), dtype=np.float16)
        mask[np.triu_indices(s, k=1)] = -np.inf
        pools.append(Pool(f"mask_{b}_{s}", s * s * 2, mask.view(np.uint8).reshape(-1).copy()))
        mask_pool = len(pools) - 1
        sets = []
        for _ in range(buffer_sets):
            pools.append(Pool(f"s_{b}_{s}", n * 2, random_values(rng, n, "normal2", F16)))
            s_pool = len(pools) - 1
            # one work pool per set: t1 | t2 | e | p (fp16, n each) | m | l (fp32, rows each)
            o_t1, o_t2, o_e, o_p = 0, _align(n * 2), 2 * _align(n * 2), 3 * _align(n * 2)
            o_m = 4 * _align(n * 2)
            o_l = o_m + _align(rows * 4)
            pools.append(Pool(f"work_{b}_{s}", o_l + _align(rows * 4)))
            sets.append(dict(s=s_pool, w=len(pools) - 1, t1=o_t1, t2=o_t2, e=o_e, p=o_p, m=o_m, l=o_l))
        layout[(b, s)] = dict(mask=mask_pool, sets=sets, used=0, last_ticket=[None] * buffer_sets)
    n_tasks = n_chains * CHAIN_LEN
    tasks, pool_of = new_tasks(n_tasks)
    chain_pair = np.zeros(n_chains, dtype=np.int32)
    chain_set = np.zeros(n_chains, dtype=np.int32)
    for c in range(n_chains):
        pi = int(order[c % len(pairs)])
        b, s = pairs[pi]
        L = layout[(b, s)]
        k = L["used"] % buffer_sets
        L["used"] += 1
        S = L["sets"][k]
        chain_pair[c], chain_set[c] = pi, k
        shape4 = [b, heads, s, s]
        st4 = contiguous_strides(shape4)
        st3 = contiguous_strides(shape4[:3])
        t0 = c * CHAIN_LEN
        first_dep = 0
        if L["last_ticket"][k] is not None:
            first_dep = t0 - L["last_ticket"][k]
        f16 = lambda i, slot, pool, off: set_tensor(tasks, pool_of, i, slot, pool, off, st4, F16)
        # 1 scale
        set_head(tasks, t0, OP["SCALE"], shape4, 1, alpha=0.125, dep=(first_dep, 0, 0))
        f16(t0, 0, S["s"], 0)
        f16(t0, 3, S["w"], S["t1"])
        # 2 add causal mask (broadcast over dims 0 and 1)
        set_head(tasks, t0 + 1, OP["ADD"], shape4, 2, dep=(1, 0, 0))
        f16(t0 + 1, 0, S["w"], S["t1"])
        set_tensor(tasks, pool_of, t0 + 1, 1, L["mask"], 0, [0, 0, s, 1], F16, 0b0011)
        f16(t0 + 1, 3, S["w"], S["t2"])
        # 3 row max -> m (fp32)
        set_head(tasks, t0 + 2, OP["MAX_LAST"], shape4, 1, dep=(1, 0, 0))
        f16(t0 + 2, 0, S["w"], S["t2"])
        set_tensor(tasks, pool_of, t0 + 2, 3, S["w"], S["m"], st3, F32)
        # 4 exp(t2 - m), m broadcast along the last dim
        set_head(tasks, t0 + 3, OP["SUB_EXP"], shape4, 2, dep=(1, 0, 0))
        f16(t0 + 3, 0, S["w"], S["t2"])
        set_tensor(tasks, pool_of, t0 + 3, 1, S["w"], S["m"], st3 + [0], F32, 0b1000)
        f16(t0 + 3, 3, S["w"], S["e"])
        # 5 row sum -> l (fp32)
        set_head(tasks, t0 + 4, OP["SUM_LAST"], shape4, 1, dep=(1, 0, 0))
        f16(t0 + 4, 0, S["w"], S["e"])
        set_tensor(tasks, pool_of, t0 + 4, 3, S["w"], S["l"], st3, F32)
        # 6 divide
        set_head(tasks, t0 + 5, OP["DIV"], shape4, 2, dep=(1, 0, 0))
        f16(t0 + 5, 0, S["w"], S["e"])
        set_tensor(tasks, pool_of, t0 + 5, 1, S["w"], S["l"], st3 + [0], F32, 0b1000)
        f16(t0 + 5, 3, S["w"], S["p"])
        L["last_ticket"][k] = t0 + 5
    return Stream("config3", tasks, pool_of, pools, batch=batch,
                  info=dict(seed=seed, pairs=pairs, chain_pair=chain_pair, chain_set=chain_set,
                            heads=heads, buffer_sets=buffer_sets,
                            layout={p: layout[p]["sets"] for p in pairs}))


def config3_fused(n_chains=2000, seed=2, buffer_sets=2, heads=16, Bs=(1, 2, 4, 8), Ss=(64, 128, 256),
                  batch=1) -> Stream:
    """The third configuration's softmax with each six-task chain replaced by ONE fused task:
    MASKED_SOFTMAX_LAST(scores, causal mask; alpha = 1/sqrt(64)) -> probabilities.  Same shapes,
    same seeded order over the (B, S) pairs, same score values and the same reuse of
    `buffer_sets` output buffers per pair (a task depends on the task that wrote its buffer
    before)."""
    rng = np.random.default_rng(seed)
    pairs = [(b, s) for b in Bs for s in Ss]
    order = rng.permutation(len(pairs))
    pools: List[Pool] = []
    layout = {}
    for (b, s) in pairs:
        n = b * heads * s * s
        mask = np.zeros((s, s), dtype=np.float16)
        mask[np.triu_indices(s, k=1)] = -np.inf
        pools.append(Pool(f"mask_{b}_{s}", s * s * 2, mask.view(np.uint8).reshape(-1).copy()))
        mask_pool = len(pools) - 1
        sets = []
        for _ in range(buffer_sets):
            pools.append(Pool(f"s_{b}_{s}", n * 2, random_values(rng, n, "normal2", F16)))
            pools.append(Pool(f"p_{b}_{s}", n * 2))
            sets.append(dict(s=len(pools) - 2, p=len(pools) - 1))
        layout[(b, s)] = dict(mask=mask_pool, sets=sets, used=0, last_ticket=[None] * buffer_sets)
    tasks, pool_of = new_tasks(n_chains)
    chain_pair = np.zeros(n_chains, dtype=np.int32)
    chain_set = np.zeros(n_chains, dtype=np.int32)
    for c in range(n_chains):
        pi = int(order[c % len(pairs)])
        b, s = pairs[pi]
        L = layout[(b, s)]
        k = L["used"] % buffer_sets
        L["used"] += 1
        chain_pair[c], chain_set[c] = pi, k
        shape4 = [b, heads, s, s]
        st4 = contiguous_strides(shape4)
        dep = 0 if L["last_ticket"][k] is None else c - L["last_ticket"][k]
        set_head(tasks, c, OP["MASKED_SOFTMAX_LAST"], shape4, 2, alpha=0.125, dep=(dep, 0, 0))
        set_tensor(tasks, pool_of, c, 0, L["sets"][k]["s"], 0, st4, F16)
        set_tensor(tasks, pool_of, c, 1, L["mask"], 0, [0, 0, s, 1], F16, 0b0011)
        set_tensor(tasks, pool_of, c, 3, L["sets"][k]["p"], 0, st4, F16)
        L["last_ticket"][k] = c
    return Stream("config3_fused", tasks, pool_of, pools, batch=batch,
                  info=dict(seed=seed, pairs=pairs, chain_pair=chain_pair, chain_set=chain_set, heads=heads,
                            buffer_sets=buffer_sets, layout={p: layout[p]["sets"] for p in pairs}))


def handoff_chains(n_chains=256, length=4096, numel=1024, n_operands=64, seed=6) -> Stream:
    """Producer -> consumer hand-offs: n_chains independent chains of `length` int32 additions on
    vectors of `numel` elements, issued round-robin.  Link t of a chain reads what link t-1 wrote
    (two buffers per chain, used in turn), adds one of n_operands seeded operand vectors, and names
    link t-1 as its dependency.  Integer arithmetic: the end of a chain is x0 + the sum of its
    operands exactly (wrap-around), so one stale or torn read anywhere in a chain shows at its end."""
    rng = np.random.default_rng(seed)
    n = n_chains * length
    tasks, pool_of = new_tasks(n)
    row = numel * 4
    x0 = rng.integers(-2 ** 31, 2 ** 31 - 1, (n_chains, numel), dtype=np.int64).astype(np.int32)
    ops = rng.integers(-2 ** 31, 2 ** 31 - 1, (n_operands, numel), dtype=np.int64).astype(np.int32)
    i = np.arange(n)
    chain, link = i % n_chains, i // n_chains
    which = (link * 7 + chain * 13) % n_operands
    tasks["op_id"] = OP["ADD"]
    tasks["ndim"] = 1
    tasks["n_inputs"] = 2
    tasks["size"][:, 0] = numel
    # pool 0: buffer A of every chain (starts as x0), pool 1: buffer B, pool 2: the operand table
    src_pool = (link % 2).astype(np.int16)                       # link 0 reads A and writes B, link 1 reads B and writes A, ...
    for slot, (pool, off) in enumerate(((src_pool, chain * row), (np.full(n, 2, np.int16), which * row))):
        tasks["inp"]["ptr"][:, slot] = off
        tasks["inp"]["stride"][:, slot, 0] = 1
        tasks["inp"]["dtype"][:, slot] = I32
        pool_of[:, slot] = pool
    tasks["out"]["ptr"] = chain * row
    tasks["out"]["stride"][:, 0] = 1
    tasks["out"]["dtype"] = I32
    pool_of[:, 3] = 1 - src_pool
    tasks["dep"][:, 0] = np.where(link > 0, n_chains, 0)
    pools = [Pool("a", n_chains * row, x0.view(np.uint8).reshape(-1).copy()), Pool("b", n_chains * row),
             Pool("operands", n_operands * row, ops.view(np.uint8).reshape(-1).copy())]
    return Stream("handoff_chains", tasks, pool_of, pools, batch=64,
                  info=dict(seed=seed, n_chains=n_chains, length=length, numel=numel, which=which.reshape(length, n_chains)))


# ---- configuration 4 ---------------------------------------------------------

def config4(n_tasks=1000000, seed=3, swap_every=10000, window=10000, numel_lo=1024,
            numel_hi=16384, in_pool_elems=1 << 22, batch=64) -> Stream:
    """Hot-swap stream: op uniform over {ADD, MUL, GELU} on fp32, numel log-uniform
    [1024, 16384], uniform[-3, 3].  The logical GELU entry is swapped erf <-> tanh before every
    `swap_every`-th task.  Outputs go into two alternating windows of `window` tasks each, so a
    window can be copied back and checked while the next one is being executed."""
    rng = np.random.default_rng(seed)
    tasks, pool_of = new_tasks(n_tasks)
    opsel = rng.integers(0, 3, n_tasks)
    numel = np.rint(np.exp(rng.uniform(np.log(numel_lo), np.log(numel_hi), n_tasks))).astype(np.int64)
    op_ids = np.array([OP["ADD"], OP["MUL"], OP_GELU], dtype=np.uint16)[opsel]
    arity = np.array([2, 2, 1], dtype=np.uint8)[opsel]
    tasks["op_id"] = op_ids
    tasks["ndim"] = 1
    tasks["n_inputs"] = arity
    tasks["size"][:, 0] = numel
    in_pool = Pool("in_f32", in_pool_elems * 4, random_values(rng, in_pool_elems, "uniform3", F32))
    for k in range(2):
        off = (rng.integers(0, in_pool_elems - numel_hi, n_tasks) // 64 * 64).astype(np.uint64)
        used = arity > k
        tasks["inp"]["ptr"][:, k] = np.where(used, off * 4, 0)
        tasks["inp"]["stride"][:, k, 0] = np.where(used, 1, 0)
        tasks["inp"]["dtype"][:, k] = F32
        pool_of[:, k] = np.where(used, 0, -1)
    # outputs: consecutive 256-byte-aligned regions inside the task's window
    nb = (numel * 4 + 255) // 256 * 256
    widx = np.arange(n_tasks) // window
    out_off = np.zeros(n_tasks, dtype=np.uint64)
    win_bytes = 0
    for w in range(int(widx[-1]) + 1):
        sel = slice(w * window, min(n_tasks, (w + 1) * window))
        c = np.cumsum(nb[sel])
        out_off[sel] = c - nb[sel]
        win_bytes = max(win_bytes, int(c[-1]))
    win_bytes = _align(win_bytes)
    tasks["out"]["ptr"] = out_off + (widx % 2).astype(np.uint64) * np.uint64(win_bytes)
    tasks["out"]["stride"][:, 0] = 1
    tasks["out"]["dtype"] = F32
    pool_of[:, 3] = 1
    out_pool = Pool("out_windows", 2 * win_bytes)
    swaps = []
    cur = IMPL["GELU_ERF"]
    for t in range(swap_every, n_tasks, swap_every):
        cur = IMPL["GELU_TANH"] if cur == IMPL["GELU_ERF"] else IMPL["GELU_ERF"]
        swaps.append((t, OP_GELU, cur))
    return Stream("config4", tasks, pool_of, [in_pool, out_pool], swaps=swaps, batch=batch,
                  info=dict(seed=seed, window=window, window_bytes=win_bytes, swap_every=swap_every))


# ---- configuration 5 ---------------------------------------------------------

def config5(n_tasks=20000, seed=4, rows_range=(64, 4096), cols_range=(256, 16384),
            max_numel=1 << 24, in_pool_bytes=1 << 32, out_slots=64, tile_elems=1 << 25,
            batch=64) -> Stream:
    """Bandwidth stream: {ADD, FMA(a,b,c)} elementwise and {SUM_LAST, MAX_LAST} over the last dim
    of contiguous [rows, cols] tensors, fp32 or bf16, rows and cols log-uniform (redrawn until
    rows*cols <= max_numel), uniform[-1, 1].  Inputs rotate through a pool far larger than the
    256 MB Infinity Cache; outputs rotate through `out_slots` fixed-size slots, and a task
    depends on the previous user of its slot so that the final contents are well defined."""
    rng = np.random.default_rng(seed)
    tasks, pool_of = new_tasks(n_tasks)
    names = ["ADD", "FMA", "SUM_LAST", "MAX_LAST"]
    opsel = rng.integers(0, 4, n_tasks)
    dsel = rng.integers(0, 2, n_tasks)                      # 0 fp32, 1 bf16
    rows = np.zeros(n_tasks, dtype=np.int64)
    cols = np.zeros(n_tasks, dtype=np.int64)
    todo = np.arange(n_tasks)
    while len(todo):
        r = np.rint(np.exp(rng.uniform(np.log(rows_range[0]), np.log(rows_range[1]), len(todo))))
        c = np.rint(np.exp(rng.uniform(np.log(cols_range[0]), np.log(cols_range[1]), len(todo))))
        rows[todo], cols[todo] = r.astype(np.int64), c.astype(np.int64)
        todo = todo[rows[todo] * cols[todo] > max_numel]
    numel = rows * cols
    es = np.where(dsel == 0, 4, 2).astype(np.int64)
    dt = np.where(dsel == 0, F32, BF16).astype(np.uint8)
    impl = np.array([IMPL[n] for n in names])[opsel]
    arity = np.array([2, 3, 1, 1], dtype=np.uint8)[opsel]
    is_red = opsel >= 2
    tasks["op_id"] = np.array([OP[n] for n in names], dtype=np.uint16)[opsel]
    tasks["ndim"] = 2
    tasks["n_inputs"] = arity
    tasks["size"][:, 0] = rows
    tasks["size"][:, 1] = cols
    # input pools (one per dtype), filled by tiling a seeded block
    tile32 = random_values(rng, tile_elems, "uniform1", F32)
    tile16 = random_values(rng, tile_elems, "uniform1", BF16)
    in32 = Pool("in_f32", in_pool_bytes, tile=tile32)
    in16 = Pool("in_bf16", in_pool_bytes // 2, tile=tile16)
    cursor = [0, 0]
    in_off = np.zeros((n_tasks, 3), dtype=np.uint64)
    nbytes = numel * es
    for i in range(n_tasks):
        p = int(dsel[i])
        cap = in_pool_bytes if p == 0 else in_pool_bytes // 2
        for k in range(int(arity[i])):
            nb = _align(int(nbytes[i]))
            if cursor[p] + nb > cap:
                cursor[p] = 0
            in_off[i, k] = cursor[p]
            cursor[p] += nb
    for k in range(3):
        used = arity > k
        tasks["inp"]["ptr"][:, k] = np.where(used, in_off[:, k], 0)
        tasks["inp"]["stride"][:, k, 0] = np.where(used, cols, 0)
        tasks["inp"]["stride"][:, k, 1] = np.where(used, 1, 0)
        tasks["inp"]["dtype"][:, k] = dt
        pool_of[:, k] = np.where(used, dsel, -1)
    slot_bytes = _align(max_numel * 4)
    slot = np.arange(n_tasks) % out_slots
    tasks["out"]["ptr"] = slot.astype(np.uint64) * np.uint64(slot_bytes)
    tasks["out"]["stride"][:, 0] = np.where(is_red, 1, cols)
    tasks["out"]["stride"][:, 1] = np.where(is_red, 0, 1)
    tasks["out"]["dtype"] = dt
    pool_of[:, 3] = 2
    tasks["dep"][:, 0] = np.where(np.arange(n_tasks) >= out_slots, out_slots, 0)
    out_pool = Pool("out_slots", out_slots * slot_bytes)
    return Stream("config5", tasks, pool_of, [in32, in16, out_pool], batch=batch,
                  info=dict(seed=seed, impl=impl, numel=numel, elem_size=es, out_slots=out_slots,
                            slot_bytes=slot_bytes))
