"""Shared test utilities: host execution of a stream through the oracle, ulp distances."""
import numpy as np

from paper_2604_17861_amd import streams as S


def np_dtype(code):
    return {S.F32: np.float32, S.F16: np.float16, S.BF16: np.uint16, S.I32: np.int32}[code]


def bf16_bits_to_f32(bits):
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def ordered_int(bits, width):
    """Map IEEE bit patterns to a monotone integer line (+0 and -0 coincide)."""
    bits = np.asarray(bits).astype(np.int64)
    sign = bits >> (width - 1)
    mag = bits & ((1 << (width - 1)) - 1)
    return np.where(sign == 1, -mag, mag)


def ulp_distance(a_bits, b_bits, dtype_code):
    """Distance in representable numbers of the output dtype; NaN vs NaN = 0, NaN vs number = huge."""
    width = 32 if dtype_code == S.F32 else 16
    a = np.asarray(a_bits)
    b = np.asarray(b_bits)
    if dtype_code == S.F32:
        fa, fb = a.view(np.float32), b.view(np.float32)
        ia, ib = a.view(np.uint32), b.view(np.uint32)
    elif dtype_code == S.F16:
        fa, fb = a.view(np.float16).astype(np.float32), b.view(np.float16).astype(np.float32)
        ia, ib = a.view(np.uint16), b.view(np.uint16)
    else:
        ia, ib = a.view(np.uint16), b.view(np.uint16)
        fa, fb = bf16_bits_to_f32(ia), bf16_bits_to_f32(ib)
    d = np.abs(ordered_int(ia, width) - ordered_int(ib, width))
    nan_a, nan_b = np.isnan(fa), np.isnan(fb)
    d = np.where(nan_a & nan_b, 0, d)
    d = np.where(nan_a ^ nan_b, 1 << 40, d)
    return d


class HostPools:
    """numpy images of a stream's pools, and the task array pointing into them."""

    def __init__(self, stream, images=None):
        self.stream = stream
        self.arrays = [np.array(p.host_image(), dtype=np.uint8, copy=True) for p in stream.pools] \
            if images is None else images
        self.bases = [a.ctypes.data for a in self.arrays]
        self.tasks = stream.materialize(self.bases)

    def view(self, pool, byte_off, count, dtype_code):
        dt = np_dtype(dtype_code)
        return self.arrays[pool][byte_off: byte_off + count * np.dtype(dt).itemsize].view(dt)


def task_out_extent(stream, i):
    """(pool, byte offset, element count spanned, dtype) of task i's output region."""
    t = stream.tasks[i]
    impl = stream.impl_for()[i] if not stream.swaps else None
    nd = int(t["ndim"])
    size = [int(x) for x in t["size"][:nd]]
    is_red = int(t["op_id"]) in (S.OP["SUM_LAST"], S.OP["MAX_LAST"], S.OP["MIN_LAST"])
    ond = nd - 1 if is_red else nd
    st = [int(x) for x in t["out"]["stride"][:ond]]
    span = 1 + sum((size[d] - 1) * st[d] for d in range(ond)) if all(s > 0 for s in size[:ond]) else 0
    return int(stream.pool_of[i, 3]), int(t["out"]["ptr"]), span, int(t["out"]["dtype"])


_NP2CODE = {np.dtype(np.float32): S.F32, np.dtype(np.float16): S.F16, np.dtype(np.uint16): S.BF16,
            np.dtype(np.int32): S.I32}


class Builder:
    """Build a small Stream from numpy views: every tensor is a view (slice, transpose,
    broadcast_to, as_strided) of a base array registered with pool()."""

    def __init__(self, table=None):
        self.bases = []
        self.rows = []
        self.table = dict(S.default_table()) if table is None else dict(table)
        self.programs = {}

    def define_program(self, op_id, code, n_inputs):
        """Bind logical op `op_id` to a program; returns the impl id it will have."""
        impl = S.PROGRAM_BASE + len(self.programs)
        self.programs[impl] = (code, n_inputs)
        self.table[op_id] = impl
        return impl

    def pool(self, arr):
        arr = np.ascontiguousarray(arr)
        self.bases.append(arr)
        return arr

    def _locate(self, v):
        lo = v.ctypes.data if v.size else v.__array_interface__["data"][0]
        for k, b in enumerate(self.bases):
            start = b.ctypes.data
            if start <= lo < start + max(b.nbytes, 1):
                return k, lo - start
        raise ValueError("view does not live in a registered pool")

    def add(self, name, out, ins, shape=None, alpha=0.0, dep=(0, 0, 0), flags=0, op_id=None,
            n_inputs=None):
        impl = S.IMPL[name]
        red = impl in S.REDUCTIONS
        if shape is None:
            shape = list(ins[0].shape) if red else list(out.shape)
        self.rows.append(dict(op=S.OP[name] if op_id is None else op_id, shape=list(shape), ins=list(ins),
                              out=out, alpha=alpha, dep=dep, flags=flags,
                              n_inputs=len(ins) if n_inputs is None else n_inputs))
        return len(self.rows) - 1

    def stream(self, name="tiny", batch=0):
        n = len(self.rows)
        tasks, pool_of = S.new_tasks(n)
        for i, r in enumerate(self.rows):
            S.set_head(tasks, i, r["op"], r["shape"], r["n_inputs"], alpha=r["alpha"], dep=r["dep"],
                       flags=r["flags"])
            nd = len(r["shape"])
            for k, v in enumerate(r["ins"]):
                p, off = self._locate(v)
                es = v.dtype.itemsize
                st = [s // es for s in v.strides]
                st = [0] * (nd - len(st)) + st
                S.set_tensor(tasks, pool_of, i, k, p, off, st, _NP2CODE[v.dtype])
            v = r["out"]
            p, off = self._locate(v)
            es = v.dtype.itemsize
            S.set_tensor(tasks, pool_of, i, 3, p, off, [s // es for s in v.strides], _NP2CODE[v.dtype])
        pools = [S.Pool("p%d" % k, b.nbytes, b.view(np.uint8).reshape(-1)) for k, b in enumerate(self.bases)]
        return S.Stream(name, tasks, pool_of, pools, table=self.table, batch=batch, programs=dict(self.programs))


def run_oracle(stream, mode=0, versions=None, images=None):
    """Execute the whole stream on the CPU oracle; returns (HostPools, status)."""
    import oracle
    hp = HostPools(stream, images)
    st = oracle.run_stream(hp.tasks, stream.impl_for(versions), mode, programs=stream.programs)
    return hp, st
