"""PyTorch integration (paper Section 5.1): a dispatch-level filter that redirects eligible small
operations of ordinary eager PyTorch code into the persistent runtime and leaves everything else
on PyTorch's normal kernel-launch path.

    rt_mode = GpuosMode(max_numel=1 << 16)
    with rt_mode:
        y = torch.relu(a + b) * 0.5          # three tasks in the ring, no kernel launch
        s = torch.softmax(y, -1)             # one fused row task
        z = y @ w                            # not in the library: PyTorch's own kernel
    print(rt_mode.stats)

The filter looks at the four things the paper names:
  operation type     the aten overloads in `GpuosMode.handlers` (elementwise arithmetic with tensors
                     and Python numbers, relu, exp, gelu, neg, abs, sqrt, sigmoid, silu, maximum,
                     minimum, clamp_min / clamp_max, last-dim sum / max / min, last-dim softmax),
                     float16 / bfloat16 / float32 (int32 for add / sub / mul of tensors), ordinary
                     strided tensors of at most 6 dims.  Operators the built-in library lacks are
                     defined on the live context as programs (`PROGRAMS`), the paper's run-time
                     operator injection put to use;
  tensor size        1 <= numel(output) <= max_numel (reductions: the input's numel);
  execution context  an (operation, shape, dtype) signature is redirected from its `min_calls`-th
                     sighting on, so one-off operations stay on the normal path;
  current load       when the ring is nearly full the operation takes the normal path instead of
                     waiting for a slot.

Sharing the GPU.  The worker kernel is resident on every compute unit, so a PyTorch kernel runs
beside it only if its registers and local memory fit into what the worker leaves free; large matrix
kernels do not (measured on MI355X: the 2048^3 GEMMs of all three float types wait for the worker
to leave at 3 workgroups per CU, the fp32 one at 2, none at 1).  The mode therefore (i) creates its
context with one workgroup per compute unit, the paper's default footprint, which the small
operations it redirects do not notice; (ii) stops the worker (gpuos_stop_worker: drain, exit)
before the operations in `yield_ops` (matrix products, convolutions, attention) and starts it
again only once `resume_after` eligible operations have been seen since the last of them, so a program that
alternates small operations with matrix products simply stays on PyTorch's path; (iii) gives the
worker an idle exit (`idle_exit_ms`, default 200): a kernel the list does not know waits at most
that long once, and the next redirected operation starts the worker again.

Everything here is argument marshalling and ordering; every redirected operation is executed by the
HIP worker kernel through the C ABI (Runtime.submit).  Ordering rules that keep eager semantics:
  * results are produced asynchronously into tensors from PyTorch's caching allocator (paper
    Section 4.4); descriptors are staged and submitted `batch` at a time or when something needs them;
  * a redirected operation that reads the result of an earlier one names it as a dependency
    (back-distance in the descriptor), so chains need no host wait;
  * a PyTorch kernel that touches memory a pending task reads or writes is held back until that
    task has completed (host wait on its ticket); view operations only pass the storage along;
  * before the first redirected operation after PyTorch launched work of its own, the current
    stream is synchronised once (its kernels may still be writing the inputs);
  * every tensor a pending task names is kept alive until the task has completed, so the caching
    allocator cannot hand its memory to somebody else;
  * leaving the `with` block (or `synchronize()`) drains everything.
"""
import struct
from collections import deque
from math import prod

import numpy as np
import torch
from torch.utils._python_dispatch import TorchDispatchMode

from . import runtime as R
from . import streams as S

_DT = {torch.float32: S.F32, torch.float16: S.F16, torch.bfloat16: S.BF16, torch.int32: S.I32}
_ITEMSIZE = {torch.float32: 4, torch.float16: 2, torch.bfloat16: 2, torch.int32: 4}
_INT_OK = ("ADD", "SUB", "MUL")
_PLAIN_TENSORS = (torch.Tensor, torch.nn.Parameter)     # no other subclass: those carry semantics of their own
# struct gpuos_task: header, size[6], in[3] + out as {ptr, stride[6], dtype, bcast_mask, pad}, alpha, dep[3], pad
_TASK = struct.Struct("<HBBI6q" + "Q6qBB6x" * 4 + "f3H6x")
assert _TASK.size == S.TASK_DT.itemsize
_NO_TENSOR = (0, 0, 0, 0, 0, 0, 0, 0, 0)
_ZEROS = (0,) * S.MAX_DIMS
_ONES = (1,) * S.MAX_DIMS
_MAX_EXTENT = (1 << 31) - 4096          # elements a tensor view may span (gpuos_submit rejects more)
aten = torch.ops.aten


class _Plan:
    __slots__ = ("impl", "inputs", "size", "out_shape", "out_dtype", "alpha", "flags", "reduce")

    def __init__(self, impl, inputs, size, out_shape, out_dtype, alpha=0.0, flags=0, reduce=False):
        self.impl, self.inputs, self.size, self.out_shape = impl, inputs, size, out_shape
        self.out_dtype, self.alpha, self.flags, self.reduce = out_dtype, alpha, flags, reduce


class GpuosMode(TorchDispatchMode):
    """Redirects eligible operations to a GPUOS context while active (see the module docstring).

    rt:         a Runtime to use (not shut down by this object), or None to create one on `device`
    max_numel:  size filter
    min_calls:  context filter (1 = redirect at first sight)
    batch:      descriptors staged before one submit
    yield_ops:  aten overloads the whole GPU is handed to (None: YIELD_OPS)
    resume_after: eligible operations seen after such a hand-over before the worker is started again
    runtime_kw: gpuos_config fields for the context this object creates (defaults: one workgroup
                per compute unit, idle exit after 200 ms)"""

    def __init__(self, rt=None, device=None, max_numel=1 << 16, min_calls=1, batch=32, yield_ops=None, resume_after=64,
                 **runtime_kw):
        super().__init__()
        self.device = torch.device(device if device is not None else "cuda:0")
        if self.device.type == "cuda" and self.device.index is None:
            self.device = torch.device("cuda", 0)          # tensors report their device with its index
        self._own = rt is None
        if rt is None:
            runtime_kw.setdefault("workgroups_per_cu", 1)
            runtime_kw.setdefault("idle_exit_ms", 200)
            rt = R.Runtime(0, device=self.device.index or 0, **runtime_kw)
        self.rt = rt
        self.yield_ops = YIELD_OPS if yield_ops is None else set(yield_ops)
        self.resume_after = int(resume_after)
        self._paused, self._since_pause = False, 0
        self.capacity = int(self.rt.peek_queue().capacity)
        for name, impl in S.IMPL.items():                       # logical id = impl id + 32, as in streams.OP
            if name not in ("NONE",):
                self.rt.register_op(S.OP[name], impl)
        # operators the built-in library lacks are added the way the paper adds operators at run time:
        # as programs defined on the live context and bound to logical ids of their own
        self.op_id = {name: S.OP[name] for name in S.IMPL if name != "NONE"}
        # (all defined before the first is bound: the native worker kernel is compiled at the first
        # binding, for every program defined by then -- one compilation instead of one per program)
        impls = [(name, self.rt.define_program(code, n_in)) for name, (code, n_in) in sorted(PROGRAMS.items())]
        for k, (name, impl) in enumerate(impls):
            self.rt.register_op(_PROGRAM_OP_BASE + k, impl)
            self.op_id[name] = _PROGRAM_OP_BASE + k
        self.max_numel, self.min_calls, self.batch = int(max_numel), int(min_calls), max(1, int(batch))
        self._buf = bytearray(self.batch * _TASK.size)
        self._tasks = np.frombuffer(self._buf, dtype=S.TASK_DT)
        self._staged = 0                 # descriptors in _buf not yet submitted
        self._next = None                # ticket the next submitted descriptor gets (None: not known yet)
        self._floor = 0                  # completed-in-order floor as last read
        self._touch = {}                 # storage address -> newest pending ticket that reads or writes it
        self._writer = {}                # storage address -> newest pending ticket that writes it
        self._inflight = deque()         # (ticket, tensors kept alive, storage addresses)
        self._seen = {}                  # context filter: signature -> sightings
        self._dirty = True               # PyTorch may have work in flight on its stream
        self.stats = dict(redirected=0, fallback_type=0, fallback_size=0, fallback_context=0, fallback_load=0,
                          fallback_paused=0, views=0, stream_syncs=0, host_waits=0, submits=0, pauses=0, resumes=0,
                          restarts=0, by_op={})
        u, b, r, sc = self._unary, self._binary, self._reduce, self._scalar
        self.handlers = {
            aten.add.Tensor: b("ADD", "ADD_SCALAR"), aten.sub.Tensor: b("SUB", "SUB_SCALAR"), aten.mul.Tensor: b("MUL", "SCALE"),
            aten.div.Tensor: b("DIV"), aten.maximum.default: b("MAXIMUM"), aten.minimum.default: b("MINIMUM"),
            aten.rsub.Scalar: sc("RSUB_SCALAR"), aten.clamp_min.default: sc("CLAMP_MIN"), aten.clamp_max.default: sc("CLAMP_MAX"),
            aten.relu.default: u("RELU"), aten.exp.default: u("EXP"), aten.gelu.default: self._gelu,
            aten.neg.default: u("NEG"), aten.abs.default: u("ABS"), aten.sqrt.default: u("SQRT"),
            aten.sigmoid.default: u("SIGMOID"), aten.silu.default: u("SILU"),
            aten.sum.dim_IntList: r("SUM_LAST"), aten.amax.default: r("MAX_LAST"), aten.amin.default: r("MIN_LAST"),
            aten._softmax.default: self._softmax,
        }

    # ---- eligibility: operation type ------------------------------------------------------------
    def _tensor_ok(self, t):
        if (type(t) not in _PLAIN_TENSORS or t.dtype not in _DT or t.device != self.device or t.layout is not torch.strided
                or t.is_conj() or t.is_neg()):
            return False
        nd = t.dim()
        if nd == 0:
            return True
        if nd > S.MAX_DIMS:
            return False
        n = t.numel()
        if n < _MAX_EXTENT and t.is_contiguous():
            return True
        # the ring record holds 32-bit element offsets: a quick bound, then the extent of the view itself
        return (max(t.stride()) * n < _MAX_EXTENT
                or sum((k - 1) * st for k, st in zip(t.shape, t.stride())) < _MAX_EXTENT)

    def _unary(self, name):
        def plan(args, kwargs):
            if len(args) != 1 or kwargs or not self._tensor_ok(args[0]) or args[0].dtype is torch.int32:
                return None
            x = args[0]
            shape = tuple(x.shape)
            return _Plan(name, (x,), shape, shape, x.dtype)
        return plan

    def _gelu(self, args, kwargs):
        approx = kwargs.get("approximate", args[1] if len(args) > 1 else "none")
        if not args or not self._tensor_ok(args[0]) or args[0].dtype is torch.int32 or approx not in ("none", "tanh"):
            return None
        x = args[0]
        shape = tuple(x.shape)
        return _Plan("GELU_TANH" if approx == "tanh" else "GELU_ERF", (x,), shape, shape, x.dtype)

    def _scalar(self, name):
        """tensor (op) python number: the number travels in the descriptor's alpha."""
        def plan(args, kwargs):
            if len(args) != 2 or kwargs or not self._tensor_ok(args[0]) or args[0].dtype is torch.int32:
                return None
            x, c = args
            if isinstance(c, (bool, complex)) or not isinstance(c, (int, float)):
                return None
            shape = tuple(x.shape)
            return _Plan(name, (x,), shape, shape, x.dtype, alpha=float(c))
        return plan

    def _binary(self, name, with_number=None):
        def plan(args, kwargs):
            if len(args) != 2 or not isinstance(args[0], torch.Tensor):
                return None
            a, o = args
            if kwargs and (kwargs.get("alpha", 1) != 1 or kwargs.get("rounding_mode") is not None or any(
                    k not in ("alpha", "rounding_mode") for k in kwargs)):
                return None
            if not self._tensor_ok(a):
                return None
            if not isinstance(o, torch.Tensor):
                # tensor (op) python number: scale, or the one-instruction programs; a division stays with
                # PyTorch (it multiplies by the reciprocal, which rounds differently)
                if with_number is None or isinstance(o, (bool, complex)) or not isinstance(o, (int, float)) or a.dtype is torch.int32:
                    return None
                shape = tuple(a.shape)
                return _Plan(with_number, (a,), shape, shape, a.dtype, alpha=float(o))
            if not self._tensor_ok(o):
                return None
            dt = a.dtype
            if dt is not o.dtype:
                dt = torch.result_type(a, o)
                if dt not in _DT or (dt is torch.int32) != (a.dtype is torch.int32) or (a.dtype is torch.int32) != (o.dtype is torch.int32):
                    return None
                # PyTorch converts an operand to the result dtype before computing; the kernel computes on
                # the operand as stored.  The two agree when that conversion is exact (same dtype, or a
                # 16-bit operand under a float32 result); a float32 0-dim operand under a 16-bit result is not.
                if dt is not torch.float32:
                    return None
            if dt is torch.int32 and name not in _INT_OK:         # (the programs are float operators)
                return None
            shape = tuple(a.shape)
            if shape != tuple(o.shape):
                try:
                    shape = tuple(torch.broadcast_shapes(a.shape, o.shape))
                except RuntimeError:
                    return None
            return _Plan(name, (a, o), shape, shape, dt)
        return plan

    def _reduce(self, name):
        def plan(args, kwargs):
            if not args or not self._tensor_ok(args[0]):
                return None
            x = args[0]
            dim = args[1] if len(args) > 1 else kwargs.get("dim")
            keep = args[2] if len(args) > 2 else kwargs.get("keepdim", False)
            want = kwargs.get("dtype", args[3] if len(args) > 3 else None)
            if x.dim() < 1 or dim is None or len(dim) != 1 or dim[0] % x.dim() != x.dim() - 1 or x.shape[-1] < 1:
                return None
            if want not in (None, x.dtype) or (x.dtype is torch.int32 and name == "SUM_LAST"):
                return None                              # torch sums int32 into int64
            outer = tuple(x.shape[:-1])
            return _Plan(name, (x,), tuple(x.shape), outer + ((1,) if keep else ()), x.dtype,
                         flags=S.FLAG_KEEPDIM if keep else 0, reduce=True)
        return plan

    def _softmax(self, args, kwargs):
        if len(args) != 3 or kwargs or not self._tensor_ok(args[0]):
            return None
        x, dim, half_to_float = args
        if x.dim() < 1 or dim % x.dim() != x.dim() - 1 or half_to_float or x.dtype is torch.int32:
            return None
        shape = tuple(x.shape)
        return _Plan("SOFTMAX_LAST", (x,), shape, shape, x.dtype)

    # ---- the dispatch hook ------------------------------------------------------------------------
    def __torch_dispatch__(self, func, types, args=(), kwargs=None):
        kwargs = kwargs or {}
        h = self.handlers.get(func)
        if h is not None:
            plan = h(args, kwargs)
            if plan is None:
                self.stats["fallback_type"] += 1
            else:
                out = self._redirect(func, plan)
                if out is not None:
                    return out
        elif getattr(func, "is_view", False):
            self.stats["views"] += 1
            return func(*args, **kwargs)               # no kernel, no data touched: the storage carries the ordering
        else:
            self.stats["fallback_type"] += 1
            if func in self.yield_ops:
                if self._paused:
                    self._since_pause = 0                # the count is of eligible operations in a row
                else:
                    self._pause()
        return self._normal_path(func, args, kwargs)

    def _redirect(self, func, p):
        n = prod(p.size)
        if n < 1 or n > self.max_numel or len(p.size) > S.MAX_DIMS:       # tensor size
            self.stats["fallback_size"] += 1
            return None
        if self.min_calls > 1:                                            # execution context
            sig = (p.impl, p.size, p.out_dtype)
            c = self._seen.get(sig, 0) + 1
            self._seen[sig] = c
            if c < self.min_calls:
                self.stats["fallback_context"] += 1
                return None
        if self._paused:                                                  # the GPU was handed to PyTorch's big kernels
            self._since_pause += 1
            if self._since_pause < self.resume_after:
                self.stats["fallback_paused"] += 1
                return None
            self.rt.start_worker()
            self._paused = False
            self.stats["resumes"] += 1
        if not self._room():                                              # current load
            self.stats["fallback_load"] += 1
            return None
        if self._dirty and self.device.type == "cuda":
            torch.cuda.current_stream(self.device).synchronize()
            self.stats["stream_syncs"] += 1
        self._dirty = False
        out = torch.empty(p.out_shape, dtype=p.out_dtype, device=self.device)
        self._stage(p, out)
        self.stats["redirected"] += 1
        self.stats["by_op"][p.impl] = self.stats["by_op"].get(p.impl, 0) + 1
        return out

    def _room(self):
        if self._next is None:
            return True
        margin = self.capacity - self.batch - 1
        if self._next + self._staged - self._floor < margin:
            return True
        self._floor = int(self.rt.peek_queue().completed)
        self._retire()
        return self._next + self._staged - self._floor < margin

    # ---- descriptor marshalling -----------------------------------------------------------------
    @staticmethod
    def _operand(t, ptr, size, nd):
        """{ptr, stride[6], dtype, bcast_mask} of `t` broadcast to the iteration shape `size`
        (dims aligned at the right, as PyTorch broadcasts)."""
        shape, stride = t.shape, t.stride()
        if shape == size:                                   # nothing to broadcast
            return (ptr, *stride, *_ZEROS[nd:], _DT[t.dtype], 0)
        td = len(shape)
        st = [0] * S.MAX_DIMS
        mask = 0
        for d in range(nd):
            k = d - (nd - td)
            if k >= 0 and shape[k] != 1:
                st[d] = stride[k]
            elif size[d] != 1:
                mask |= 1 << d
        return (ptr, *st, _DT[t.dtype], mask)

    def _stage(self, p, out):
        size = p.size if p.size else (1,)                  # a 0-dim tensor iterates as [1]
        nd = len(size)
        if p.reduce and nd == 1:
            size, nd = (1,) + size, 2                      # a vector reduces as one row
        me = (self._next if self._next is not None else 0) + self._staged
        writer, touch, cap = self._writer, self._touch, self.capacity
        deps, ops, keys = [], [], []
        for t in p.inputs:
            ptr = t.data_ptr()
            k = ptr - t.storage_offset() * _ITEMSIZE[t.dtype]                # the storage's address
            w = writer.get(k)
            if w is not None:
                d = me - w
                if 0 < d < cap and d not in deps:           # further back: the ring wrapped past it, it has completed
                    deps.append(d)
            touch[k] = me
            keys.append(k)
            ops.append(self._operand(t, ptr, size, nd))
        ko = out.data_ptr()                                 # freshly allocated: offset 0
        if p.reduce:
            # the output walks the outer dims (size[:-1]); it is freshly allocated and contiguous
            ost = [0] * S.MAX_DIMS
            acc = 1
            for d in range(nd - 2, -1, -1):
                ost[d] = acc
                acc *= size[d]
            o = (ko, *ost, _DT[out.dtype], 0)
        else:
            o = self._operand(out, ko, size, nd)
        while len(ops) < 3:
            ops.append(_NO_TENSOR)
        while len(deps) < 3:
            deps.append(0)
        _TASK.pack_into(self._buf, self._staged * _TASK.size, self.op_id[p.impl], nd, len(p.inputs), p.flags,
                        *size, *_ONES[nd:], *ops[0], *ops[1], *ops[2], *o, p.alpha, *deps)
        touch[ko] = me
        writer[ko] = me
        keys.append(ko)
        self._inflight.append((me, (out, p.inputs), keys, ko))
        self._staged += 1
        if self._staged == self.batch:
            self._submit()

    def _pause(self):
        """Hand the whole GPU to PyTorch: drain, stop the worker."""
        self.synchronize()
        self.rt.stop_worker()
        self._paused, self._since_pause = True, 0
        self.stats["pauses"] += 1

    def _submit(self):
        if not self._staged:
            return
        try:
            first = self.rt.submit(self._tasks, 0, self._staged)
        except R.GpuosError as e:
            if e.status != R.E_DEAD:
                raise
            self.rt.start_worker()                      # it left by itself (idle exit): nothing was lost
            self.stats["restarts"] += 1
            first = self.rt.submit(self._tasks, 0, self._staged)
        if self._next is None:
            # the context may have been used before this object got it: rebase what was staged from 0
            if first:
                self._inflight = deque((t + first, r, k, ko) for t, r, k, ko in self._inflight)
                self._touch = {k: t + first for k, t in self._touch.items()}
                self._writer = {k: t + first for k, t in self._writer.items()}
            self._next = first
        elif first != self._next:
            raise RuntimeError("another producer submitted to this context: tickets %d, expected %d" % (first, self._next))
        self._next += self._staged
        self._staged = 0
        self.stats["submits"] += 1

    def _retire(self):
        """Drop the references of tasks below the completed floor."""
        q = self._inflight
        while q and q[0][0] < self._floor:
            t, _, keys, ko = q.popleft()
            for k in keys:
                if self._touch.get(k) == t:
                    del self._touch[k]
            if self._writer.get(ko) == t:
                del self._writer[ko]

    # ---- PyTorch's own path -------------------------------------------------------------------
    def _normal_path(self, func, args, kwargs):
        if self._touch:
            newest = -1
            for t in _tensors(args, kwargs):
                if t.device == self.device:
                    k = self._touch.get(t.data_ptr() - t.storage_offset() * t.element_size())
                    if k is not None and k > newest:
                        newest = k
            if newest >= 0:
                self._wait(newest)
        out = func(*args, **kwargs)
        self._dirty = True
        return out

    def _wait(self, ticket):
        """Until `ticket` and every ticket before it have completed (tasks complete in any order, and
        an older task may read the same memory)."""
        self._submit()
        while ticket >= self._floor:
            self._wait_one(ticket)
            self.stats["host_waits"] += 1
            self._floor = max(self._floor, int(self.rt.peek_queue().completed))
            if ticket >= self._floor:
                self._wait_one(self._floor)            # the oldest one still running
                self._floor = max(self._floor, int(self.rt.peek_queue().completed))
        self._retire()

    def _wait_one(self, ticket):
        try:
            self.rt.wait(ticket)
        except R.GpuosError as e:
            if e.status != R.E_DEAD:
                raise
            # the worker's idle exit raced with the submit: the records are in the ring, the next run takes them
            self.rt.start_worker()
            self.stats["restarts"] += 1
            self.rt.wait(ticket)

    def synchronize(self):
        """Submit what is staged and wait until every redirected operation has completed."""
        self._submit()
        if self._inflight:
            self._wait(self._inflight[-1][0])
        self._floor = int(self.rt.peek_queue().completed)
        self._retire()

    def __exit__(self, *exc):
        try:
            self.synchronize()
        finally:
            r = super().__exit__(*exc)
        return r

    def close(self):
        self.synchronize()
        if self._own and self.rt is not None:
            self.rt.shutdown()
        self.rt = None


P_ = S.program
_PROGRAM_OP_BASE = 160
# name -> (instructions, inputs).  r0..r2 are the inputs, r3 the descriptor's alpha, r4..r7 start at zero.
PROGRAMS = {
    "ADD_SCALAR": (P_(("ADD", 0, 0, 3)), 1), "SUB_SCALAR": (P_(("SUB", 0, 0, 3)), 1), "RSUB_SCALAR": (P_(("SUB", 0, 3, 0)), 1),
    "CLAMP_MIN": (P_(("MAX", 0, 0, 3)), 1), "CLAMP_MAX": (P_(("MIN", 0, 0, 3)), 1),
    "NEG": (P_(("NEG", 0, 0)), 1), "ABS": (P_(("ABS", 0, 0)), 1), "SQRT": (P_(("SQRT", 0, 0)), 1),
    "MAXIMUM": (P_(("MAX", 0, 0, 1)), 2), "MINIMUM": (P_(("MIN", 0, 0, 1)), 2),
    "SIGMOID": (P_(("NEG", 4, 0), ("EXP", 4, 4), ("IMM", 5, 1.0), ("ADD", 4, 4, 5), ("DIV", 0, 5, 4)), 1),
    "SILU": (P_(("NEG", 4, 0), ("EXP", 4, 4), ("IMM", 5, 1.0), ("ADD", 4, 4, 5), ("DIV", 0, 0, 4)), 1),
}


def _overloads(*names):
    out = set()
    for n in names:
        packet, _, overload = n.partition(".")
        op = getattr(aten, packet, None)
        if op is not None and hasattr(op, overload or "default"):
            out.add(getattr(op, overload or "default"))
    return out


# operations whose kernels do not fit beside the resident worker (large register / local-memory footprints)
YIELD_OPS = _overloads("mm", "addmm", "bmm", "baddbmm", "_scaled_mm", "convolution", "cudnn_convolution", "miopen_convolution",
                       "_scaled_dot_product_flash_attention", "_scaled_dot_product_efficient_attention",
                       "_scaled_dot_product_attention_math", "_flash_attention_forward", "_efficient_attention_forward",
                       "linalg_solve_ex", "_linalg_svd", "linalg_cholesky_ex", "linalg_inv_ex")


def _tensors(args, kwargs):
    for a in list(args) + list(kwargs.values()):
        if isinstance(a, torch.Tensor):
            yield a
        elif isinstance(a, (list, tuple)):
            for b in a:
                if isinstance(b, torch.Tensor):
                    yield b
