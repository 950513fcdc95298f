"""Structural oracle: trace recording, canonical numbering, serialisation,
hash, special-scalar folding and region partitioning, in plain Python.

TEST INFRASTRUCTURE -- see oracle/__init__.py.  This is a second, independent
implementation of the written IR specification that the C++ library follows;
the two share no code, only the specification text.  The library's graph
hash, cache hit sequence and region list must equal this module's bit for bit.

What the paper fixes and where:
* a tensor is a handle to either materialised data or a pending IR node;
  ops append nodes instead of running (section 3);
* the barrier evaluates the pending computation of all live tensors, and
  liveness is tracked by unique tensor ids (section 4, the barrier and
  DeviceContextArena paragraphs);
* IR nodes carry op, dtype, shape, attributes; inputs are device_data leaves;
  scalars are rank 0 (section 4.1 and figure 1);
* only the scalars 0 and 1 are part of the graph's identity, all other
  scalars are dynamic parameters (section 4.1, the special-scalar heuristic);
* loops unroll, shared nodes are emitted once (section 4.2 and figure 2);
* in-place update = rebinding the destination to the right-hand side's
  computation; the old buffer may be donated at the step barrier when nothing
  else can observe it (section 4.3).
The numbering order is not stated in the text; figures 1, 2 and 3 are all
reproduced by a post-order walk from each root that visits operands from last
to first and emits each node once, which is what ``canonical_order`` does.
Everything else (byte layout, hash function, fusion rules) is this build's
own convention and is pinned by two implementations agreeing.
"""
from __future__ import annotations

import math
import struct
import weakref

# ---- dtypes -----------------------------------------------------------------
F32, BF16, S32, S64 = 0, 1, 2, 3
DTYPE_NAME = {F32: "f32", BF16: "bf16", S32: "s32", S64: "s64"}
DTYPE_ID = {v: k for k, v in DTYPE_NAME.items()}
_IS_FLOAT = {F32: True, BF16: True, S32: False, S64: False}

# ---- opcodes ----------------------------------------------------------------
DEVICE_DATA, SCALAR_PARAM, CONSTANT = 1, 2, 3
NEG, ABS, EXP, LOG, TANH, SQRT, RSQRT, RECIP, RELU, GELU, SQUARE, CAST, SIGMOID = range(16, 29)
ADD, SUB, MUL, DIV, MAXIMUM, MINIMUM, RELU_GRAD, GELU_GRAD = range(32, 40)
EXPAND, RESHAPE, PERMUTE, NARROW, SLICE_UPDATE = 48, 49, 50, 51, 52
SUM, AMAX, MEAN = 64, 65, 66
SOFTMAX, SOFTMAX_GRAD, LAYER_NORM, LAYER_NORM_GRAD, XENT, XENT_GRAD = range(80, 86)
MATMUL = 96

OP_NAME = {
    DEVICE_DATA: "xla::device_data", SCALAR_PARAM: "xla::device_data", CONSTANT: "prim::Constant",
    NEG: "aten::neg", ABS: "aten::abs", EXP: "aten::exp", LOG: "aten::log", TANH: "aten::tanh",
    SQRT: "aten::sqrt", RSQRT: "aten::rsqrt", RECIP: "aten::reciprocal", RELU: "aten::relu",
    GELU: "aten::gelu", SQUARE: "aten::square", CAST: "aten::to", SIGMOID: "aten::sigmoid",
    ADD: "aten::add", SUB: "aten::sub", MUL: "aten::mul", DIV: "aten::div",
    MAXIMUM: "aten::maximum", MINIMUM: "aten::minimum", RELU_GRAD: "aten::threshold_backward",
    GELU_GRAD: "aten::gelu_backward", EXPAND: "aten::expand", RESHAPE: "aten::view",
    PERMUTE: "aten::permute", NARROW: "aten::narrow", SLICE_UPDATE: "aten::slice_scatter", SUM: "aten::sum", AMAX: "aten::amax", MEAN: "aten::mean",
    SOFTMAX: "aten::_softmax", SOFTMAX_GRAD: "aten::_softmax_backward_data",
    LAYER_NORM: "aten::native_layer_norm", LAYER_NORM_GRAD: "aten::native_layer_norm_backward",
    XENT: "aten::nll_loss_of_log_softmax", XENT_GRAD: "aten::nll_loss_of_log_softmax_backward",
    MATMUL: "aten::matmul",
}

# ---- attribute keys -----------------------------------------------------------
A_VALUE, A_DTYPE, A_AXIS, A_EPS, A_TRANS_A, A_TRANS_B, A_START, A_LENGTH, A_DIM0 = 1, 2, 3, 4, 5, 6, 7, 8, 16

UNARY = {NEG, ABS, EXP, LOG, TANH, SQRT, RSQRT, RECIP, RELU, GELU, SQUARE, CAST, SIGMOID}
BINARY = {ADD, SUB, MUL, DIV, MAXIMUM, MINIMUM, RELU_GRAD, GELU_GRAD}
PLAIN_REDUCE = {SUM, AMAX, MEAN}
ROW_OPS = {SOFTMAX, SOFTMAX_GRAD, LAYER_NORM, LAYER_NORM_GRAD, XENT, XENT_GRAD}

# caps on one fused region
MAX_INPUTS, MAX_OUTPUTS, MAX_SLOTS, MAX_FINALISER_ELEMS = 8, 8, 32, 65536


def fnv1a64(data: bytes) -> int:
    """FNV-1a, 64 bit (public-domain hash by Fowler, Noll and Vo)."""
    h = 0xCBF29CE484222325
    for byte in data:
        h ^= byte
        h = (h * 0x100000001B3) & 0xFFFFFFFFFFFFFFFF
    return h


def broadcast_shapes(a, b):
    ra, rb = len(a), len(b)
    out = []
    for i in range(max(ra, rb)):
        da = a[ra - 1 - i] if i < ra else 1
        db = b[rb - 1 - i] if i < rb else 1
        if da != db and da != 1 and db != 1:
            raise ValueError(f"shapes {a} and {b} do not broadcast")
        out.append(max(da, db) if da != 0 and db != 0 else 0)
    return tuple(reversed(out))


def numel(shape):
    n = 1
    for d in shape:
        n *= d
    return n


class Node:
    __slots__ = ("op", "dtype", "shape", "attrs", "ins", "buffer", "value")

    def __init__(self, op, dtype, shape, attrs=(), ins=(), buffer=None, value=None):
        self.op = op
        self.dtype = dtype
        self.shape = tuple(int(d) for d in shape)
        self.attrs = tuple(sorted(attrs, key=lambda kv: kv[0]))  # (key, is_float, payload)
        self.ins = tuple(ins)          # ((node_index, slot), ...)
        self.buffer = buffer           # DEVICE_DATA: Buffer
        self.value = value             # SCALAR_PARAM: the dynamic value (not hashed)


class Buffer:
    """A materialised device buffer, as far as structure is concerned."""
    __slots__ = ("dtype", "shape", "donatable", "data_refs")

    def __init__(self, dtype, shape, donatable):
        self.dtype, self.shape, self.donatable = dtype, tuple(shape), donatable
        self.data_refs = 0             # live handles currently bound to it


class STensor:
    """A tensor handle: unique id + binding (pending node | data | scalar)."""
    __slots__ = ("tid", "kind", "node", "slot", "buffer", "value", "dtype", "shape",
                 "donor", "memo_epoch", "memo_node", "alive", "version", "view", "seen", "__weakref__")

    def __del__(self):
        # dropping the last reference to a handle is UnregisterTensor
        if self.alive and self.kind == "data":
            self.buffer.data_refs -= 1

    def __init__(self, tid):
        self.tid = tid
        self.kind = None               # "pending" | "data" | "scalar"
        self.node = self.slot = None
        self.buffer = None
        self.value = None
        self.dtype = None
        self.shape = None
        self.donor = None
        self.memo_epoch = -1
        self.memo_node = None
        self.alive = True
        self.version = 0               # bumped whenever the handle's value is replaced
        self.view = None               # (base handle, view op, arguments) for a view (section 4.4)
        self.seen = 0                  # version of the base that the current value was derived from


class Tracer:
    """Records a trace exactly like the library's front end and reproduces the
    barrier's structural results (order, bytes, hash, cache verdict, plan)."""

    def __init__(self, device_name: str = "CPU:0"):
        self.device_name = device_name
        self.nodes: list[Node] = []
        self.handles = weakref.WeakValueDictionary()   # live handles only
        self.next_tid = 1
        self.epoch = 0
        self.cache: dict[tuple[int, int], bytes] = {}
        self.last = None               # results of the last barrier

    # ---- handles ----------------------------------------------------------
    def _new_handle(self) -> STensor:
        t = STensor(self.next_tid)
        self.next_tid += 1
        self.handles[t.tid] = t
        return t

    def _bind_data(self, t: STensor, buf: Buffer):
        t.kind, t.buffer, t.dtype, t.shape = "data", buf, buf.dtype, buf.shape
        t.node = t.slot = None
        buf.data_refs += 1

    def _unbind(self, t: STensor):
        if t.kind == "data":
            t.buffer.data_refs -= 1
        t.kind = None

    def tensor(self, array_or_shape, dtype="f32", donatable=False) -> STensor:
        """Factory from existing device data.  Accepts an array (its shape is
        used) or a bare shape tuple."""
        shape = tuple(array_or_shape.shape) if hasattr(array_or_shape, "shape") else tuple(array_or_shape)
        if hasattr(array_or_shape, "dtype") and dtype == "f32":
            kind = array_or_shape.dtype.kind
            if kind == "i":
                dtype = "s32" if array_or_shape.dtype.itemsize == 4 else "s64"
        t = self._new_handle()
        self._bind_data(t, Buffer(DTYPE_ID[dtype], shape, donatable))
        return t

    def scalar(self, value, dtype="f32") -> STensor:
        t = self._new_handle()
        t.kind, t.value, t.dtype, t.shape = "scalar", value, DTYPE_ID[dtype], ()
        return t

    def release(self, t: STensor):
        if t.alive:
            self._unbind(t)
            t.alive = False
            t.donor = None
            del self.handles[t.tid]

    def _t(self, x) -> STensor:
        return x if isinstance(x, STensor) else self.scalar(x)

    # ---- views (section 4.4) -------------------------------------------------
    def _view_op(self, base, kind, args):
        if kind == PERMUTE:
            return self.permute(base, args)
        if kind == RESHAPE:
            return self.reshape(base, args)
        return self.narrow(base, *args)

    def _make_view(self, base, kind, args):
        t = self._view_op(base, kind, args)
        t.view, t.seen = (base, kind, args), base.version
        return t

    def view_permute(self, x, dims): return self._make_view(x, PERMUTE, tuple(int(d) for d in dims))
    def view_reshape(self, x, size): return self._make_view(x, RESHAPE, tuple(int(d) for d in size))
    def view_narrow(self, x, axis, start, length): return self._make_view(x, NARROW, (int(axis), int(start), int(length)))

    def _refresh(self, t: STensor):
        """Forward sequence: a view is its view op applied to the base's current value."""
        if t.view is None:
            return
        base, kind, args = t.view
        self._refresh(base)
        if t.seen == base.version:
            return
        fresh = self._view_op(base, kind, args)
        self._unbind(t)
        t.kind, t.node, t.slot, t.donor, t.memo_epoch = "pending", fresh.node, 0, None, -1
        t.version += 1
        t.seen = base.version
        self.release(fresh)

    def _refresh_views(self):
        for _, t in sorted(self.handles.items()):
            if t.alive and t.view is not None:
                self._refresh(t)

    def _use(self, t: STensor):
        """Operand reference (node, slot) for a handle in the current trace."""
        assert t.alive
        self._refresh(t)
        if t.kind == "pending":
            return (t.node, t.slot)
        if t.memo_epoch != self.epoch or t.memo_node is None:
            if t.kind == "data":
                n = Node(DEVICE_DATA, t.dtype, t.shape, buffer=t.buffer)
            else:
                v = t.value
                special = v == 1 or (v == 0 and math.copysign(1.0, float(v)) > 0)
                if special:
                    isf = _IS_FLOAT[t.dtype]
                    n = Node(CONSTANT, t.dtype, (), attrs=[(A_VALUE, isf, float(v) if isf else int(v))])
                else:
                    n = Node(SCALAR_PARAM, t.dtype, (), value=v)
            self.nodes.append(n)
            t.memo_epoch, t.memo_node = self.epoch, len(self.nodes) - 1
        return (t.memo_node, 0)

    def _emit(self, op, dtype, shape, attrs, operands, n_out=1):
        ins = [self._use(self._t(o)) for o in operands]
        self.nodes.append(Node(op, dtype, shape, attrs, ins))
        idx = len(self.nodes) - 1
        outs = []
        for s in range(n_out):
            t = self._new_handle()
            t.kind, t.node, t.slot = "pending", idx, s
            t.dtype, t.shape = self.out_dtype(idx, s), self.out_shape(idx, s)
            outs.append(t)
        return outs[0] if n_out == 1 else tuple(outs)

    def out_shape(self, idx, slot):
        n = self.nodes[idx]
        if n.op == LAYER_NORM and slot > 0:
            return n.shape[:-1]
        return n.shape

    def out_dtype(self, idx, slot):
        n = self.nodes[idx]
        if n.op == LAYER_NORM and slot > 0:
            return F32
        return n.dtype

    @staticmethod
    def _promote(a: STensor, b: STensor):
        if a.dtype == b.dtype:
            return a.dtype
        if len(a.shape) == 0 and len(b.shape) > 0:
            return b.dtype
        if len(b.shape) == 0 and len(a.shape) > 0:
            return a.dtype
        fa, fb = _IS_FLOAT[a.dtype], _IS_FLOAT[b.dtype]
        if fa and fb:
            return F32
        if fa:
            return a.dtype
        if fb:
            return b.dtype
        return S64

    # ---- ops ----------------------------------------------------------------
    def _unary(self, op, x, attrs=(), dtype=None):
        x = self._t(x)
        return self._emit(op, x.dtype if dtype is None else dtype, x.shape, attrs, [x])

    def neg(self, x): return self._unary(NEG, x)
    def abs(self, x): return self._unary(ABS, x)
    def exp(self, x): return self._unary(EXP, x)
    def log(self, x): return self._unary(LOG, x)
    def tanh(self, x): return self._unary(TANH, x)
    def sqrt(self, x): return self._unary(SQRT, x)
    def rsqrt(self, x): return self._unary(RSQRT, x)
    def recip(self, x): return self._unary(RECIP, x)
    def relu(self, x): return self._unary(RELU, x)
    def gelu(self, x): return self._unary(GELU, x)
    def square(self, x): return self._unary(SQUARE, x)
    def sigmoid(self, x): return self._unary(SIGMOID, x)

    def cast(self, x, dtype):
        d = DTYPE_ID[dtype]
        return self._unary(CAST, x, [(A_DTYPE, False, d)], dtype=d)

    def _binary(self, op, a, b, extra=()):
        a, b = self._t(a), self._t(b)
        shape = broadcast_shapes(a.shape, b.shape)
        return self._emit(op, self._promote(a, b), shape, (), [a, b, *extra])

    def add(self, a, b, alpha=None):
        return self._binary(ADD, a, b, () if alpha is None else (self._t(alpha),))

    def sub(self, a, b): return self._binary(SUB, a, b)
    def mul(self, a, b): return self._binary(MUL, a, b)
    def div(self, a, b): return self._binary(DIV, a, b)
    def maximum(self, a, b): return self._binary(MAXIMUM, a, b)
    def minimum(self, a, b): return self._binary(MINIMUM, a, b)
    def relu_grad(self, dy, x): return self._binary(RELU_GRAD, dy, x)
    def gelu_grad(self, dy, x): return self._binary(GELU_GRAD, dy, x)

    @staticmethod
    def _dims_attrs(dims):
        return [(A_DIM0 + i, False, int(d)) for i, d in enumerate(dims)]

    def expand(self, x, size):
        x = self._t(x)
        size = tuple(int(d) for d in size)
        assert broadcast_shapes(x.shape, size) == size
        return self._emit(EXPAND, x.dtype, size, self._dims_attrs(size), [x])

    def reshape(self, x, size):
        x = self._t(x)
        size = tuple(int(d) for d in size)
        assert numel(size) == numel(x.shape)
        return self._emit(RESHAPE, x.dtype, size, self._dims_attrs(size), [x])

    def permute(self, x, dims):
        x = self._t(x)
        dims = tuple(int(d) for d in dims)
        assert sorted(dims) == list(range(len(x.shape)))
        return self._emit(PERMUTE, x.dtype, tuple(x.shape[d] for d in dims), self._dims_attrs(dims), [x])

    def narrow(self, x, axis, start, length):
        x = self._t(x)
        ax = int(axis) + (len(x.shape) if axis < 0 else 0)
        assert 0 <= start and start + length <= x.shape[ax]
        shape = x.shape[:ax] + (int(length),) + x.shape[ax + 1:]
        return self._emit(NARROW, x.dtype, shape, [(A_AXIS, False, ax), (A_START, False, int(start)), (A_LENGTH, False, int(length))], [x])

    def slice_update(self, base, update, axis, start):
        base, update = self._t(base), self._t(update)
        ax = int(axis) + (len(base.shape) if axis < 0 else 0)
        assert update.dtype == base.dtype and len(update.shape) == len(base.shape)
        assert all(u == b for i, (u, b) in enumerate(zip(update.shape, base.shape)) if i != ax)
        assert 0 <= start and start + update.shape[ax] <= base.shape[ax]
        return self._emit(SLICE_UPDATE, base.dtype, base.shape, [(A_AXIS, False, ax), (A_START, False, int(start))], [base, update])

    def _reduce(self, op, x, axis):
        x = self._t(x)
        if axis is None:
            return self._emit(op, x.dtype, (), (), [x])
        ax = int(axis) + (len(x.shape) if axis < 0 else 0)
        shape = x.shape[:ax] + x.shape[ax + 1:]
        return self._emit(op, x.dtype, shape, [(A_AXIS, False, ax)], [x])

    def sum(self, x, axis=None): return self._reduce(SUM, x, axis)
    def amax(self, x, axis=None): return self._reduce(AMAX, x, axis)
    def mean(self, x, axis=None): return self._reduce(MEAN, x, axis)

    def softmax(self, x):
        x = self._t(x)
        return self._emit(SOFTMAX, x.dtype, x.shape, (), [x])

    def softmax_grad(self, dy, y):
        y = self._t(y)
        return self._emit(SOFTMAX_GRAD, y.dtype, y.shape, (), [dy, y])

    def layer_norm(self, x, gamma, beta, eps=1e-5):
        x = self._t(x)
        return self._emit(LAYER_NORM, x.dtype, x.shape, [(A_EPS, True, float(eps))], [x, gamma, beta], n_out=3)

    def layer_norm_grad(self, dy, x, gamma, mean, rstd):
        x = self._t(x)
        return self._emit(LAYER_NORM_GRAD, x.dtype, x.shape, (), [dy, x, gamma, mean, rstd])

    def xent(self, logits, labels):
        logits = self._t(logits)
        return self._emit(XENT, F32, logits.shape[:-1], (), [logits, labels])

    def xent_grad(self, logits, labels, scale):
        logits = self._t(logits)
        return self._emit(XENT_GRAD, logits.dtype, logits.shape, (), [logits, labels, scale])

    def matmul(self, a, b, trans_a=False, trans_b=False, dtype=None):
        a, b = self._t(a), self._t(b)
        m, k = (a.shape[-1], a.shape[-2]) if trans_a else (a.shape[-2], a.shape[-1])
        k2, n = (b.shape[-1], b.shape[-2]) if trans_b else (b.shape[-2], b.shape[-1])
        assert k == k2, (a.shape, b.shape, trans_a, trans_b)
        if len(b.shape) > 2:
            assert a.shape[:-2] == b.shape[:-2]
        lead = a.shape[:-2]
        out_dt = DTYPE_ID[dtype] if dtype is not None else (a.dtype if a.dtype == b.dtype else F32)
        attrs = [(A_DTYPE, False, out_dt), (A_TRANS_A, False, int(bool(trans_a))),
                 (A_TRANS_B, False, int(bool(trans_b)))]
        return self._emit(MATMUL, out_dt, lead + (m, n), attrs, [a, b])

    def assign(self, dst: STensor, src: STensor):
        """In-place update as substitution of the destination's computation."""
        assert dst.alive and src.alive
        if dst is src:
            return
        self._refresh(src)
        if dst.view is not None:
            assert dst.dtype == src.dtype and dst.shape == src.shape
        donor = dst.donor
        if dst.kind == "data" and dst.buffer.donatable:
            donor = dst.buffer
        self._unbind(dst)
        dst.kind, dst.dtype, dst.shape = src.kind, src.dtype, src.shape
        dst.node, dst.slot, dst.buffer, dst.value = src.node, src.slot, src.buffer, src.value
        dst.memo_epoch, dst.memo_node = src.memo_epoch, src.memo_node
        if dst.kind == "data":
            dst.buffer.data_refs += 1
        dst.donor = donor
        dst.version += 1
        if dst.view is None:
            return
        # backward sequence: the base is rebuilt from the view's new value by the inverse view op
        base, kind, args = dst.view
        self._refresh(base)
        dst.seen = base.version
        if kind == PERMUTE:
            inv = [0] * len(args)
            for j, src_axis in enumerate(args):
                inv[src_axis] = j
            rebuilt = self.permute(dst, tuple(inv))
        elif kind == RESHAPE:
            rebuilt = self.reshape(dst, base.shape)
        else:
            rebuilt = self.slice_update(base, dst, args[0], args[1])
        self.assign(base, rebuilt)
        self.release(rebuilt)
        dst.seen = base.version

    # ---- barrier -------------------------------------------------------------
    def roots(self):
        """Live handles with a pending computation, ascending tensor id."""
        return [t for _, t in sorted(self.handles.items()) if t.alive and t.kind == "pending"]

    def canonical_order(self, root_values):
        """Post-order from each root in turn; operands visited last to first;
        every node emitted once.  Returns (order, index_of)."""
        order, index_of = [], {}
        for (rn, _slot) in root_values:
            if rn in index_of:
                continue
            stack = [(rn, False)]
            while stack:
                n, expanded = stack.pop()
                if n in index_of:
                    continue
                if expanded:
                    index_of[n] = len(order)
                    order.append(n)
                    continue
                stack.append((n, True))
                # pushed first-to-last => popped last-to-first
                for (c, _s) in self.nodes[n].ins:
                    if c not in index_of:
                        stack.append((c, False))
        return order, index_of

    def _donor_ordinal(self, t: STensor, param_ordinal_of_buffer, claimed):
        b = t.donor
        if b is None or id(b) not in param_ordinal_of_buffer or id(b) in claimed:
            return 0xFFFFFFFF
        if b.data_refs != 0 or b.dtype != t.dtype or b.shape != t.shape:
            return 0xFFFFFFFF
        claimed.add(id(b))
        return param_ordinal_of_buffer[id(b)]

    def serialise(self, order, index_of, roots):
        """Canonical little-endian byte string of the cut trace."""
        out = bytearray()
        n_param = n_scalar = 0
        param_ordinal_of_buffer = {}
        for n_idx in order:
            n = self.nodes[n_idx]
            out += struct.pack("<HBB", n.op, n.dtype, len(n.shape))
            for d in n.shape:
                out += struct.pack("<q", d)
            out += struct.pack("<B", len(n.attrs))
            for (key, isf, payload) in n.attrs:
                out += struct.pack("<HB", key, 1 if isf else 0)
                out += struct.pack("<d", payload) if isf else struct.pack("<q", payload)
            out += struct.pack("<B", len(n.ins))
            for (c, s) in n.ins:
                out += struct.pack("<IB", index_of[c], s)
            if n.op == DEVICE_DATA:
                # own ordinal, then that of the first leaf on the same buffer (its alias class)
                first = param_ordinal_of_buffer.setdefault(id(n.buffer), n_param)
                out += struct.pack("<II", n_param, first)
                n_param += 1
            elif n.op == SCALAR_PARAM:
                out += struct.pack("<I", n_scalar)
                n_scalar += 1
        out += struct.pack("<I", len(roots))
        claimed = set()
        donors = []
        for t in roots:
            d = self._donor_ordinal(t, param_ordinal_of_buffer, claimed)
            donors.append(d)
            out += struct.pack("<IBI", index_of[t.node], t.slot, d)
        return bytes(out), donors

    def dump_ir(self) -> str:
        """Text form of the pending trace, in the layout of the paper's figure 1."""
        self._refresh_views()
        roots = self.roots()
        order, index_of = self.canonical_order([(t.node, t.slot) for t in roots])
        lines = ["IR {"]
        for i, n_idx in enumerate(order):
            n = self.nodes[n_idx]
            dims = ",".join(str(d) for d in n.shape)
            args = ", ".join(f"%{index_of[c]}" + (f".{s}" if s else "") for (c, s) in n.ins)
            line = f"    %{i} = {DTYPE_NAME[n.dtype]}[{dims}] {OP_NAME[n.op]}({args})"
            extras = []
            if n.op in (DEVICE_DATA, SCALAR_PARAM):
                extras.append(f"device={self.device_name}")
            elif n.op == CONSTANT:
                v = n.attrs[0][2]
                extras.append(f"value={int(v) if float(v).is_integer() else v}")
            elif n.op in (EXPAND, RESHAPE):
                extras.append("size=(" + ", ".join(str(d) for d in n.shape) + ")")
            elif n.op == PERMUTE:
                extras.append("dims=(" + ", ".join(str(a[2]) for a in n.attrs) + ")")
            else:
                for (key, isf, payload) in n.attrs:
                    name = {A_DTYPE: "dtype", A_AXIS: "axis", A_EPS: "eps",
                            A_TRANS_A: "trans_a", A_TRANS_B: "trans_b"}.get(key, f"attr{key}")
                    if key == A_DTYPE:
                        payload = DTYPE_NAME[payload]
                    extras.append(f"{name}={payload:g}" if isf else f"{name}={payload}")
            for k, t in enumerate(roots):
                if t.node == n_idx:
                    extras.append(f"ROOT={k}" + (f".{t.slot}" if t.slot else ""))
            lines.append(", ".join([line] + extras))
        lines.append("}")
        return "\n".join(lines)

    def barrier(self, blocking: bool = True):
        """Cut, number, serialise, hash, consult the cache, lower on a miss,
        then rebind every root to fresh data.  Returns a dict of results."""
        self._refresh_views()
        roots = self.roots()
        order, index_of = self.canonical_order([(t.node, t.slot) for t in roots])
        blob, donors = self.serialise(order, index_of, roots)
        h = fnv1a64(blob)
        key = (h, len(blob))
        hit = key in self.cache and self.cache[key][0] == blob
        if not hit:
            self.cache[key] = (blob, self.lower(order, index_of, roots, donors))
        low = self.cache[key][1]
        plan_text = low["plan"]
        # result binding: every root becomes data -- on the donated buffer when it
        # was written in place, on the aliased input when folding reduced it to a
        # leaf, else on a fresh library-owned (hence donatable) buffer
        param_nodes = [i for i in order if self.nodes[i].op == DEVICE_DATA]
        for k, t in enumerate(roots):
            v = low["root_vals"][k]
            leaf = self.nodes[order[v[0]]]
            t.kind = None
            if k in low["inplace_roots"]:
                self._bind_data(t, self.nodes[param_nodes[low["inplace_roots"][k]]].buffer)
            elif leaf.op == DEVICE_DATA:
                self._bind_data(t, leaf.buffer)
            elif leaf.op in (SCALAR_PARAM, CONSTANT):
                t.kind, t.value = "scalar", (leaf.value if leaf.op == SCALAR_PARAM else leaf.attrs[0][2])
            else:
                self._bind_data(t, Buffer(t.dtype, t.shape, True))
        for t in list(self.handles.values()):
            t.donor = None
        self.nodes = []
        self.epoch += 1
        self.last = {"hash": h, "cache_hit": hit, "n_nodes": len(order), "bytes": blob,
                     "plan": plan_text, "n_regions": plan_text.count("\n") + (1 if plan_text else 0)}
        return self.last

    def fetch(self, t: STensor):
        self._refresh(t)
        if t.kind == "pending":
            self.barrier(True)
        return None

    # ---- lowering: folding + partition ------------------------------------------
    def lower(self, order, index_of, roots, donors) -> dict:
        """Returns {"plan": text, "root_vals": resolved root values,
        "inplace_roots": {root position: donated parameter ordinal}}."""
        N = len(order)
        nd = [self.nodes[i] for i in order]
        ins = [[(index_of[c], s) for (c, s) in n.ins] for n in nd]

        def oshape(v):
            n = nd[v[0]]
            return n.shape[:-1] if (n.op == LAYER_NORM and v[1] > 0) else n.shape

        def odtype(v):
            n = nd[v[0]]
            return F32 if (n.op == LAYER_NORM and v[1] > 0) else n.dtype

        # -- special-scalar folding (values 0 and 1 only) --------------------------
        fwd = {}                       # node index -> replacement value (node, slot)

        def res(v):
            while v[1] == 0 and v[0] in fwd:
                v = fwd[v[0]]
            return v

        def const_of(v):
            v = res(v)
            n = nd[v[0]]
            if n.op == CONSTANT:
                return n.attrs[0][2]
            if n.op in (EXPAND, RESHAPE):
                return const_of(ins[v[0]][0])
            return None

        drop_alpha = set()
        for i in range(N):
            n = nd[i]

            def same(v):
                return oshape(res(v)) == n.shape and odtype(res(v)) == n.dtype

            o = ins[i]
            if n.op == ADD and len(o) == 3 and const_of(o[2]) == 1:
                drop_alpha.add(i)
            two = len(o) == 2 or i in drop_alpha
            if n.op == MUL:
                if const_of(o[1]) == 1 and same(o[0]):
                    fwd[i] = res(o[0])
                elif const_of(o[0]) == 1 and same(o[1]):
                    fwd[i] = res(o[1])
            elif n.op == ADD and two:
                if const_of(o[1]) == 0 and same(o[0]):
                    fwd[i] = res(o[0])
                elif const_of(o[0]) == 0 and same(o[1]):
                    fwd[i] = res(o[1])
            elif n.op == SUB:
                if const_of(o[1]) == 0 and same(o[0]):
                    fwd[i] = res(o[0])
            elif n.op == DIV:
                if const_of(o[1]) == 1 and same(o[0]):
                    fwd[i] = res(o[0])
        rins = []
        for i in range(N):
            o = [res(v) for v in ins[i]]
            if i in drop_alpha:
                o = o[:2]
            rins.append(o)
        root_vals = [res((index_of[t.node], t.slot)) for t in roots]

        # -- liveness after folding ----------------------------------------------
        live = [False] * N
        stack = [v[0] for v in root_vals]
        while stack:
            i = stack.pop()
            if live[i]:
                continue
            live[i] = True
            stack.extend(v[0] for v in rins[i])

        LEAF, VIEW, EW, ROW, COL, ALL, MM, SLICE = "LEAF", "VIEW", "EW", "ROW", "COL", "ALL", "MM", "SLICE"

        def klass(i):
            n = nd[i]
            if n.op in (DEVICE_DATA, SCALAR_PARAM, CONSTANT):
                return LEAF
            if n.op in (EXPAND, RESHAPE):
                # a view that must itself be materialised (it is a root) is a copy
                return EW if is_root[i] else VIEW
            if n.op == PERMUTE:
                # a permutation that only feeds contractions is addressing (operand strides), not a copy
                return VIEW if (not is_root[i] and pre_users[i] and all(nd[u].op == MATMUL for u in pre_users[i])) else EW
            if n.op == NARROW:
                # a window is addressing for elementwise ops, contractions and permutations; otherwise a copy
                ok = not is_root[i] and pre_users[i] and all(
                    nd[u].op in UNARY or nd[u].op in BINARY or nd[u].op in (MATMUL, PERMUTE) for u in pre_users[i])
                return VIEW if ok else EW
            if n.op == SLICE_UPDATE:
                return SLICE
            if n.op in UNARY or n.op in BINARY:
                return EW
            if n.op in PLAIN_REDUCE:
                in_shape = oshape(rins[i][0])
                axis = [a for a in n.attrs if a[0] == A_AXIS]
                if not axis or len(in_shape) <= 1:
                    return ALL
                ax = axis[0][2]
                if ax == len(in_shape) - 1:
                    return ROW
                if ax == 0:
                    return COL
                raise NotImplementedError("reduction over a middle axis")
            if n.op in ROW_OPS:
                return ROW
            if n.op == MATMUL:
                return MM
            raise NotImplementedError(n.op)

        is_root = [False] * N
        for v in root_vals:
            is_root[v[0]] = True
        pre_users = [[] for _ in range(N)]      # live users, needed before classes exist
        for j in range(N):
            if live[j]:
                for v in rins[j]:
                    if j not in pre_users[v[0]]:
                        pre_users[v[0]].append(j)
        cls = [klass(i) if live[i] else "DEAD" for i in range(N)]

        def is_imm(v):
            n = nd[v[0]]
            if n.op in (CONSTANT, SCALAR_PARAM):
                return True
            if n.op in (EXPAND, RESHAPE):
                return is_imm(rins[v[0]][0])
            return False

        def base(v):
            while cls[v[0]] == VIEW:
                v = rins[v[0]][0]
            return v

        users = [[] for _ in range(N)]          # direct users (live)
        for j in range(N):
            if live[j]:
                for v in rins[j]:
                    if j not in users[v[0]]:
                        users[v[0]].append(j)

        def eff_users(i):
            out, stack = [], list(users[i])
            while stack:
                u = stack.pop()
                if cls[u] == VIEW:
                    stack.extend(users[u])
                elif u not in out:
                    out.append(u)
            return out

        # -- pass 0: singleton regions -----------------------------------------------
        region_of = {}
        regions = {}                            # rid -> dict

        def rid_of(r):
            return r["anchor"] if r["anchor"] is not None else min(r["members"])

        for i in range(N):
            if cls[i] in (EW, ROW, COL, ALL, MM, SLICE):
                r = {"kind": cls[i], "anchor": None if cls[i] == EW else i, "members": {i}, "fin_shape": None}
                regions[id(r)] = r
                region_of[i] = r

        def region_io(members):
            inputs, outputs = [], []
            for m in sorted(members):
                for v in rins[m]:
                    if v[0] in members or is_imm(v):
                        continue
                    if v not in inputs:
                        inputs.append(v)
            for m in sorted(members):
                n_out = 3 if nd[m].op == LAYER_NORM else 1
                for s in range(n_out):
                    ext = any(r == (m, s) for r in root_vals)
                    for u in users[m]:
                        if (m, s) in rins[u] and not (u in members):
                            ext = True
                    if ext:
                        outputs.append((m, s))
            return inputs, outputs

        def caps_ok(members):
            # a permutation's operand must be in memory: never computed in the permutation's own region
            if any(nd[m].op == PERMUTE and rins[m][0][0] in members for m in members):
                return False
            # ... and so must any value that a member reads through a view
            if any(cls[v[0]] == VIEW and base(v)[0] in members for m in members for v in rins[m]):
                return False
            inputs, outputs = region_io(members)
            return (len(inputs) <= MAX_INPUTS and len(outputs) <= MAX_OUTPUTS
                    and len(inputs) + len(members) <= MAX_SLOTS)

        def merge(r, i):
            s = region_of[i]
            del regions[id(s)]
            r["members"].add(i)
            region_of[i] = r

        # -- pass 1: prologue absorption into plain reductions ------------------------
        for a in range(N):
            if cls[a] in (ROW, COL, ALL) and nd[a].op in PLAIN_REDUCE:
                r = region_of[a]
                in_shape = oshape(rins[a][0])
                for i in range(a - 1, -1, -1):
                    if cls[i] != EW or len(region_of[i]["members"]) != 1 or is_root[i]:
                        continue
                    if nd[i].shape != in_shape or not users[i]:
                        continue
                    if not all(u in r["members"] for u in users[i]):
                        continue
                    if not caps_ok(r["members"] | {i}):
                        continue
                    merge(r, i)

        # -- pass 2: epilogue / finaliser / elementwise grouping -----------------------
        extra_succ = {}                         # ordering-only edges added by donation

        def successors(r):
            out = list(extra_succ.get(id(r), []))
            for m in r["members"]:
                for u in eff_users(m):
                    ru = region_of[u]
                    if ru is not r and ru not in out:
                        out.append(ru)
            return out

        def reachable(src, dst):
            seen, stack = set(), [src]
            while stack:
                x = stack.pop()
                if x is dst:
                    return True
                if id(x) in seen:
                    continue
                seen.add(id(x))
                stack.extend(successors(x))
            return False

        def compatible(r, i):
            if r.get("sealed"):
                return False
            shape = nd[i].shape
            if r["kind"] == EW:
                return shape == nd[min(r["members"])].shape
            a = r["anchor"]
            if r["kind"] == MM:
                return shape == nd[a].shape
            if nd[a].op in PLAIN_REDUCE:
                if shape == nd[a].shape:
                    return True
                if (r["kind"] == ALL and len(shape) >= 1 and numel(shape) <= MAX_FINALISER_ELEMS
                        and r["fin_shape"] in (None, shape)):
                    return True
            return False

        def can_union(a, b):
            """Merging regions a and b keeps the region graph acyclic iff neither
            reaches the other through a third region."""
            for x in successors(a):
                if x is not b and reachable(x, b):
                    return False
            for x in successors(b):
                if x is not a and reachable(x, a):
                    return False
            return True

        def union(home, other):
            for m in other["members"]:
                region_of[m] = home
            home["members"] |= other["members"]
            del regions[id(other)]

        for i in range(N):
            if cls[i] != EW or len(region_of[i]["members"]) != 1:
                continue
            if nd[i].op == PERMUTE:
                # a permutation of a bare contraction result that nothing else reads becomes the
                # contraction's output layout
                v = rins[i][0]
                a = v[0]
                if (cls[a] == MM and v[1] == 0 and region_of[a]["members"] == {a} and users[a] == [i]
                        and not is_root[a]):
                    union(region_of[a], region_of[i])
                    region_of[a]["sealed"] = True      # the layout change ends the region
                continue
            cand = []
            for v in rins[i]:
                if v[0] in region_of and region_of[v[0]] not in cand:
                    cand.append(region_of[v[0]])
            cand.sort(key=lambda r: (0 if r["kind"] != EW else 1, -rid_of(r)))
            home = region_of[i]
            for r in cand:
                if id(r) not in regions or r is home:
                    continue
                if r["kind"] != EW:
                    # join an anchored region as epilogue / finaliser member
                    if len(home["members"]) != 1:
                        continue
                    if not compatible(r, i) or not caps_ok(r["members"] | {i}) or not can_union(r, home):
                        continue
                    if r["kind"] == ALL and nd[i].shape != nd[r["anchor"]].shape:
                        r["fin_shape"] = nd[i].shape
                    union(r, home)
                    home = r
                    # elementwise producers of i that feed nothing but this region (e.g. beta*m of
                    # an optimiser update) are computed by the region's post program too
                    for v in rins[i]:
                        q = region_of.get(v[0])
                        if q is None or q is home or q["kind"] != EW or id(q) not in regions:
                            continue
                        if nd[min(q["members"])].shape != nd[i].shape or any(is_root[m] for m in q["members"]):
                            continue
                        if not all(u in q["members"] or u in home["members"] for m in q["members"] for u in users[m]):
                            continue
                        if any(u == home["anchor"] for m in q["members"] for u in users[m]):
                            continue      # (what the anchor itself reads must exist in memory)
                        if not caps_ok(home["members"] | q["members"]) or not can_union(home, q):
                            continue
                        union(home, q)
                elif home["kind"] == EW:
                    # grow one elementwise region out of producer regions of equal shape
                    if not compatible(r, i) or not caps_ok(r["members"] | home["members"]):
                        continue
                    if not can_union(r, home):
                        continue
                    union(r, home)
                    home = r

        # -- pass 3: donation.  A root whose old buffer was donated is written in place
        # when (i) inside the writing region the donor is only read index-aligned (by
        # elementwise members, directly -- never as the anchor's operand, through a
        # view or by a permute) and (ii) every other region that reads the donor can
        # be ordered before the writer.  (ii) is enforced by adding reader->writer
        # ordering edges, which is refused when the reader depends on the writer.
        param_nodes = [i for i in range(N) if nd[i].op == DEVICE_DATA]   # ordinal = position
        rlist = list(regions.values())
        inplace = {id(r): [] for r in rlist}
        inplace_roots = {}
        for k, (t, d, v) in enumerate(zip(roots, donors, root_vals)):
            if d == 0xFFFFFFFF or v[0] not in region_of:
                continue
            rw = region_of[v[0]]
            dup = [w for w, _ in inplace[id(rw)] if w == v]
            if dup:
                continue
            # every leaf that names the donated buffer
            pn = {(i, 0) for i in param_nodes if nd[i].buffer is nd[param_nodes[d]].buffer}
            # a second live tensor that folding reduced to the donor leaf itself (b = a * 1) is
            # rebound to the donor's buffer by the barrier: it must keep the old value
            ok = not any(w in pn for j, w in enumerate(root_vals) if j != k)
            # a buffer that the cut knows under two parameter numbers is never written in place
            if sum(1 for (i, _) in pn if live[i]) > 1:
                ok = False
            readers = []
            for r in sorted(rlist, key=rid_of):
                if not any(base(x) in pn for m in r["members"] for x in rins[m]):
                    continue
                if r is rw:
                    for m in r["members"]:
                        for x in rins[m]:
                            if base(x) not in pn:
                                continue
                            # a window update may overwrite its own base (operand 0) in place
                            if (m == rw["anchor"] and nd[m].op == SLICE_UPDATE and x in pn and x == rins[m][0]
                                    and base(rins[m][1]) not in pn):
                                continue
                            if m == rw["anchor"] or x not in pn or nd[m].op in (PERMUTE, EXPAND, RESHAPE, NARROW):
                                ok = False
                else:
                    readers.append(r)
            if ok and any(reachable(rw, r) for r in readers):
                ok = False
            if ok:
                for r in readers:
                    if rw not in extra_succ.setdefault(id(r), []):
                        extra_succ[id(r)].append(rw)
                inplace[id(rw)].append((v, d))
                inplace_roots[k] = d

        # -- pass 4: deterministic topological order of regions (smallest id first) ----------
        preds = {id(r): set() for r in rlist}
        for r in rlist:
            for s in successors(r):
                preds[id(s)].add(id(r))
        done, ordered = set(), []
        while len(ordered) < len(rlist):
            ready = [r for r in rlist if id(r) not in done and preds[id(r)] <= done]
            r = min(ready, key=rid_of)
            done.add(id(r))
            ordered.append(r)

        lines = []
        for k, r in enumerate(ordered):
            inputs, outputs = region_io(r["members"])
            a = "-" if r["anchor"] is None else str(r["anchor"])
            lines.append(
                f"R{k} {r['kind']} anchor={a} members=[{','.join(str(m) for m in sorted(r['members']))}]"
                f" inputs=[{','.join(f'{n}.{s}' for n, s in inputs)}]"
                f" outputs=[{','.join(f'{n}.{s}' for n, s in outputs)}]"
                f" inplace=[{','.join(f'{v[0]}.{v[1]}->p{d}' for v, d in inplace[id(r)])}]")
        return {"plan": "\n".join(lines), "root_vals": root_vals, "inplace_roots": inplace_roots}
