"""ctypes binding with the same names as include/lt.h.  Argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

DTYPES = {"f32": 0, "bf16": 1, "s32": 2, "s64": 3}
_DTYPE_NAMES = {v: k for k, v in DTYPES.items()}
_DTYPE_BYTES = {0: 4, 1: 2, 2: 4, 3: 8}

OPCODES = {
    "neg": 16, "abs": 17, "exp": 18, "log": 19, "tanh": 20, "sqrt": 21, "rsqrt": 22, "recip": 23,
    "relu": 24, "gelu": 25, "square": 26, "cast": 27, "sigmoid": 28,
    "add": 32, "sub": 33, "mul": 34, "div": 35, "maximum": 36, "minimum": 37, "relu_grad": 38, "gelu_grad": 39,
    "expand": 48, "reshape": 49, "permute": 50, "narrow": 51, "slice_update": 52,
    "sum": 64, "amax": 65, "mean": 66,
    "softmax": 80, "softmax_grad": 81, "layer_norm": 82, "layer_norm_grad": 83, "xent": 84, "xent_grad": 85,
    "matmul": 96,
}
ATTR_VALUE, ATTR_DTYPE, ATTR_AXIS, ATTR_EPS, ATTR_TRANS_A, ATTR_TRANS_B, ATTR_START, ATTR_LENGTH, ATTR_DIM0 = 1, 2, 3, 4, 5, 6, 7, 8, 16
LT_DONATABLE = 1
MAX_RANK = 6


class _AttrV(C.Union):
    _fields_ = [("i", C.c_int64), ("f", C.c_double)]


class lt_attr(C.Structure):
    _fields_ = [("key", C.c_uint16), ("is_float", C.c_uint8), ("v", _AttrV)]


class BarrierInfo(C.Structure):
    _fields_ = [("hash", C.c_uint64), ("key_bytes", C.c_uint64), ("cache_hit", C.c_int32),
                ("n_nodes", C.c_int32), ("n_roots", C.c_int32), ("n_regions", C.c_int32),
                ("n_launches", C.c_int32), ("bytes_planned", C.c_uint64), ("flops_planned", C.c_uint64),
                ("ns_collect", C.c_uint64), ("ns_hash", C.c_uint64), ("ns_lower", C.c_uint64),
                ("ns_launch", C.c_uint64)]


class Stats(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in (
        "barriers", "cache_hits", "cache_misses", "nodes_recorded", "regions_launched", "kernels_launched",
        "ns_lowering_total", "arena_bytes_in_use", "arena_bytes_peak", "live_tensors", "fallback_ops", "replays", "graph_launches", "graphs_built", "quick_hits")]


class TensorDesc(C.Structure):
    _fields_ = [("dptr", C.c_void_p), ("dtype", C.c_int32), ("rank", C.c_int32), ("dims", C.c_int64 * 6),
                ("is_scalar", C.c_int32), ("scalar", C.c_double)]


FALLBACK_FN = C.CFUNCTYPE(C.c_int, C.c_void_p, C.c_uint16, C.POINTER(TensorDesc), C.c_int, C.POINTER(lt_attr), C.c_int,
                          C.POINTER(TensorDesc), C.c_int, C.c_int, C.c_void_p)
OP_CUSTOM = 1024


class LaunchRecord(C.Structure):
    _fields_ = [("kernel", C.c_char * 48), ("region", C.c_int32), ("ms", C.c_float),
                ("bytes", C.c_uint64), ("flops", C.c_uint64)]


class Step:
    """A captured step (lt_step): `replay` runs its plan again on the current data of the same
    tensors; `scalars` are the captured values of its non-special scalars in canonical order."""

    def __init__(self, ctx, handle):
        self._ctx, self._h = ctx, handle
        n = ctx._lib.lt_step_scalars(handle, None, 0)
        buf = (C.c_double * max(1, n))()
        ctx._lib.lt_step_scalars(handle, buf, n)
        self.scalars = [buf[i] for i in range(n)]

    def replay(self, scalars=None, blocking=True) -> "BarrierInfo":
        ctx = self._ctx
        ctx._flush()
        info = BarrierInfo()
        if scalars is None:
            arr, n = None, 0
        else:
            n = len(scalars)
            arr = (C.c_double * max(1, n))(*[float(v) for v in scalars])
        ctx._check(ctx._lib.lt_step_replay(ctx._h, self._h, arr, n, 1 if blocking else 0, C.byref(info)))
        ctx._kept.clear()
        return info

    def free(self):
        if self._h:
            self._ctx._lib.lt_step_free(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


class LtError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"lt_status {status}: {message}")
        self.status = status


def library_path() -> str:
    return os.path.join(_HERE, "liblt.so")


def load_library():
    """Load liblt.so.  It must have been built (python -m paper_2102_13267_amd.build);
    there is no fallback: without the native library nothing in this package works."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it with `python -m paper_2102_13267_amd.build`")
    # PyTorch-ROCm ships its own HIP runtime under the same soname as /opt/rocm's.  One process
    # must use one runtime, so torch's is loaded first and liblt.so then binds to it.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = C.CDLL(path)
    P, u64, i32 = C.c_void_p, C.c_uint64, C.c_int
    sig = {
        "lt_init": [i32, P, P, C.c_size_t, C.POINTER(P)],
        "lt_shutdown": [P],
        "lt_tensor_from_device": [P, P, i32, i32, C.POINTER(C.c_int64), C.c_uint32, C.POINTER(u64)],
        "lt_scalar": [P, i32, C.c_double, C.POINTER(u64)],
        "lt_op": [P, C.c_uint16, C.POINTER(u64), i32, C.POINTER(lt_attr), i32, C.POINTER(u64), i32],
        "lt_assign": [P, u64, u64],
        "lt_view": [P, u64, C.c_uint16, C.POINTER(lt_attr), i32, C.POINTER(u64)],
        "lt_release": [P, u64],
        "lt_barrier": [P, i32, C.POINTER(BarrierInfo)],
        "lt_barrier_static": [P, i32, C.POINTER(BarrierInfo)],
        "lt_fetch": [P, u64, P, C.c_size_t],
        "lt_device_ptr": [P, u64, C.POINTER(P)],
        "lt_shape": [P, u64, C.POINTER(i32), C.POINTER(i32), C.POINTER(C.c_int64)],
        "lt_dump_ir": [P, C.c_char_p, C.c_size_t, C.POINTER(C.c_size_t)],
        "lt_dump_plan": [P, C.c_char_p, C.c_size_t, C.POINTER(C.c_size_t)],
        "lt_dump_schedule": [P, C.c_char_p, C.c_size_t, C.POINTER(C.c_size_t)],
        "lt_dump_key": [P, P, C.c_size_t, C.POINTER(C.c_size_t)],
        "lt_stats": [P, C.POINTER(Stats)],
        "lt_release_many": [P, C.POINTER(C.c_uint64), C.c_size_t],
        "lt_set_profiling": [P, i32],
        "lt_set_streams": [P, i32],
        "lt_set_fusion": [P, i32],
        "lt_set_graphs": [P, i32],
        "lt_set_quick_lookup": [P, i32],
        "lt_set_fallback": [P, FALLBACK_FN, P],
        "lt_last_launches": [P, C.POINTER(LaunchRecord), i32, C.POINTER(i32)],
        "lt_step_capture": [P, C.POINTER(P)],
        "lt_step_replay": [P, P, C.POINTER(C.c_double), i32, i32, C.POINTER(BarrierInfo)],
        "lt_step_scalars": [P, C.POINTER(C.c_double), i32],
        "lt_tensor_rebind": [P, u64, P],
    }
    for name, argtypes in sig.items():
        fn = getattr(lib, name)
        fn.argtypes = argtypes
        fn.restype = C.c_int
    lib.lt_step_free.argtypes = [P]
    lib.lt_step_free.restype = None
    lib.lt_last_error.argtypes = [P]
    lib.lt_last_error.restype = C.c_char_p
    # the recording fast path makes the same calls from C; it gets the entry points' addresses
    if _ltrec is None:   # no fallback: without the native parts nothing in this package works
        raise ImportError("paper_2102_13267_amd/_ltrec extension is missing or stale: run python -m paper_2102_13267_amd.build")
    addr = lambda fn: C.cast(fn, C.c_void_p).value
    _ltrec.init(addr(lib.lt_op), addr(lib.lt_scalar), addr(lib.lt_release), addr(lib.lt_last_error), addr(lib.lt_assign),
                addr(lib.lt_release_many), addr(lib.lt_barrier))
    global _REC
    _REC = _ltrec
    _LIB = lib
    return lib


_NO_ATTRS = (lt_attr * 1)()   # what an op without attributes passes (never read)
_NO_ATTRS_ADDR = C.addressof(_NO_ATTRS)
_REC = None                   # the _ltrec extension (set by load_library)


# The tensor handle is a C type of the recording extension (creating and dropping one per recorded
# op is part of the hot path): Tensor(ctx, tid, dtype=None, shape=None, keep=None) with attributes
# ctx, tid, dtype, shape.  Dropping the last Python reference releases the tensor, which is how the
# library learns that it is no longer live (liveness matters when the trace is cut, not before: dead
# ids are collected in Context._dead and handed over in one call -- see Context._flush).  Element
# type and shape of an op's result are asked from the library only when somebody reads them.
_LTREC_API = 6   # what this file expects of the extension (its `API` attribute)
try:
    from . import _ltrec
    if getattr(_ltrec, "API", 0) != _LTREC_API:
        raise ImportError("stale _ltrec")
    Tensor = _ltrec.Tensor
except ImportError:   # not built yet, or built from older sources: load_library() says so
    _ltrec = None     # (the package must stay importable for its own build module)
    Tensor = None


def _query(t):
    dt, rank = C.c_int(), C.c_int()
    dims = (C.c_int64 * MAX_RANK)()
    t.ctx._check(t.ctx._lib.lt_shape(t.ctx._h, t.tid, C.byref(dt), C.byref(rank), dims))
    t._dtype, t._shape = _DTYPE_NAMES[dt.value], tuple(dims[i] for i in range(rank.value))


if _ltrec is not None:
    _ltrec.set_query(_query)
    _ltrec.set_error(LtError)   # a failed call raises LtError(status, message) straight from C
    _rec_op = _ltrec.op


def _plain(name, arity):
    """Context method that records op `name` (no attributes, `arity` operands: tensors or numbers):
    a method descriptor of the extension, called without a Python frame of its own."""
    if _ltrec is None:      # (not built: nothing can be recorded anyway, load_library() says so)
        return None
    return _ltrec.PlainOp(name, OPCODES[name], arity, arity)


_CAST, _EXPAND, _RESHAPE, _PERMUTE = OPCODES["cast"], OPCODES["expand"], OPCODES["reshape"], OPCODES["permute"]
_NARROW, _SLICE_UPDATE = OPCODES["narrow"], OPCODES["slice_update"]
_SUM, _AMAX, _MEAN = OPCODES["sum"], OPCODES["amax"], OPCODES["mean"]
_LAYER_NORM, _MATMUL = OPCODES["layer_norm"], OPCODES["matmul"]


class Context:
    """One lt_ctx.  device=None gives the null device ("CPU:0": records, hashes, lowers, launches
    nothing).  Otherwise `device` is a HIP ordinal and the workspace is a torch byte tensor."""

    def __init__(self, device=None, workspace_bytes=None, stream=None):
        self._lib = load_library()
        self._h = C.c_void_p()
        self._ids, self._outs, self._attrs = {}, {}, {}     # reusable ctypes argument arrays of op()
        self._dead = []                                     # ids of dropped tensors, not yet released
        self._kept = []                                     # owners of device memory that dropped leaves of the pending trace name
        self._torch = None
        self._workspace = None
        if device is None:   # (no size given: addresses are planned in an unbounded workspace)
            self._check_init(self._lib.lt_init(-1, None, None, int(workspace_bytes or 0), C.byref(self._h)))
            self.device = None
        else:
            import torch
            if not torch.cuda.is_available():
                raise RuntimeError("no GPU visible: the HIP path cannot run (there is no CPU fallback)")
            self._torch = torch
            self.device = int(device)
            workspace_bytes = int(workspace_bytes or (1 << 30))
            torch.cuda.set_device(self.device)
            self._workspace = torch.empty(int(workspace_bytes), dtype=torch.uint8, device=f"cuda:{self.device}")
            st = stream if stream is not None else torch.cuda.current_stream(self.device)
            self._stream = st
            self._check_init(self._lib.lt_init(self.device, C.c_void_p(st.cuda_stream), C.c_void_p(self._workspace.data_ptr()),
                                               int(workspace_bytes), C.byref(self._h)))

    def _check_init(self, st):
        if st != 0:
            raise LtError(st, (self._lib.lt_last_error(None) or b"").decode())
        self._hv = self._h.value or 0   # the context pointer as a plain int, for the recording fast path

    def _check(self, st):
        if st != 0:
            raise LtError(st, (self._lib.lt_last_error(self._h) or b"").decode())

    def _flush(self):
        """Release the tensors that Python dropped since the last call (one call for all of them).
        Runs before anything that looks at liveness: barrier, fetch, the dumps, the statistics."""
        if self._dead:
            _ltrec.release_many(self._hv, self._dead)   # (empties the list; a closed context just forgets them)

    def close(self):
        if self._h:
            self._flush()
            self._lib.lt_shutdown(self._h)
            self._h = C.c_void_p()
            self._hv = 0

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- factories -----------------------------------------------------------------------
    def from_device(self, dptr, dtype, shape, donatable=False, keep=None) -> Tensor:
        dims = (C.c_int64 * max(1, len(shape)))(*shape)
        out = C.c_uint64()
        self._check(self._lib.lt_tensor_from_device(self._h, C.c_void_p(dptr), DTYPES[dtype], len(shape), dims,
                                                     LT_DONATABLE if donatable else 0, C.byref(out)))
        return Tensor(self, out.value, dtype, shape, keep)

    def tensor(self, array, dtype=None, donatable=False) -> Tensor:
        """Upload a NumPy array (or adopt a torch tensor already on the device)."""
        if self.device is None:
            a = np.asarray(array)
            if dtype is None:
                dtype = "s32" if a.dtype == np.int32 else "s64" if a.dtype == np.int64 else "f32"
            return self.from_device(0, dtype, a.shape, donatable)
        torch = self._torch
        if isinstance(array, torch.Tensor):
            t = array
            if dtype is None:
                dtype = {torch.float32: "f32", torch.bfloat16: "bf16", torch.int32: "s32", torch.int64: "s64"}[t.dtype]
        else:
            a = np.ascontiguousarray(array)
            if dtype is None:
                dtype = "s32" if a.dtype == np.int32 else "s64" if a.dtype == np.int64 else "f32"
            if a.dtype == np.float64:
                a = a.astype(np.float32)
            t = torch.from_numpy(a).to(f"cuda:{self.device}")
            if dtype == "bf16":
                t = t.to(torch.bfloat16)
        t = t.contiguous()
        return self.from_device(t.data_ptr(), dtype, tuple(t.shape), donatable, keep=t)

    def scalar(self, value, dtype="f32") -> Tensor:
        out = C.c_uint64()
        self._check(self._lib.lt_scalar(self._h, DTYPES[dtype], float(value), C.byref(out)))
        return Tensor(self, out.value, dtype, ())

    # ---- generic op -------------------------------------------------------------------------
    def _t(self, x) -> Tensor:
        return x if isinstance(x, Tensor) else self.scalar(x)

    def _encode(self, key, attrs):
        """The lt_attr block of `attrs` ((key, value) pairs), built once per distinct `key` and kept."""
        arr = (lt_attr * max(1, len(attrs)))()
        for i, (k, val) in enumerate(attrs):
            arr[i].key = k
            if isinstance(val, float):
                arr[i].is_float = 1
                arr[i].v.f = val
            else:
                arr[i].is_float = 0
                arr[i].v.i = int(val)
        at = self._attrs[key] = (C.addressof(arr), len(attrs), arr)   # (arr is kept alive here)
        return at

    def op(self, name, inputs, attrs=(), n_out=1):
        # recording an op is a hot path of the method: the call goes through the C fast path, which
        # also turns Python numbers among the operands into scalar tensors that live for the call
        if attrs:
            key = tuple(attrs)
            at = self._attrs.get(key) or self._encode(key, key)
            addr, n_attr = at[0], at[1]
        else:
            addr, n_attr = _NO_ATTRS_ADDR, 0
        return _rec_op(self, self._hv, OPCODES[name], inputs, addr, n_attr, n_out)

    def _dims_op(self, code, x, dims):
        # (the attribute block of a shape is looked up by the shape itself, not rebuilt per call)
        key = (code, dims if type(dims) is tuple else tuple(dims))
        at = self._attrs.get(key) or self._encode(key, [(ATTR_DIM0 + i, int(d)) for i, d in enumerate(key[1])])
        return _rec_op(self, self._hv, code, (x,), at[0], at[1], 1)

    def _axis_op(self, code, x, axis):
        if axis is None:
            return _rec_op(self, self._hv, code, (x,), _NO_ATTRS_ADDR, 0, 1)
        key = (code, int(axis))
        at = self._attrs.get(key) or self._encode(key, [(ATTR_AXIS, key[1])])
        return _rec_op(self, self._hv, code, (x,), at[0], at[1], 1)

    # ---- the tensor API shared with the oracle's back ends -------------------------------------------
    # ops without attributes skip op(): one Python frame per recorded op
    neg, abs, exp, log = _plain("neg", 1), _plain("abs", 1), _plain("exp", 1), _plain("log", 1)
    tanh, sqrt, rsqrt, recip = _plain("tanh", 1), _plain("sqrt", 1), _plain("rsqrt", 1), _plain("recip", 1)
    relu, gelu, square, sigmoid = _plain("relu", 1), _plain("gelu", 1), _plain("square", 1), _plain("sigmoid", 1)
    sub, mul, div = _plain("sub", 2), _plain("mul", 2), _plain("div", 2)
    maximum, minimum = _plain("maximum", 2), _plain("minimum", 2)
    relu_grad, gelu_grad = _plain("relu_grad", 2), _plain("gelu_grad", 2)    # (dy, x)

    add = None if _ltrec is None else _ltrec.PlainOp("add", OPCODES["add"], 2, 3, "alpha")   # add(a, b, alpha=None): a + alpha * b

    softmax, softmax_grad = _plain("softmax", 1), _plain("softmax_grad", 2)                 # (x), (dy, y)
    layer_norm_grad = _plain("layer_norm_grad", 5)                                            # (dy, x, gamma, mean, rstd)
    xent, xent_grad = _plain("xent", 2), _plain("xent_grad", 3)                               # (logits, labels[, scale])

    def cast(self, x, dtype):
        key = (_CAST, dtype)
        at = self._attrs.get(key) or self._encode(key, [(ATTR_DTYPE, DTYPES[dtype])])
        return _rec_op(self, self._hv, _CAST, (x,), at[0], at[1], 1)

    def expand(self, x, size): return self._dims_op(_EXPAND, x, size)
    def reshape(self, x, size): return self._dims_op(_RESHAPE, x, size)
    def permute(self, x, dims): return self._dims_op(_PERMUTE, x, dims)
    def sum(self, x, axis=None): return self._axis_op(_SUM, x, axis)
    def amax(self, x, axis=None): return self._axis_op(_AMAX, x, axis)
    def mean(self, x, axis=None): return self._axis_op(_MEAN, x, axis)

    def layer_norm(self, x, gamma, beta, eps=1e-5):
        key = (_LAYER_NORM, float(eps))
        at = self._attrs.get(key) or self._encode(key, [(ATTR_EPS, key[1])])
        return _rec_op(self, self._hv, _LAYER_NORM, (x, gamma, beta), at[0], at[1], 3)

    def matmul(self, a, b, trans_a=False, trans_b=False, dtype=None):
        key = (_MATMUL, bool(trans_a), bool(trans_b), dtype)
        at = self._attrs.get(key)
        if at is None:
            attrs = [(ATTR_TRANS_A, int(key[1])), (ATTR_TRANS_B, int(key[2]))]
            if dtype is not None:
                attrs.append((ATTR_DTYPE, DTYPES[dtype]))
            at = self._encode(key, attrs)
        return _rec_op(self, self._hv, _MATMUL, (a, b), at[0], at[1], 1)

    def narrow(self, x, axis, start, length):
        key = (_NARROW, int(axis), int(start), int(length))
        at = self._attrs.get(key) or self._encode(key, [(ATTR_AXIS, key[1]), (ATTR_START, key[2]), (ATTR_LENGTH, key[3])])
        return _rec_op(self, self._hv, _NARROW, (x,), at[0], at[1], 1)

    def slice_update(self, base, update, axis, start):
        key = (_SLICE_UPDATE, int(axis), int(start))
        at = self._attrs.get(key) or self._encode(key, [(ATTR_AXIS, key[1]), (ATTR_START, key[2])])
        return _rec_op(self, self._hv, _SLICE_UPDATE, (base, update), at[0], at[1], 1)

    # views (lt_view): tensors that share storage with their base as far as a program can tell
    def _view(self, code, x, attrs):
        key = ("view", code) + tuple(attrs)
        at = self._attrs.get(key) or self._encode(key, list(attrs))
        out = C.c_uint64()
        self._check(self._lib.lt_view(self._h, x.tid, code, C.cast(at[0], C.POINTER(lt_attr)), at[1], C.byref(out)))
        return Tensor(self, out.value)

    def view_permute(self, x, dims): return self._view(_PERMUTE, x, [(ATTR_DIM0 + i, int(d)) for i, d in enumerate(dims)])
    def view_reshape(self, x, size): return self._view(_RESHAPE, x, [(ATTR_DIM0 + i, int(d)) for i, d in enumerate(size)])

    def view_narrow(self, x, axis, start, length):
        return self._view(_NARROW, x, [(ATTR_AXIS, int(axis)), (ATTR_START, int(start)), (ATTR_LENGTH, int(length))])

    def assign(self, dst: Tensor, src: Tensor):
        _ltrec.assign(self._hv, dst, src)   # (what is known of src's type and shape becomes dst's)

    def release(self, t: Tensor):
        self._flush()
        self._check(self._lib.lt_release(self._h, t.tid))
        if t._keep is not None:
            self._kept.append(t._keep)
        t.ctx = None

    # ---- barrier, fetch, diagnostics -----------------------------------------------------------------------
    def barrier(self, blocking=True) -> BarrierInfo:
        info = BarrierInfo()
        _ltrec.barrier(self._hv, self._dead, blocking, C.addressof(info))   # (hands the dropped tensors over first)
        # Every launch that reads a dropped leaf's memory is now enqueued on the context's stream, which is
        # the stream the memory was allocated on: torch hands a freed block out again in stream order only.
        self._kept.clear()
        return info

    def barrier_static(self, blocking=True) -> BarrierInfo:
        """lt_barrier_static: the barrier that keeps its scratch in the library's own device array."""
        self._flush()
        info = BarrierInfo()
        self._check(self._lib.lt_barrier_static(self._h, 1 if blocking else 0, C.byref(info)))
        self._kept.clear()
        return info

    # ---- a captured step (section 7 of the paper: no tracing when the computation is the same) --
    def capture_step(self) -> "Step":
        """lt_step_capture: the step that the last barrier ran, to be run again with Step.replay."""
        h = C.c_void_p()
        self._check(self._lib.lt_step_capture(self._h, C.byref(h)))
        return Step(self, h)

    def rebind(self, t: Tensor, array):
        """lt_tensor_rebind: `t` now names the device memory of `array` (a torch tensor of the same
        dtype and shape on this device), keeping its id -- the next batch of a captured step."""
        a = array.contiguous()
        if tuple(a.shape) != tuple(t.shape):
            raise ValueError(f"rebind: shape {tuple(a.shape)} is not the tensor's {tuple(t.shape)}")
        self._check(self._lib.lt_tensor_rebind(self._h, t.tid, C.c_void_p(a.data_ptr())))
        if t._keep is not None:
            self._kept.append(t._keep)   # a step still in flight may read the old memory
        t._keep = a

    def fetch(self, t: Tensor) -> np.ndarray:
        """Blocking barrier if needed, then device-to-host copy.  bf16 comes back as float32."""
        self._flush()
        code = DTYPES[t.dtype]
        n = int(np.prod(t.shape, dtype=np.int64)) if t.shape else 1
        np_t = {0: np.float32, 1: np.uint16, 2: np.int32, 3: np.int64}[code]
        out = np.empty(n, dtype=np_t)
        before = self.stats().barriers if self._kept else 0
        self._check(self._lib.lt_fetch(self._h, t.tid, out.ctypes.data_as(C.c_void_p), out.nbytes))
        if self._kept and self.stats().barriers != before:   # the fetch of a pending tensor ran a barrier
            self._kept.clear()
        if code == 1:
            out = (out.astype(np.uint32) << 16).view(np.float32)
        return out.reshape(t.shape)

    def device_ptr(self, t: Tensor) -> int:
        p = C.c_void_p()
        self._check(self._lib.lt_device_ptr(self._h, t.tid, C.byref(p)))
        return p.value or 0

    def _dump(self, fn, binary=False):
        self._flush()
        n = C.c_size_t()
        self._check(fn(self._h, None, 0, C.byref(n)))
        buf = C.create_string_buffer(n.value + 1)
        self._check(fn(self._h, C.cast(buf, C.c_void_p) if binary else buf, n.value + 1, C.byref(n)))
        return buf.raw[:n.value] if binary else buf.value.decode()

    def dump_ir(self) -> str:
        return self._dump(self._lib.lt_dump_ir)

    def dump_plan(self) -> str:
        return self._dump(self._lib.lt_dump_plan)

    def dump_schedule(self) -> str:
        return self._dump(self._lib.lt_dump_schedule)

    def dump_key(self) -> bytes:
        return self._dump(self._lib.lt_dump_key, binary=True)

    def stats(self) -> Stats:
        self._flush()
        s = Stats()
        self._check(self._lib.lt_stats(self._h, C.byref(s)))
        return s

    def set_profiling(self, on: bool):
        self._check(self._lib.lt_set_profiling(self._h, 1 if on else 0))

    def set_streams(self, n: int) -> None:
        self._check(self._lib.lt_set_streams(self._h, int(n)))

    # ---- ops without a lowering (lt_set_fallback) ----------------------------------------------------
    def set_fallback(self, fn):
        """fn(opcode, inputs, attrs, outputs, run) -> None.  inputs / outputs: lists of dicts with keys
        ptr (device pointer; None for a host scalar), dtype, shape, scalar.  run False: set
        outputs[i]["dtype"] and ["shape"] (shape inference); run True: outputs have ptr set, compute
        them.  An exception raised by fn makes the op fail with LT_ERR_UNSUPPORTED.  None unregisters."""
        if fn is None:
            self._fallback_c = None
            self._check(self._lib.lt_set_fallback(self._h, C.cast(None, FALLBACK_FN), None))
            return

        def trampoline(user, opcode, ins, n_in, attrs, n_attr, outs, n_out, run, stream):
            try:
                def desc(d):
                    return {"ptr": d.dptr, "dtype": _DTYPE_NAMES[d.dtype], "shape": tuple(d.dims[i] for i in range(d.rank)),
                            "scalar": d.scalar if d.is_scalar else None}
                i_list = [desc(ins[i]) for i in range(n_in)]
                a_dict = {attrs[i].key: (attrs[i].v.f if attrs[i].is_float else attrs[i].v.i) for i in range(n_attr)}
                o_list = [desc(outs[i]) if run else {"ptr": None, "dtype": None, "shape": None} for i in range(n_out)]
                fn(opcode, i_list, a_dict, o_list, bool(run))
                if not run:
                    for i, o in enumerate(o_list):
                        outs[i].dtype = DTYPES[o["dtype"]]
                        outs[i].rank = len(o["shape"])
                        for k, dim in enumerate(o["shape"]):
                            outs[i].dims[k] = int(dim)
                return 0
            except Exception as e:      # an exception cannot cross the C boundary
                self._fallback_error = e
                return 1
        self._fallback_c = FALLBACK_FN(trampoline)       # (kept alive as long as it is registered)
        self._check(self._lib.lt_set_fallback(self._h, self._fallback_c, None))

    def custom_op(self, opcode, inputs, attrs=(), n_out=1):
        """Record (or, with a fallback registered, run) an op by number: opcodes from OP_CUSTOM up have no lowering."""
        self._flush()
        ts = [self._t(x) for x in inputs]           # (numbers become scalar tensors that live for the call)
        ids = (C.c_uint64 * len(ts))(*[t.tid for t in ts])
        arr = (lt_attr * max(1, len(attrs)))()
        for i, (k, val) in enumerate(attrs):
            arr[i].key = k
            if isinstance(val, float):
                arr[i].is_float, arr[i].v.f = 1, val
            else:
                arr[i].is_float, arr[i].v.i = 0, int(val)
        outs = (C.c_uint64 * n_out)()
        self._check(self._lib.lt_op(self._h, opcode, ids, len(inputs), arr, len(attrs), outs, n_out))
        res = [Tensor(self, outs[i]) for i in range(n_out)]
        return res[0] if n_out == 1 else tuple(res)

    def device_array(self, desc):
        """A fallback descriptor's device memory as a torch tensor (no copy): for fallbacks that call
        the eager framework's own op on the device."""
        torch = self._torch
        code = {"f32": ("<f4", torch.float32), "bf16": ("<i2", torch.bfloat16), "s32": ("<i4", torch.int32), "s64": ("<i8", torch.int64)}[desc["dtype"]]

        class _Mem:
            pass
        m = _Mem()
        m.__cuda_array_interface__ = {"shape": tuple(desc["shape"]), "typestr": code[0], "data": (int(desc["ptr"]), False),
                                      "version": 2, "strides": None}
        t = torch.as_tensor(m, device=f"cuda:{self.device}")
        return t.view(code[1]) if desc["dtype"] == "bf16" else t

    def set_quick_lookup(self, mode: int):
        """lt_set_quick_lookup: 0 off, 1 plans found by the record-time fingerprint, 2 the same with
        every hit checked against the canonical key."""
        self._check(self._lib.lt_set_quick_lookup(self._h, int(mode)))

    def set_graphs(self, on: bool):
        """lt_set_graphs: steps whose buffers sit where they sat before run as one HIP graph."""
        self._check(self._lib.lt_set_graphs(self._h, 1 if on else 0))

    def set_fusion(self, on: bool) -> None:
        self._check(self._lib.lt_set_fusion(self._h, 1 if on else 0))

    def last_launches(self):
        n = C.c_int()
        self._check(self._lib.lt_last_launches(self._h, None, 0, C.byref(n)))
        recs = (LaunchRecord * max(1, n.value))()
        self._check(self._lib.lt_last_launches(self._h, recs, n.value, C.byref(n)))
        return [{"kernel": r.kernel.decode(), "region": r.region, "ms": r.ms, "bytes": r.bytes, "flops": r.flops}
                for r in recs[:n.value]]
