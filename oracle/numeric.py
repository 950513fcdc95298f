"""Numeric oracle: an eager, op-by-op tensor evaluator on the CPU (NumPy).

TEST INFRASTRUCTURE -- see oracle/__init__.py.  Shares no code with the
C++/HIP library and is never imported by the product package.

What it computes.  Section 3 of the paper states the contract of a lazily
traced program: the compiled trace must be semantically equivalent to running
the recorded operations individually.  This module *is* "running the
operations individually": each call evaluates one tensor op immediately and
materialises its full result; nothing is fused, blocked or reordered.

Two precisions, selected at construction:

* ``Eager("f32")``: what an eager fp32/bf16 framework would store.  Values of
  dtype f32 live in float32 arrays; values of dtype bf16 live in float32
  arrays whose low 16 mantissa bits are zero (round-to-nearest-even at every
  op output).  Plain arithmetic (+ - * /) is done in float32; transcendental
  functions are evaluated in float64 and rounded once; every reduction and
  every matrix product accumulates in float64 and is rounded once.
* ``Eager("f64")``: the same ops in float64 with no intermediate rounding at
  all (bf16 rounding is skipped too).  This is the brute-force evaluator used
  on tiny graphs to bound the f32 evaluator itself.

The paper delegates all op semantics to the host framework (section 4 lists
ops by their framework names only), so the op definitions below are the
standard framework ones; each deviation-prone choice is stated at the op.
"""
from __future__ import annotations

import math

import numpy as np
from scipy.special import erf as _erf

F32, BF16, S32, S64 = "f32", "bf16", "s32", "s64"
_FLOAT = (F32, BF16)


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """float32 -> nearest bfloat16 value (ties to even), returned as float32.

    bfloat16 is the upper 16 bits of an IEEE binary32.  NaNs stay NaNs (a
    quiet bit is forced so that truncation cannot turn a NaN into infinity).
    """
    shape = np.shape(a)                       # (ascontiguousarray makes a rank-0 value rank 1)
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32).astype(np.uint64)
    lsb = (bits >> 16) & 1
    rounded = ((bits + 0x7FFF + lsb) >> 16) << 16
    nan = np.isnan(a)
    rounded = np.where(nan, (bits | 0x00400000) & 0xFFFF0000, rounded)
    return (rounded & 0xFFFFFFFF).astype(np.uint32).view(np.float32).reshape(shape)


class ETensor:
    """A materialised value: NumPy data plus the logical dtype tag."""

    __slots__ = ("data", "dtype", "shared")

    def __init__(self, data: np.ndarray, dtype: str):
        self.data = data
        self.dtype = dtype
        self.shared = False     # True: other tensors are views into (or the base of) this memory

    @property
    def shape(self):
        return tuple(self.data.shape)


class Eager:
    """Eager evaluator with the same method names as the lazy front end."""

    def __init__(self, precision: str = "f32"):
        assert precision in ("f32", "f64")
        self.exact = precision == "f64"
        self.ops_run = 0

    # ---- storage helpers -------------------------------------------------
    def _store(self, value: np.ndarray, dtype: str) -> ETensor:
        """Round a freshly computed value to what dtype would hold."""
        self.ops_run += 1
        if dtype in _FLOAT:
            if self.exact:
                return ETensor(np.asarray(value, dtype=np.float64), dtype)
            v = np.asarray(value).astype(np.float32)
            if dtype == BF16:
                v = round_to_bf16(v)
            return ETensor(v, dtype)
        np_t = np.int32 if dtype == S32 else np.int64
        return ETensor(np.asarray(value).astype(np_t), dtype)

    def _wide(self, t: ETensor) -> np.ndarray:
        return t.data.astype(np.float64)

    def _work(self, t: ETensor) -> np.ndarray:
        """Working precision for plain arithmetic: float32 (or float64 if exact)."""
        if t.dtype in _FLOAT:
            return t.data if not self.exact else t.data.astype(np.float64)
        return t.data.astype(np.float64 if self.exact else np.float32)

    # ---- factories -------------------------------------------------------
    def tensor(self, array, dtype: str | None = None, donatable: bool = False) -> ETensor:
        a = np.array(array)
        if dtype is None:
            dtype = {np.dtype(np.float32): F32, np.dtype(np.float64): F32,
                     np.dtype(np.int32): S32, np.dtype(np.int64): S64}[a.dtype]
        self.ops_run -= 1
        return self._store(a, dtype)

    def scalar(self, value, dtype: str = F32) -> ETensor:
        self.ops_run -= 1
        return self._store(np.array(value), dtype)

    def _t(self, x) -> ETensor:
        return x if isinstance(x, ETensor) else self.scalar(x)

    @staticmethod
    def _promote(a: ETensor, b: ETensor) -> str:
        """Result dtype of a binary op: a rank-0 operand adopts the other
        side's dtype; f32 with bf16 gives f32; an integer with a float gives
        the float."""
        if a.dtype == b.dtype:
            return a.dtype
        if a.data.ndim == 0 and b.data.ndim > 0:
            return b.dtype
        if b.data.ndim == 0 and a.data.ndim > 0:
            return a.dtype
        fa, fb = a.dtype in _FLOAT, b.dtype in _FLOAT
        if fa and fb:
            return F32
        if fa:
            return a.dtype
        if fb:
            return b.dtype
        return S64

    # ---- elementwise unary ----------------------------------------------
    def _unary_wide(self, x, fn):
        x = self._t(x)
        with np.errstate(all="ignore"):
            return self._store(fn(self._wide(x)), x.dtype)

    def neg(self, x):
        x = self._t(x)
        return self._store(-self._work(x), x.dtype)

    def abs(self, x):
        x = self._t(x)
        return self._store(np.abs(self._work(x)), x.dtype)

    def square(self, x):
        x = self._t(x)
        w = self._work(x)
        return self._store(w * w, x.dtype)

    def relu(self, x):
        x = self._t(x)
        w = self._work(x)
        return self._store(np.where(w > 0, w, np.zeros_like(w)), x.dtype)

    def exp(self, x):
        return self._unary_wide(x, np.exp)

    def log(self, x):
        return self._unary_wide(x, np.log)

    def tanh(self, x):
        return self._unary_wide(x, np.tanh)

    def sqrt(self, x):
        return self._unary_wide(x, np.sqrt)

    def rsqrt(self, x):
        return self._unary_wide(x, lambda v: 1.0 / np.sqrt(v))

    def recip(self, x):
        return self._unary_wide(x, lambda v: 1.0 / v)

    def sigmoid(self, x):
        return self._unary_wide(x, lambda v: 1.0 / (1.0 + np.exp(-v)))

    def gelu(self, x):
        """Exact GELU: x * Phi(x), Phi the standard normal CDF (erf form)."""
        return self._unary_wide(x, lambda v: 0.5 * v * (1.0 + _erf(v / math.sqrt(2.0))))

    def cast(self, x, dtype: str):
        x = self._t(x)
        if dtype in _FLOAT:
            return self._store(x.data, dtype)
        # float -> integer truncates toward zero, as a C cast does
        return self._store(np.trunc(x.data) if x.dtype in _FLOAT else x.data, dtype)

    # ---- elementwise binary (NumPy broadcasting) --------------------------
    def _binary(self, a, b, fn):
        a, b = self._t(a), self._t(b)
        dt = self._promote(a, b)
        with np.errstate(all="ignore"):
            return self._store(fn(self._work(a), self._work(b)), dt)

    def add(self, a, b, alpha=None):
        """a + b, or a + alpha*b when the framework-style scale is given
        (section 4.1 of the paper describes this scaled form of add)."""
        if alpha is None:
            return self._binary(a, b, lambda x, y: x + y)
        a, b, alpha = self._t(a), self._t(b), self._t(alpha)
        dt = self._promote(a, b)
        with np.errstate(all="ignore"):
            return self._store(self._work(a) + self._work(alpha) * self._work(b), dt)

    def sub(self, a, b):
        return self._binary(a, b, lambda x, y: x - y)

    def mul(self, a, b):
        return self._binary(a, b, lambda x, y: x * y)

    def div(self, a, b):
        return self._binary(a, b, lambda x, y: x / y)

    def maximum(self, a, b):
        return self._binary(a, b, np.maximum)

    def minimum(self, a, b):
        return self._binary(a, b, np.minimum)

    def relu_grad(self, dy, x):
        """dy where x > 0, else 0."""
        return self._binary(dy, x, lambda g, v: np.where(v > 0, g, np.zeros_like(g)))

    def gelu_grad(self, dy, x):
        """dy * d/dx[x Phi(x)] = dy * (Phi(x) + x phi(x))."""
        dy, x = self._t(dy), self._t(x)
        dt = self._promote(dy, x)
        v = self._wide(x)
        cdf = 0.5 * (1.0 + _erf(v / math.sqrt(2.0)))
        pdf = np.exp(-0.5 * v * v) / math.sqrt(2.0 * math.pi)
        return self._store(self._wide(dy) * (cdf + v * pdf), dt)

    # ---- shape ops --------------------------------------------------------
    def expand(self, x, size):
        x = self._t(x)
        return self._store(np.broadcast_to(x.data, tuple(size)).copy(), x.dtype)

    def reshape(self, x, size):
        x = self._t(x)
        return self._store(x.data.reshape(tuple(size)).copy(), x.dtype)

    def permute(self, x, dims):
        x = self._t(x)
        return self._store(np.transpose(x.data, tuple(dims)).copy(), x.dtype)

    def narrow(self, x, axis, start, length):
        """The window [start, start + length) along one axis, as a copy."""
        x = self._t(x)
        idx = [slice(None)] * x.data.ndim
        idx[axis] = slice(start, start + length)
        return self._store(x.data[tuple(idx)].copy(), x.dtype)

    def slice_update(self, base, update, axis, start):
        """base with the window that starts at `start` along `axis` replaced by update."""
        base, update = self._t(base), self._t(update)
        out = base.data.copy()
        idx = [slice(None)] * out.ndim
        idx[axis] = slice(start, start + update.data.shape[axis])
        out[tuple(idx)] = update.data
        return self._store(out, base.dtype)

    # ---- views: tensors that share their base's storage (section 4.4 of the paper) ----------
    # The plain definition: a view IS the base's memory seen through other strides, so the view
    # is a NumPy view, and an in-place update of either tensor writes into that memory.
    def _share(self, x, view_data):
        x = self._t(x)
        x.shared = True
        v = ETensor(view_data, x.dtype)
        v.shared = True
        return v

    def view_permute(self, x, dims):
        return self._share(x, np.transpose(self._t(x).data, tuple(dims)))

    def view_reshape(self, x, size):
        x = self._t(x)
        v = x.data.reshape(tuple(size))
        assert np.shares_memory(v, x.data), "a reshape that needs a copy is not a view"
        return self._share(x, v)

    def view_narrow(self, x, axis, start, length):
        x = self._t(x)
        idx = [slice(None)] * x.data.ndim
        idx[axis] = slice(start, start + length)
        return self._share(x, x.data[tuple(idx)])

    # ---- reductions -------------------------------------------------------
    def _reduce(self, x, axis, fn):
        x = self._t(x)
        ax = None if axis is None else int(axis)
        return self._store(fn(self._wide(x), axis=ax), x.dtype)

    def sum(self, x, axis=None):
        return self._reduce(x, axis, np.sum)

    def amax(self, x, axis=None):
        return self._reduce(x, axis, np.max)

    def mean(self, x, axis=None):
        return self._reduce(x, axis, np.mean)

    # ---- row ops (last axis) ----------------------------------------------
    def softmax(self, x):
        x = self._t(x)
        v = self._wide(x)
        e = np.exp(v - v.max(axis=-1, keepdims=True))
        return self._store(e / e.sum(axis=-1, keepdims=True), x.dtype)

    def softmax_grad(self, dy, y):
        """dx = y * (dy - sum_j dy_j y_j), the Jacobian-vector product of softmax."""
        dy, y = self._t(dy), self._t(y)
        g, p = self._wide(dy), self._wide(y)
        return self._store(p * (g - (g * p).sum(axis=-1, keepdims=True)), y.dtype)

    def layer_norm(self, x, gamma, beta, eps: float = 1e-5):
        """Returns (y, mean, rstd); biased variance over the last axis."""
        x, gamma, beta = self._t(x), self._t(gamma), self._t(beta)
        v = self._wide(x)
        mu = v.mean(axis=-1, keepdims=True)
        var = ((v - mu) ** 2).mean(axis=-1, keepdims=True)
        rstd = 1.0 / np.sqrt(var + eps)
        y = (v - mu) * rstd * self._wide(gamma) + self._wide(beta)
        return (self._store(y, x.dtype), self._store(mu[..., 0], F32),
                self._store(rstd[..., 0], F32))

    def layer_norm_grad(self, dy, x, gamma, mean, rstd):
        """dx of layer_norm given the saved row statistics."""
        dy, x, gamma = self._t(dy), self._t(x), self._t(gamma)
        mu = self._wide(mean)[..., None]
        rs = self._wide(rstd)[..., None]
        xhat = (self._wide(x) - mu) * rs
        g = self._wide(dy) * self._wide(gamma)
        dx = rs * (g - g.mean(axis=-1, keepdims=True)
                   - xhat * (g * xhat).mean(axis=-1, keepdims=True))
        return self._store(dx, x.dtype)

    def xent(self, logits, labels):
        """Per-row softmax cross-entropy: logsumexp(row) - row[label]."""
        logits, labels = self._t(logits), self._t(labels)
        v = self._wide(logits)
        m = v.max(axis=-1, keepdims=True)
        lse = np.log(np.exp(v - m).sum(axis=-1)) + m[..., 0]
        picked = np.take_along_axis(v, labels.data.astype(np.int64)[..., None], axis=-1)[..., 0]
        return self._store(lse - picked, F32)

    def xent_grad(self, logits, labels, scale):
        """(softmax(row) - onehot(label)) * scale."""
        logits, labels, scale = self._t(logits), self._t(labels), self._t(scale)
        v = self._wide(logits)
        e = np.exp(v - v.max(axis=-1, keepdims=True))
        p = e / e.sum(axis=-1, keepdims=True)
        onehot = np.zeros_like(p)
        np.put_along_axis(onehot, labels.data.astype(np.int64)[..., None], 1.0, axis=-1)
        return self._store((p - onehot) * self._wide(scale), logits.dtype)

    # ---- contraction --------------------------------------------------------
    def matmul(self, a, b, trans_a: bool = False, trans_b: bool = False, dtype: str | None = None):
        """Matrix product over the last two axes, float64 accumulation.
        Leading axes of a and b must match, or b is a plain matrix."""
        a, b = self._t(a), self._t(b)
        A, B = self._wide(a), self._wide(b)
        if trans_a:
            A = np.swapaxes(A, -1, -2)
        if trans_b:
            B = np.swapaxes(B, -1, -2)
        out_dt = dtype if dtype is not None else (a.dtype if a.dtype == b.dtype else F32)
        return self._store(np.matmul(A, B), out_dt)

    # ---- mutation, barrier, fetch -------------------------------------------
    def assign(self, dst: ETensor, src: ETensor) -> None:
        """In-place update = rebind the destination to the new value; a tensor whose memory is
        shared with views (or that is a view) is written in place instead, so that every tensor on
        that memory sees the update."""
        if dst.shared:
            assert dst.dtype == src.dtype and dst.data.shape == src.data.shape
            dst.data[...] = src.data
            return
        # a copy: the destination must not see later in-place writes to the source's memory (the
        # source may become the base of a view afterwards) -- an in-place update is a substitution
        # of one tensor's value, never of another's (sections 4.3 and 4.4 of the paper)
        dst.data, dst.dtype = src.data.copy(), src.dtype

    def barrier(self, blocking: bool = True) -> None:
        return None

    def fetch(self, t: ETensor) -> np.ndarray:
        return np.array(t.data)
