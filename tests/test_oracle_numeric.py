"""Pins for the numeric oracle (no GPU): closed forms, invariants, float64
brute force and finite differences.  A dropped term, a wrong sign or index or
a transposed operand in oracle/numeric.py fails at least one of these."""
import math

import numpy as np
import pytest

from oracle.numeric import Eager, round_to_bf16
from workloads import programs
from workloads.inputs import C4_HYPER, c1_inputs, c2_inputs


def rng(seed=0):
    return np.random.Generator(np.random.PCG64(seed))


def f(E, t):
    return E.fetch(t).astype(np.float64)


# ---- rounding ------------------------------------------------------------------
def test_bf16_round_to_nearest_even_bit_patterns():
    def r(bits):
        return round_to_bf16(np.array([bits], dtype=np.uint32).view(np.float32)).view(np.uint32)[0]
    assert r(0x3F800000) == 0x3F800000          # 1.0 exact
    assert r(0x3F808000) == 0x3F800000          # tie -> even (down)
    assert r(0x3F818000) == 0x3F820000          # tie -> even (up)
    assert r(0x3F808001) == 0x3F810000          # just above tie -> up
    assert r(0x3F807FFF) == 0x3F800000          # just below tie -> down
    assert r(0x7F7FFFFF) == 0x7F800000          # overflow to +inf
    assert np.isnan(round_to_bf16(np.array([np.nan], np.float32)))[0]
    assert r(0xBF808000) == 0xBF800000          # sign kept


# ---- elementwise: special values and textbook identities ----------------------------
def test_elementwise_special_values():
    E = Eager()
    z = E.tensor(np.zeros(3, np.float32))
    assert np.all(f(E, E.tanh(z)) == 0) and np.all(f(E, E.exp(z)) == 1) and np.all(f(E, E.gelu(z)) == 0)
    x = E.tensor(np.array([-np.inf, np.inf, np.nan], np.float32))
    assert list(f(E, E.tanh(x))[:2]) == [-1.0, 1.0] and np.isnan(f(E, E.tanh(x))[2])
    assert list(f(E, E.relu(E.tensor(np.array([-2.0, 0.0, 3.0], np.float32))))) == [0.0, 0.0, 3.0]
    assert list(f(E, E.relu_grad(E.tensor(np.array([5.0, 5.0, 5.0], np.float32)),
                                 E.tensor(np.array([-1.0, 0.0, 2.0], np.float32))))) == [0.0, 0.0, 5.0]


def test_elementwise_against_math_module():
    E = Eager("f64")
    xs = np.linspace(-3, 3, 25)
    x = E.tensor(xs.astype(np.float32))
    xs = xs.astype(np.float32).astype(np.float64)
    ref = lambda fn: np.array([fn(v) for v in xs])
    assert np.allclose(f(E, E.gelu(x)), ref(lambda v: 0.5 * v * (1 + math.erf(v / math.sqrt(2)))), rtol=1e-14)
    assert np.allclose(f(E, E.sigmoid(x)), ref(lambda v: 1 / (1 + math.exp(-v))), rtol=1e-14)
    nz = xs != 0
    assert np.allclose((f(E, E.rsqrt(E.square(x))) * np.abs(xs))[nz], 1.0, rtol=1e-12)
    # gelu_grad against a central difference of gelu
    h = 1e-6
    g = lambda v: 0.5 * v * (1 + math.erf(v / math.sqrt(2)))
    fd = ref(lambda v: (g(v + h) - g(v - h)) / (2 * h))
    assert np.allclose(f(E, E.gelu_grad(E.tensor(np.ones(25, np.float32)), x)), fd, atol=1e-8)


def test_add_alpha_and_broadcast_and_promotion():
    E = Eager()
    a = E.tensor(np.arange(6, dtype=np.float32).reshape(2, 3))
    b = E.tensor(np.array([10, 20, 30], np.float32))
    assert np.array_equal(f(E, E.add(a, b, alpha=0.5)), np.arange(6).reshape(2, 3) + 0.5 * np.array([10, 20, 30]))
    assert np.array_equal(f(E, E.sub(b, a)), np.array([10, 20, 30]) - np.arange(6).reshape(2, 3))
    assert np.array_equal(f(E, E.div(a, 2.0)), np.arange(6).reshape(2, 3) / 2)
    h = E.cast(a, "bf16")
    assert E.mul(h, h).dtype == "bf16" and E.mul(h, a).dtype == "f32" and E.mul(h, 3.0).dtype == "bf16"


# ---- reductions -------------------------------------------------------------------
def test_reductions_closed_forms():
    E = Eager()
    ones = E.tensor(np.ones((37, 53), np.float32))
    assert f(E, E.sum(ones)) == 37 * 53
    assert np.array_equal(f(E, E.sum(ones, axis=1)), np.full(37, 53.0))
    assert np.array_equal(f(E, E.sum(ones, axis=0)), np.full(53, 37.0))
    perm = rng(1).permutation(1000).astype(np.float32)
    assert f(E, E.amax(E.tensor(perm))) == 999
    m = E.tensor(np.arange(12, dtype=np.float32).reshape(3, 4))
    assert np.array_equal(f(E, E.mean(m, axis=-1)), [1.5, 5.5, 9.5])
    assert np.array_equal(f(E, E.amax(m, axis=0)), [8, 9, 10, 11])


def test_c1_trace_closed_structure():
    """max|out| is exactly 1 (x / |x| is exact in IEEE arithmetic) and the
    trace equals a directly typed float64 formula."""
    inp = c1_inputs(64, 48)
    E = Eager()
    out = f(E, programs.c1_trace(E, *(E.tensor(inp[k]) for k in ("x", "y", "bias"))))
    assert np.max(np.abs(out)) == 1.0
    x, y, b = (inp[k].astype(np.float64) for k in ("x", "y", "bias"))
    s = (np.tanh(x * y + b) * np.exp(-x * x) + 0.5 * y).sum(axis=1)
    assert np.allclose(out, s / np.abs(s).max(), rtol=2e-6, atol=2e-6)


# ---- softmax / layer norm / cross entropy ---------------------------------------------
def test_softmax_invariants():
    E = Eager()
    x = rng(2).standard_normal((5, 7)).astype(np.float32) * 3
    p = f(E, E.softmax(E.tensor(x)))
    assert np.allclose(p.sum(axis=1), 1.0, atol=1e-6)
    assert np.allclose(f(E, E.softmax(E.tensor(x + 11.0))), p, atol=1e-6)       # shift invariance
    e = np.exp(x.astype(np.float64))
    assert np.allclose(p, e / e.sum(axis=1, keepdims=True), atol=1e-7)


def test_layer_norm_invariants():
    E = Eager()
    x = rng(3).standard_normal((4, 64)).astype(np.float32) * 2 + 1
    ones, zeros = E.tensor(np.ones(64, np.float32)), E.tensor(np.zeros(64, np.float32))
    y, mu, rstd = E.layer_norm(E.tensor(x), ones, zeros, eps=1e-5)
    y = f(E, y)
    assert np.allclose(y.mean(axis=1), 0, atol=1e-6)
    var = x.astype(np.float64).var(axis=1)
    assert np.allclose(y.var(axis=1), var / (var + 1e-5), rtol=1e-5)
    assert np.allclose(f(E, mu), x.astype(np.float64).mean(axis=1), atol=1e-6)
    assert np.allclose(f(E, rstd), 1 / np.sqrt(var + 1e-5), rtol=1e-6)
    beta = E.tensor(np.arange(64, dtype=np.float32))
    const = E.tensor(np.full((2, 64), 3.25, np.float32))
    assert np.allclose(f(E, E.layer_norm(const, ones, beta)[0]), np.arange(64), atol=1e-6)  # constant row -> beta


def test_cross_entropy_closed_forms():
    E = Eager()
    logits = E.tensor(np.full((6, 10), 0.37, np.float32))
    labels = E.tensor(np.arange(6, dtype=np.int32))
    assert np.allclose(f(E, E.xent(logits, labels)), math.log(10), atol=1e-6)
    x = rng(4).standard_normal((3, 4)).astype(np.float32)
    lab = np.array([1, 3, 0], np.int32)
    g = f(E, E.xent_grad(E.tensor(x), E.tensor(lab), 1.0))
    assert np.allclose(g.sum(axis=1), 0, atol=1e-6)
    # finite differences of the per-row loss, in float64
    E64 = Eager("f64")
    h = 1e-5
    for r in range(3):
        for c in range(4):
            xp, xm = x.astype(np.float64).copy(), x.astype(np.float64).copy()
            xp[r, c] += h
            xm[r, c] -= h
            lp = E64.fetch(E64.xent(E64.tensor(xp), E64.tensor(lab)))[r]
            lm = E64.fetch(E64.xent(E64.tensor(xm), E64.tensor(lab)))[r]
            assert abs((lp - lm) / (2 * h) - g[r, c]) < 1e-6


def _fd(fun, x, h=1e-5):
    g = np.zeros_like(x)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        xp, xm = x.copy(), x.copy()
        xp[i] += h
        xm[i] -= h
        g[i] = (fun(xp) - fun(xm)) / (2 * h)
    return g


def test_softmax_and_layer_norm_backward_by_finite_differences():
    E = Eager("f64")
    r = rng(5)
    x = r.standard_normal((3, 6))
    w = r.standard_normal((3, 6))          # upstream gradient
    p = E.softmax(E.tensor(x))
    dx = E.fetch(E.softmax_grad(E.tensor(w), p))
    fd = _fd(lambda v: float((E.fetch(E.softmax(E.tensor(v))) * w).sum()), x)
    assert np.allclose(dx, fd, atol=1e-8)
    gamma, beta = r.standard_normal(6), r.standard_normal(6)
    y, mu, rstd = E.layer_norm(E.tensor(x), E.tensor(gamma), E.tensor(beta))
    dx = E.fetch(E.layer_norm_grad(E.tensor(w), E.tensor(x), E.tensor(gamma), mu, rstd))
    fd = _fd(lambda v: float((E.fetch(E.layer_norm(E.tensor(v), E.tensor(gamma), E.tensor(beta))[0]) * w).sum()), x)
    assert np.allclose(dx, fd, atol=1e-6)


# ---- matmul ---------------------------------------------------------------------------
def test_matmul_pins():
    E = Eager()
    a = rng(6).standard_normal((5, 7)).astype(np.float32)
    A = E.tensor(a)
    assert np.array_equal(f(E, E.matmul(A, E.tensor(np.eye(7, dtype=np.float32)))), a)
    assert np.all(f(E, E.matmul(E.tensor(np.ones((4, 200), np.float32)), E.tensor(np.ones((200, 3), np.float32)))) == 200)
    b = rng(7).standard_normal((7, 4)).astype(np.float32)
    brute = np.zeros((5, 4))
    for i in range(5):
        for j in range(4):
            for k in range(7):
                brute[i, j] += float(a[i, k]) * float(b[k, j])
    assert np.allclose(f(E, E.matmul(A, E.tensor(b))), brute, rtol=1e-6)
    # transposed variants against explicit transposes; a non-symmetric case catches swapped flags
    assert np.array_equal(f(E, E.matmul(E.tensor(a.T.copy()), E.tensor(b), trans_a=True)), f(E, E.matmul(A, E.tensor(b))))
    assert np.array_equal(f(E, E.matmul(A, E.tensor(b.T.copy()), trans_b=True)), f(E, E.matmul(A, E.tensor(b))))
    # batched, and bf16 output rounding
    A3 = rng(8).standard_normal((2, 3, 5, 7)).astype(np.float32)
    B3 = rng(9).standard_normal((2, 3, 7, 4)).astype(np.float32)
    out = f(E, E.matmul(E.tensor(A3), E.tensor(B3)))
    assert np.allclose(out[1, 2], A3[1, 2].astype(np.float64) @ B3[1, 2].astype(np.float64), rtol=1e-6)
    hb = E.matmul(E.cast(A, "bf16"), E.cast(E.tensor(b), "bf16"))
    assert hb.dtype == "bf16" and np.array_equal(round_to_bf16(hb.data), hb.data)


# ---- optimiser closed forms ----------------------------------------------------------------
def test_adam_first_step_closed_form_and_clipping():
    """m = v = 0 and t = 1  =>  delta p = -lr * g / (|g| + eps)."""
    E = Eager("f64")
    g = rng(10).standard_normal(50) * 0.1
    p0 = rng(11).standard_normal(50)
    p, gt = E.tensor(p0), E.tensor(g)
    m, v = E.tensor(np.zeros(50)), E.tensor(np.zeros(50))
    programs.adam_update(E, p, gt, m, v, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, t=1)
    assert np.allclose(E.fetch(p) - p0, -1e-3 * g / (np.abs(g) + 1e-8), rtol=1e-9)
    assert np.allclose(E.fetch(m), 0.1 * g) and np.allclose(E.fetch(v), 0.001 * g * g)
    # clipping: the scaled gradient has norm max_norm when ||g|| > max_norm, and is unchanged otherwise
    for scale, clipped in ((10.0, True), (1e-3, False)):
        gg = g * scale
        gn = E.sqrt(E.sum(E.square(E.tensor(gg))))
        c = E.fetch(E.minimum(1.0, E.div(1.0, E.add(gn, 1e-6))))
        if clipped:
            assert abs(np.linalg.norm(c * gg) - 1.0) < 1e-5
        else:
            assert c == 1.0


def test_mlp_step_properties():
    """He-init loss is on the ln(10) scale; on a fixed batch SGD with lr 0.01
    does not increase the loss; analytic gradients match finite differences."""
    inp = c2_inputs(batch=16, dims=(12, 8, 8, 10), steps=1)
    E = Eager("f64")
    params = [E.tensor(inp[k].astype(np.float64)) for k in ("W1", "b1", "W2", "b2", "W3", "b3")]
    X, lab = E.tensor(inp["X"][0].astype(np.float64)), E.tensor(inp["labels"][0])
    losses = [float(E.fetch(programs.c2_step(E, X, lab, params, 0.01))) for _ in range(5)]
    assert 0.5 * math.log(10) < losses[0] < 3 * math.log(10)
    assert all(b <= a for a, b in zip(losses, losses[1:]))
    # gradient check: W2 update equals -lr * dLoss/dW2 by central differences
    params = [E.tensor(inp[k].astype(np.float64)) for k in ("W1", "b1", "W2", "b2", "W3", "b3")]
    before = [E.fetch(q).copy() for q in params]

    def loss_at(idx, arr):
        ps = [E.tensor(b) for b in before]
        ps[idx] = E.tensor(arr)
        h = X
        for i in range(3):
            h = E.add(E.matmul(h, ps[2 * i]), ps[2 * i + 1])
            if i < 2:
                h = E.relu(h)
        return float(E.fetch(E.mean(E.xent(h, lab))))
    programs.c2_step(E, X, lab, params, 0.01)
    for idx in (2, 3, 4):
        fd = _fd(lambda a: loss_at(idx, a), before[idx], h=1e-6)
        assert np.allclose((before[idx] - E.fetch(params[idx])) / 0.01, fd, atol=1e-6)


def test_f32_evaluator_close_to_f64_brute_force():
    inp = c1_inputs(8, 8)
    outs = []
    for prec in ("f32", "f64"):
        E = Eager(prec)
        outs.append(f(E, programs.c1_trace(E, *(E.tensor(inp[k]) for k in ("x", "y", "bias")))))
    assert np.max(np.abs(outs[0] - outs[1])) <= 1e-6 * np.max(np.abs(outs[1]))


def test_in_place_is_substitution():
    E = Eager()
    a = E.tensor(np.ones(4, np.float32))
    b = E.add(a, 2.0)
    E.assign(a, E.add(a, 1.0))
    assert np.all(f(E, a) == 2) and np.all(f(E, a) == 2) and np.all(f(E, b) == 3)


# ---- the remaining unary / binary / shape ops ---------------------------------------------
def test_log_recip_sqrt_neg_abs_closed_forms():
    E = Eager("f64")
    xs = np.array([0.125, 0.5, 1.0, 2.0, 3.0, 10.0, 1e-3, 12345.0], np.float32)
    x = E.tensor(xs)
    xs = xs.astype(np.float64)
    assert np.allclose(f(E, E.log(x)), [math.log(v) for v in xs], rtol=1e-15, atol=0)
    assert np.allclose(f(E, E.log(E.exp(E.tensor(np.linspace(-5, 5, 21).astype(np.float32))))), np.linspace(-5, 5, 21), atol=1e-14)
    assert f(E, E.log(E.tensor(np.array([1.0], np.float32))))[0] == 0.0
    assert np.allclose(f(E, E.mul(x, E.recip(x))), 1.0, rtol=1e-15)
    assert np.array_equal(f(E, E.recip(E.tensor(np.array([2.0, -4.0, 0.5], np.float32)))), [0.5, -0.25, 2.0])
    assert np.array_equal(f(E, E.sqrt(E.tensor(np.array([0.0, 4.0, 9.0, 0.25], np.float32)))), [0.0, 2.0, 3.0, 0.5])
    assert np.array_equal(f(E, E.neg(E.tensor(np.array([1.5, -2.0, 0.0], np.float32)))), [-1.5, 2.0, 0.0])
    assert np.array_equal(f(E, E.abs(E.tensor(np.array([1.5, -2.0, -0.0], np.float32)))), [1.5, 2.0, 0.0])
    assert np.array_equal(f(E, E.square(E.tensor(np.array([1.5, -2.0], np.float32)))), [2.25, 4.0])
    # the f32 evaluator rounds once: special values
    F = Eager()
    with np.errstate(all="ignore"):
        sp = F.fetch(F.log(F.tensor(np.array([0.0, -1.0, np.inf], np.float32))))
        rc = F.fetch(F.recip(F.tensor(np.array([0.0, np.inf], np.float32))))
    assert sp[0] == -np.inf and np.isnan(sp[1]) and sp[2] == np.inf
    assert rc[0] == np.inf and rc[1] == 0.0


def test_maximum_minimum_are_elementwise_and_ordered():
    E = Eager()
    p = rng(2).permutation(64).astype(np.float32)
    q = p[::-1].copy()
    hi, lo = f(E, E.maximum(E.tensor(p), E.tensor(q))), f(E, E.minimum(E.tensor(p), E.tensor(q)))
    assert np.array_equal(hi, [max(a, b) for a, b in zip(p, q)])          # typed out pair by pair
    assert np.array_equal(lo, [min(a, b) for a, b in zip(p, q)])
    assert np.array_equal(hi + lo, p + q) and np.all(hi >= lo)
    assert np.array_equal(f(E, E.maximum(E.tensor(p), 31.5)), np.where(p > 31.5, p, 31.5))    # rank-0 operand
    assert np.array_equal(f(E, E.minimum(1.0, E.tensor(np.array([0.25, 4.0], np.float32)))), [0.25, 1.0])


def test_shape_ops_against_hand_typed_index_maps():
    """expand / reshape / permute on a 2 x 3 x 4 iota, checked element by element against the index
    arithmetic of a row-major tensor written out here."""
    E = Eager()
    iota = np.arange(24, dtype=np.float32).reshape(2, 3, 4)
    t = E.tensor(iota)
    p = f(E, E.permute(t, (1, 2, 0)))                       # out[j, k, i] = in[i, j, k]
    assert p.shape == (3, 4, 2)
    for i in range(2):
        for j in range(3):
            for k in range(4):
                assert p[j, k, i] == 12 * i + 4 * j + k
    back = f(E, E.permute(E.permute(t, (1, 2, 0)), (2, 0, 1)))   # the inverse permutation of figure 3
    assert np.array_equal(back, iota)
    r = f(E, E.reshape(t, (6, 4)))                          # flat order is kept
    assert r.shape == (6, 4)
    for a in range(6):
        for b in range(4):
            assert r[a, b] == 4 * a + b
    assert np.array_equal(f(E, E.reshape(t, (4, 6)))[3], [18, 19, 20, 21, 22, 23])
    v = E.tensor(np.array([10.0, 20.0, 30.0, 40.0], np.float32))
    e = f(E, E.expand(v, (2, 3, 4)))                        # trailing axes align, leading ones repeat
    assert e.shape == (2, 3, 4)
    for i in range(2):
        for j in range(3):
            assert list(e[i, j]) == [10.0, 20.0, 30.0, 40.0]
    col = f(E, E.expand(E.tensor(np.array([[1.0], [2.0], [3.0]], np.float32)), (3, 4)))
    assert [list(row) for row in col] == [[1.0] * 4, [2.0] * 4, [3.0] * 4]
    assert np.array_equal(f(E, E.expand(E.scalar(7.0), (2, 2))), [[7.0, 7.0], [7.0, 7.0]])
    assert E.permute(E.cast(t, "bf16"), (2, 1, 0)).dtype == "bf16" and E.reshape(t, (24,)).dtype == "f32"


def test_cast_to_integer_truncates_towards_zero_and_back():
    E = Eager()
    x = E.tensor(np.array([2.7, -2.7, 0.5, -0.5, 3.0, -1e6 - 0.25], np.float32))
    i32 = E.cast(x, "s32")
    assert i32.dtype == "s32" and E.fetch(i32).dtype == np.int32
    assert list(E.fetch(i32)) == [2, -2, 0, 0, 3, -1000000]
    i64 = E.cast(x, "s64")
    assert E.fetch(i64).dtype == np.int64 and list(E.fetch(i64)) == [2, -2, 0, 0, 3, -1000000]
    assert list(E.fetch(E.cast(i32, "f32"))) == [2.0, -2.0, 0.0, 0.0, 3.0, -1000000.0]
    h = E.cast(E.tensor(np.array([1.00390625, 257.0], np.float32)), "bf16")      # 1 + 2^-8: a tie, to even
    assert list(E.fetch(h)) == [1.0, 256.0]


# ---- the transformer layer's hand-written backward pass ---------------------------------------
def test_c3_step_gradients_by_finite_differences():
    """workloads.programs.c3_step spells out its own backward pass.  In float64, on a tiny encoder
    (d = 8, seq 4, 2 heads, FFN 16, batch 2), dx and all sixteen parameter gradients (read from the
    first Adam moment: with m = 0 and beta1 = 0.9 the new moment is 0.1 g) must equal central
    finite differences of  L = sum(y * dy)  with respect to x and to every parameter."""
    from workloads.inputs import c3_inputs
    bsz, seq, d, ffn, heads = 2, 4, 8, 16, 2
    inp = c3_inputs(bsz, seq, d, ffn, seed_extra=3)
    r = rng(11)
    keys = programs.C3_WEIGHTS + programs.C3_VECTORS
    vals = {k: inp[k].astype(np.float64) for k in keys}
    for k in keys:   # biases and gains away from their trivial initial values, weights large enough to matter
        vals[k] = vals[k] * (10.0 if k in programs.C3_WEIGHTS else 1.0) + 0.3 * r.standard_normal(vals[k].shape)
    x0, dy0 = inp["x"].astype(np.float64), inp["dy"].astype(np.float64)

    def run(x, params):
        E = Eager("f64")
        P = {k: E.tensor(params[k].copy(), dtype="f32") for k in keys}
        M = {k: E.tensor(np.zeros_like(params[k]), dtype="f32") for k in keys}
        V = {k: E.tensor(np.zeros_like(params[k]), dtype="f32") for k in keys}
        y, dx = programs.c3_step(E, E.tensor(x, dtype="f32"), E.tensor(dy0, dtype="f32"), P, M, V, heads)
        return f(E, y).reshape(x.shape), f(E, dx).reshape(x.shape), {k: f(E, M[k]) / 0.1 for k in keys}

    y, dx, grads = run(x0, vals)
    loss = lambda x, params: float(np.sum(run(x, params)[0] * dy0))
    h = 1e-5

    def fd(target, idx, is_x):
        def at(delta):
            if is_x:
                xx = x0.copy(); xx[idx] += delta
                return loss(xx, vals)
            pp = dict(vals); pp[target] = vals[target].copy(); pp[target][idx] += delta
            return loss(x0, pp)
        return (at(h) - at(-h)) / (2 * h)

    scale = max(np.max(np.abs(dx)), 1e-30)
    for _ in range(6):
        idx = tuple(int(r.integers(0, n)) for n in x0.shape)
        assert abs(fd(None, idx, True) - dx[idx]) <= 1e-6 * scale, ("dx", idx)
    for k in keys:
        g = grads[k]
        scale = max(np.max(np.abs(g)), 1e-30)
        picks = [tuple(int(r.integers(0, n)) for n in g.shape) for _ in range(3)]
        for idx in picks:
            num = fd(k, idx, False)
            if k == "bk":      # softmax ignores a shift of its row: the key bias has no gradient at all
                assert abs(num) <= 1e-7 and abs(g[idx]) <= 1e-9 * max(np.max(np.abs(grads["bq"])), 1e-30) + 1e-12
            else:
                assert abs(num - g[idx]) <= 1e-6 * scale, (k, idx, num, g[idx])


def test_views_share_storage_and_window_ops():
    """narrow / slice_update against hand-typed windows, and the shared-storage semantics of views:
    an in-place update through any view shows in the base and in every other view."""
    E = Eager()
    iota = np.arange(24, dtype=np.float32).reshape(2, 3, 4)
    x = E.tensor(iota.copy())
    assert np.array_equal(f(E, E.narrow(x, 1, 1, 2)), [[[4, 5, 6, 7], [8, 9, 10, 11]], [[16, 17, 18, 19], [20, 21, 22, 23]]])
    assert np.array_equal(f(E, E.narrow(x, 2, 3, 1))[..., 0], [[3, 7, 11], [15, 19, 23]])
    up = f(E, E.slice_update(x, E.tensor(np.full((2, 1, 4), -1.0, np.float32)), 1, 2))
    assert np.array_equal(up[:, 2], -np.ones((2, 4))) and np.array_equal(up[:, :2], iota[:, :2])
    assert np.array_equal(f(E, x), iota)                         # functional forms leave their operands alone
    v = E.view_permute(x, (1, 2, 0))                             # figure 3's view
    E.assign(v, E.add(v, 42.0))
    assert np.array_equal(f(E, x), iota + 42) and f(E, v)[1, 2, 0] == iota[0, 1, 2] + 42
    w = E.view_narrow(x, 1, 1, 2)
    E.assign(w, E.mul(w, 2.0))
    want = iota + 42
    want[:, 1:3] *= 2
    assert np.array_equal(f(E, x), want) and np.array_equal(f(E, v), want.transpose(1, 2, 0))   # the sibling view sees it
    r = E.view_reshape(x, (6, 4))
    E.assign(x, E.neg(x))                                        # updating the base shows in its views
    assert np.array_equal(f(E, r), -want.reshape(6, 4)) and np.array_equal(f(E, w), -want[:, 1:3])


def test_assign_gives_the_destination_a_value_of_its_own():
    """Sections 4.3 / 4.4: an in-place update substitutes ONE tensor's value.  After `b <- a`, an
    update of a through a view (which writes a's memory) must leave b alone -- values typed by hand."""
    E = Eager()
    a = E.tensor(np.array([[1.0, 2.0], [3.0, 4.0]], np.float32))
    b = E.tensor(np.zeros((2, 2), np.float32))
    c = E.tensor(np.array([[10.0, 20.0], [30.0, 40.0]], np.float32))
    E.assign(b, a)                                    # b = [[1, 2], [3, 4]]
    v = E.view_permute(a, (1, 0))                     # a view of a: a is written in place from now on
    E.assign(v, c)                                    # a = c^T
    assert np.array_equal(E.fetch(a), [[10.0, 30.0], [20.0, 40.0]])
    assert np.array_equal(E.fetch(b), [[1.0, 2.0], [3.0, 4.0]])
    # and the other way round: a destination bound to a base's value does not follow the base
    d = E.tensor(np.zeros((2, 2), np.float32))
    E.assign(d, a)
    E.assign(v, E.mul(v, 2.0))
    assert np.array_equal(E.fetch(a), [[20.0, 60.0], [40.0, 80.0]])
    assert np.array_equal(E.fetch(d), [[10.0, 30.0], [20.0, 40.0]])


def test_bf16_rounding_keeps_rank_zero():
    """A bf16 reduction over everything is a rank-0 tensor, like its fp32 counterpart."""
    assert round_to_bf16(np.float32(1.00390625)).shape == () and float(round_to_bf16(np.float32(1.00390625))) == 1.0
    E = Eager()
    x = E.tensor(np.full((4, 4), 0.5, np.float32), dtype="bf16")
    s = E.sum(x)
    assert s.shape == () and E.fetch(s).shape == () and float(E.fetch(s)) == 8.0
