"""GPU parity (-m gpu): the HIP path through the C ABI against the CPU oracle, element by element.
Tolerances, norm-wise per tensor (max|got - ref| <= tol * max|ref|): 1e-5 for fp32 paths (a short
chain of <= 1-ulp operations, or an fp32 reduction whose error grows like sqrt(n) * 6e-8), 2e-2 for bf16."""
import numpy as np
import pytest

from oracle.numeric import Eager, round_to_bf16
from workloads import programs
from workloads.inputs import C4_HYPER, c1_inputs, c2_inputs, c4_inputs, c5_batch, c5_inputs

pytestmark = pytest.mark.gpu

TOL32, TOL16 = 1e-5, 2e-2


@pytest.fixture(scope="module")
def ctx():
    from paper_2102_13267_amd import Context
    c = Context(device=0, workspace_bytes=2 << 30)
    yield c
    c.close()


def rel_err(got, ref):
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.array_equal(np.isnan(got), np.isnan(ref))
    fin = np.isfinite(ref)
    assert np.array_equal(got[~fin & ~np.isnan(ref)], ref[~fin & ~np.isnan(ref)])
    if not fin.any():
        return 0.0
    scale = max(float(np.max(np.abs(ref[fin]))), 1e-30)
    return float(np.max(np.abs(got[fin] - ref[fin]))) / scale


REPORT = {}   # test id -> [worst norm-wise error / tol, elements, elements inside the two element-wise bounds]


def elementwise_report(got, ref, tol):
    """Element-wise pass counts next to the norm-wise verdict (which is the parity criterion):
    (a) |got - ref| <= tol * |ref| + tol * max|ref|  (numpy.allclose with rtol = tol, atol = tol * max|ref|);
    (b) the stricter |got - ref| <= tol * |ref| + 0.01 * tol * max|ref|, i.e. relative per element
        down to one hundredth of the tensor's scale."""
    got, ref = np.asarray(got, np.float64).ravel(), np.asarray(ref, np.float64).ravel()
    fin = np.isfinite(ref)
    got, ref = got[fin], ref[fin]
    if ref.size == 0:
        return 0, 0, 0
    scale = max(float(np.max(np.abs(ref))), 1e-30)
    d = np.abs(got - ref)
    return ref.size, int(np.sum(d <= tol * np.abs(ref) + tol * scale)), int(np.sum(d <= tol * np.abs(ref) + 0.01 * tol * scale))


def note(got, ref, tol, err):
    import os
    test = os.environ.get("PYTEST_CURRENT_TEST", "?").split("::")[-1].split(" ")[0]
    n, a, b = elementwise_report(got, ref, tol)
    r = REPORT.setdefault(test, [0.0, 0, 0, 0])
    r[0] = max(r[0], err / tol)
    r[1] += n
    r[2] += a
    r[3] += b


def check(ctx, E, got_t, ref_t, tol, what=""):
    got, ref = ctx.fetch(got_t), E.fetch(ref_t)
    err = rel_err(got, ref)
    note(got, ref, tol, err)
    assert err <= tol, (what, err)
    return err


def rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


UNARY = ["neg", "abs", "exp", "tanh", "sqrt", "rsqrt", "recip", "relu", "gelu", "square", "sigmoid", "log"]


@pytest.mark.parametrize("shape", [(1,), (3, 5), (257,), (64, 100), (1000, 33), (128, 1024)])
def test_unary_ops_each_alone(ctx, shape):
    """Spans one lane, ragged tails, non-multiple-of-4 rows and several workgroup tiles."""
    E = Eager()
    x = (rng(1).random(shape, dtype=np.float32) * 4 + 0.05).astype(np.float32)
    for name in UNARY:
        xin = x if name in ("sqrt", "rsqrt", "log", "recip") else (x - 2.0).astype(np.float32)
        got = getattr(ctx, name)(ctx.tensor(xin))
        ref = getattr(E, name)(E.tensor(xin))
        check(ctx, E, got, ref, TOL32, name)


def test_special_values(ctx):
    E = Eager()
    x = np.array([0.0, -0.0, np.inf, -np.inf, np.nan, 1e-40, -1e-40, 88.0, -104.0], np.float32)
    for name in ["neg", "abs", "exp", "tanh", "relu", "gelu", "square", "sigmoid"]:
        with np.errstate(all="ignore"):
            got = ctx.fetch(getattr(ctx, name)(ctx.tensor(x)))
            ref = E.fetch(getattr(E, name)(E.tensor(x)))
        assert np.array_equal(np.isnan(got), np.isnan(ref)), name
        ok = ~np.isnan(ref)
        assert np.allclose(got[ok], ref[ok], rtol=1e-5, atol=1e-37), (name, got, ref)
    assert ctx.fetch(ctx.tanh(ctx.tensor(np.zeros(4, np.float32)))).tolist() == [0, 0, 0, 0]
    assert ctx.fetch(ctx.exp(ctx.tensor(np.zeros(4, np.float32)))).tolist() == [1, 1, 1, 1]
    assert ctx.fetch(ctx.gelu(ctx.tensor(np.zeros(4, np.float32)))).tolist() == [0, 0, 0, 0]


@pytest.mark.parametrize("shapes", [((64, 48), (64, 48)), ((64, 48), (48,)), ((64, 48), (64, 1)), ((64, 48), ()),
                                    ((7, 5), (5,)), ((7, 5), (7, 1)), ((4, 6, 10), (6, 1)), ((2, 3, 4, 5), (3, 1, 5))])
def test_binary_ops_and_broadcast_modes(ctx, shapes):
    E = Eager()
    a = (rng(2).random(shapes[0], dtype=np.float32) - 0.5).astype(np.float32)
    b = (rng(3).random(shapes[1], dtype=np.float32) + 0.5).astype(np.float32)
    for name in ["add", "sub", "mul", "div", "maximum", "minimum", "relu_grad", "gelu_grad"]:
        check(ctx, E, getattr(ctx, name)(ctx.tensor(a), ctx.tensor(b)), getattr(E, name)(E.tensor(a), E.tensor(b)), TOL32, name)
        check(ctx, E, getattr(ctx, name)(ctx.tensor(b), ctx.tensor(a)), getattr(E, name)(E.tensor(b), E.tensor(a)), TOL32, name)
    check(ctx, E, ctx.add(ctx.tensor(a), ctx.tensor(b), alpha=0.37), E.add(E.tensor(a), E.tensor(b), alpha=0.37), TOL32)
    check(ctx, E, ctx.div(ctx.tensor(a), 3.0), E.div(E.tensor(a), 3.0), TOL32)


def test_empty_and_scalar_tensors(ctx):
    E = Eager()
    e = ctx.add(ctx.tensor(np.zeros((0, 8), np.float32)), 1.0)
    assert ctx.fetch(e).shape == (0, 8)
    s = ctx.mul(ctx.tensor(np.array(3.0, np.float32)), ctx.tensor(np.array(4.0, np.float32)))
    assert ctx.fetch(s) == 12.0


@pytest.mark.parametrize("shape", [(5,), (1000,), (33, 7), (64, 1024), (300, 515), (1 << 20,)])
def test_reductions(ctx, shape):
    E = Eager()
    x = (rng(4).random(shape, dtype=np.float32) - 0.3).astype(np.float32)
    for name in ["sum", "amax", "mean"]:
        check(ctx, E, getattr(ctx, name)(ctx.tensor(x)), getattr(E, name)(E.tensor(x)), TOL32, name)
        if len(shape) == 2:
            check(ctx, E, getattr(ctx, name)(ctx.tensor(x), -1), getattr(E, name)(E.tensor(x), -1), TOL32, name + " rows")
            check(ctx, E, getattr(ctx, name)(ctx.tensor(x), 0), getattr(E, name)(E.tensor(x), 0), TOL32, name + " cols")


def test_sum_of_ones_is_exact(ctx):
    for n in (1, 63, 4096, 1 << 22):
        assert ctx.fetch(ctx.sum(ctx.tensor(np.ones(n, np.float32)))) == n
    assert np.array_equal(ctx.fetch(ctx.sum(ctx.tensor(np.ones((100, 300), np.float32)), 0)), np.full(300, 100.0))
    assert np.array_equal(ctx.fetch(ctx.sum(ctx.tensor(np.ones((100, 300), np.float32)), 1)), np.full(100, 300.0))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_global_norms_over_several_trips(ctx, dtype):
    """Global reductions large enough for the streamed kernel's trips (512 workgroups x 8 tiles) plus
    a ragged rest: the bare operand, a lone square / abs (applied in place), and a prologue that
    goes through the interpreter; signs alternate so that a dropped tile or a wrong sign shows."""
    E = Eager()
    n = 2 * 512 * 8 * 1024 + 5 * 4096 + 7
    x = (rng(11).standard_normal(n, dtype=np.float32) * (1.0 + (np.arange(n) % 3))).astype(np.float32)
    if dtype == "bf16":
        x = round_to_bf16(x)

    def prog(B, x):
        return (B.sum(x), B.sum(B.square(x)), B.sum(B.abs(x)), B.amax(B.abs(x)), B.sqrt(B.sum(B.square(x))),
                B.sum(B.mul(B.square(x), 0.5)), B.amax(B.neg(x)))
    got = prog(ctx, ctx.tensor(x, dtype=dtype))
    ref = prog(E, E.tensor(x, dtype=dtype))
    val = lambda B, t: float(np.asarray(B.fetch(t)).reshape(-1)[0])
    gv, rv = [val(ctx, t) for t in got], [val(E, t) for t in ref]
    tol = TOL16 if dtype == "bf16" else TOL32               # (bf16 results are rounded to bf16)
    assert abs(gv[0] - rv[0]) <= 2e-6 * rv[2]                # the plain sum cancels: against the sum of magnitudes
    for k in range(1, len(gv)):
        assert abs(gv[k] - rv[k]) <= tol * abs(rv[k]), (k, gv[k], rv[k])


@pytest.mark.parametrize("rows,cols", [(1, 1024), (7, 1024), (130, 2048), (33, 4096), (5, 8192), (9, 3072), (6, 1000)])
def test_row_reductions_streamed(ctx, rows, cols):
    """Row reductions whose rows are whole multiples of what a wave (1024 columns) or a workgroup
    (4096) takes per trip -- four 4-vectors per lane and interpreter dispatch -- with one and two
    whole inputs, a vector broadcast along rows, sum / max / mean, row counts that do not fill the
    last workgroup; the last two shapes take the one-vector-at-a-time kernel."""
    E = Eager()
    g = rng(900 + rows + cols)
    x, y = (g.standard_normal((rows, cols), dtype=np.float32) for _ in range(2))
    b = g.standard_normal(cols, dtype=np.float32)

    def prog(B, x, y, b):
        s1 = B.sum(x, axis=1)                                          # the bare operand
        s2 = B.amax(B.mul(B.tanh(B.add(B.mul(x, y), b)), 0.5), axis=1)  # two whole inputs + a row vector
        s3 = B.mean(B.square(B.sub(y, b)), axis=1)                     # one whole input + a row vector
        s4 = B.add(B.sum(B.exp(B.neg(B.abs(x))), axis=1), 1.0)        # a longer chain and an epilogue
        return s1, s2, s3, s4
    got = prog(ctx, ctx.tensor(x), ctx.tensor(y), ctx.tensor(b))
    ref = prog(E, E.tensor(x), E.tensor(y), E.tensor(b))
    check(ctx, E, got[0], ref[0], 2e-6 * cols ** 0.5 + TOL32, "sum")   # (sums of N(0,1) cancel: scale by sqrt(cols))
    for gt, rt, what in zip(got[1:], ref[1:], ("max", "mean", "chain")):
        check(ctx, E, gt, rt, TOL32, what)


def test_reduction_with_prologue_and_epilogue(ctx):
    E = Eager()
    x = (rng(5).random((200, 96), dtype=np.float32) - 0.5).astype(np.float32)
    w = (rng(6).random((96,), dtype=np.float32)).astype(np.float32)
    c = (rng(7).random((200,), dtype=np.float32)).astype(np.float32)

    def prog(B, x, w, c):
        z = B.mul(B.tanh(x), w)                     # prologue with a row-vector broadcast
        r = B.add(B.sum(z, axis=1), c)               # row reduce + epilogue
        k = B.sub(B.amax(B.mul(B.square(x), B.expand(B.reshape(c, (200, 1)), (200, 96))), axis=0), w)   # column-vector broadcast, column reduce
        t = B.sqrt(B.add(B.mean(B.abs(x)), 1.0))     # global reduce + scalar epilogue
        return r, k, t
    got = prog(ctx, ctx.tensor(x), ctx.tensor(w), ctx.tensor(c))
    ref = prog(E, E.tensor(x), E.tensor(w), E.tensor(c))
    for g, r in zip(got, ref):
        check(ctx, E, g, r, TOL32)


@pytest.mark.parametrize("rows,cols", [(64, 48), (1024, 1024), (100, 1000), (37, 4100)])
def test_c1_trace(ctx, rows, cols):
    E = Eager()
    inp = c1_inputs(rows, cols)
    hits = []
    for it in range(3):
        out = programs.c1_trace(ctx, *(ctx.tensor(inp[k]) for k in ("x", "y", "bias")))
        info = ctx.barrier()
        hits.append(info.cache_hit)
        got = ctx.fetch(out)
        if it == 0:
            first = got
        else:
            assert np.array_equal(got, first)        # a cache hit gives the same bits as the fresh lowering
    assert hits == [0, 1, 1] and info.n_regions == 2
    ref = E.fetch(programs.c1_trace(E, *(E.tensor(inp[k]) for k in ("x", "y", "bias"))))
    assert rel_err(got, ref) <= TOL32
    assert np.max(np.abs(got)) == 1.0                # x / |x| is exact


def test_c1_trace_streaming_size_sampled_rows():
    """The C1 trace on [16384, 16384] operands (the size at which bench.py quotes the row kernel's
    rate against HBM): row sums of sampled rows against the oracle's, which computes them one row
    at a time, and the normalised output's exact maximum."""
    import torch
    from paper_2102_13267_amd import Context
    n = 16384
    c = Context(device=0, workspace_bytes=64 << 20)
    gen = torch.Generator(device="cuda:0").manual_seed(1001)
    x, y = (torch.rand(n, n, device="cuda:0", generator=gen) * 2 - 1 for _ in range(2))
    b = torch.rand(n, device="cuda:0", generator=gen) * 2 - 1
    tx, ty, tb = c.tensor(x), c.tensor(y), c.tensor(b)
    t = c.tanh(c.add(c.mul(tx, ty), tb))
    e = c.exp(c.neg(c.square(tx)))
    s = c.sum(c.add(c.mul(t, e), ty, alpha=0.5), axis=1)      # the trace's row reduction, kept as a result
    out = c.div(s, c.amax(c.abs(s)))
    del t, e                                                  # (dead at the barrier, as inside c1_trace: never materialised)
    info = c.barrier()
    assert info.n_regions == 2
    got_s, got_out = c.fetch(s), c.fetch(out)
    assert np.max(np.abs(got_out)) == 1.0                     # x / |x| is exact
    E = Eager()
    bias = b.cpu().numpy()
    for r in (0, 1, 4095, 4096, 9999, n - 1):
        xr, yr = x[r].cpu().numpy()[None, :], y[r].cpu().numpy()[None, :]
        zr = E.add(E.mul(E.tanh(E.add(E.mul(E.tensor(xr), E.tensor(yr)), E.tensor(bias))), E.exp(E.neg(E.square(E.tensor(xr))))),
                   E.tensor(yr), alpha=0.5)
        ref = float(np.asarray(E.fetch(E.sum(zr, axis=1))).reshape(-1)[0])
        mag = float(np.asarray(E.fetch(E.sum(E.abs(zr), axis=1))).reshape(-1)[0])
        assert abs(float(got_s[r]) - ref) <= 2e-6 * mag, (r, got_s[r], ref, mag)
    c.close()


def test_c1_full_size_ten_runs():
    from paper_2102_13267_amd import Context
    ctx = Context(device=0, workspace_bytes=64 << 20)     # a fresh cache: 1 miss + 9 hits
    inp = c1_inputs()
    x, y, b = (ctx.tensor(inp[k]) for k in ("x", "y", "bias"))
    hits = []
    for _ in range(10):
        out = programs.c1_trace(ctx, x, y, b)
        hits.append(ctx.barrier().cache_hit)
    assert hits == [0] + [1] * 9
    E = Eager()
    ref = E.fetch(programs.c1_trace(E, *(E.tensor(inp[k]) for k in ("x", "y", "bias"))))
    assert rel_err(ctx.fetch(out), ref) <= TOL32


@pytest.mark.parametrize("n", [1000, 70000, (1 << 22) + 3])
def test_c4_adam_clip(ctx, n):
    E = Eager()
    inp = c4_inputs(n)
    names = ("p", "g", "m", "v")
    gt = [ctx.tensor(inp[k].copy(), donatable=True) for k in names]
    rt = [E.tensor(inp[k]) for k in names]
    for step in range(2):
        hyper = dict(C4_HYPER, t=step + 1)
        programs.c4_step(ctx, *gt, **hyper)
        info = ctx.barrier()
        programs.c4_step(E, *rt, **hyper)
        assert info.cache_hit == (step > 0)
        for g, r, k in zip(gt, rt, names):
            if k != "g":
                check(ctx, E, g, r, TOL32, f"{k} step {step}")
    if n > 65536:
        assert info.n_regions == 2
        assert ctx.dump_plan().count("->p") == 3     # p, m, v updated in place


def test_in_place_semantics_of_section_4_3(ctx):
    """a += 1; read; read  -> the second read must not add again.
    b = a + 2; a += 1      -> b sees the old a."""
    import torch
    base = torch.arange(8, dtype=torch.float32, device="cuda:0")
    a = ctx.tensor(base, donatable=True)
    ctx.assign(a, ctx.add(a, 1.0))
    assert ctx.fetch(a).tolist() == list(range(1, 9))
    assert ctx.fetch(a).tolist() == list(range(1, 9))
    assert ctx.device_ptr(a) == base.data_ptr()      # donated: updated in place
    b = ctx.add(a, 2.0)
    ctx.assign(a, ctx.add(a, 1.0))
    assert ctx.fetch(a).tolist() == list(range(2, 10))
    assert ctx.fetch(b).tolist() == list(range(3, 11))
    # a second handle on the buffer forbids donation
    keep = ctx.scalar(0.0)
    ctx.assign(keep, a)
    ctx.assign(a, ctx.mul(a, 2.0))
    assert ctx.fetch(a).tolist() == [2 * v for v in range(2, 10)]
    assert ctx.fetch(keep).tolist() == list(range(2, 10))
    # a live tensor that folding reduces to the updated buffer itself (b = a * 1) keeps the old value
    base2 = torch.arange(8, dtype=torch.float32, device="cuda:0")
    a2 = ctx.tensor(base2, donatable=True)
    b2 = ctx.mul(a2, 1.0)
    ctx.assign(a2, ctx.add(a2, 1.0))
    ctx.barrier()
    assert "->p" not in ctx.dump_plan()
    assert ctx.fetch(b2).tolist() == list(range(8)) and ctx.fetch(a2).tolist() == list(range(1, 9))
    # ... and so does a view of it that is alive at the barrier
    a3 = ctx.tensor(torch.arange(8, dtype=torch.float32, device="cuda:0"), donatable=True)
    v3 = ctx.reshape(a3, (2, 4))
    ctx.assign(a3, ctx.add(a3, 1.0))
    ctx.barrier()
    assert ctx.fetch(v3).ravel().tolist() == list(range(8)) and ctx.fetch(a3).tolist() == list(range(1, 9))


def test_permutation_of_a_value_computed_in_the_same_step(ctx):
    """A permutation reads other positions than it writes: its operand has to be in memory, so the
    producer of the operand never shares a kernel with it -- not even as the post program of the
    contraction that both hang on (s = a + a^T with a = x w), and a reshape that is itself a result
    is a flat copy whatever the two shapes are."""
    E = Eager()
    r = rng(21)
    x, w = r.standard_normal((48, 40), dtype=np.float32), r.standard_normal((40, 48), dtype=np.float32)

    def prog(B, x, w):
        a = B.matmul(x, w)
        s = B.add(a, B.permute(a, (1, 0)))
        e = B.exp(B.mul(x, 0.1))
        return s, B.add(e, 1.0), B.permute(e, (1, 0)), B.reshape(e, (40, 48)), B.reshape(e, (1920,))
    got = prog(ctx, ctx.tensor(x), ctx.tensor(w))
    ref = prog(E, E.tensor(x), E.tensor(w))
    for g, rr, what in zip(got, ref, ("a + a^T", "e + 1", "e^T", "e as 40x48", "e flat")):
        check(ctx, E, g, rr, TOL32, what)


def test_fused_and_unfused_plans_agree():
    """Section 3: a compiled trace is equivalent to running the recorded operations one by one.
    Inside the library: the same traces with fusion switched off (every op a kernel of its own,
    every intermediate in memory) against the fused plans, and both against the oracle."""
    from paper_2102_13267_amd import Context
    c = Context(device=0, workspace_bytes=1 << 30)
    E = Eager()
    inp1 = c1_inputs(300, 1028)
    inp2 = c2_inputs(steps=1)
    names = ("W1", "b1", "W2", "b2", "W3", "b3")
    cfg = (2, 16, 64, 128, 4)
    results = {}
    for fused in (True, False):
        c.set_fusion(fused)
        out1 = programs.c1_trace(c, *(c.tensor(inp1[k]) for k in ("x", "y", "bias")))
        n1 = c.barrier().n_regions
        gp = [c.tensor(inp2[k].copy(), donatable=True) for k in names]
        loss = programs.c2_step(c, c.tensor(inp2["X"][0]), c.tensor(inp2["labels"][0]), gp, 0.01)
        n2 = c.barrier().n_regions
        g3 = _c3_setup(c, lambda a, dt, don: c.tensor(a, dtype=dt, donatable=don), cfg)
        y3, dx3 = programs.c3_step(c, *g3, t=1)
        n3 = c.barrier().n_regions
        results[fused] = ([c.fetch(out1), c.fetch(loss)] + [c.fetch(p) for p in gp], [c.fetch(y3), c.fetch(dx3)] +
                          [c.fetch(g3[3][k]) for k in programs.C3_WEIGHTS + programs.C3_VECTORS if k != "bk"], (n1, n2, n3))
    assert results[True][2][0] == 2 and results[False][2][0] == 12
    assert results[False][2][1] > results[True][2][1] and results[False][2][2] > results[True][2][2]
    for a, b in zip(results[True][0], results[False][0]):
        assert rel_err(a, b) <= 2 * TOL32
    for a, b in zip(results[True][1], results[False][1]):
        assert rel_err(a, b) <= 2 * TOL16
    ref1 = E.fetch(programs.c1_trace(E, *(E.tensor(inp1[k]) for k in ("x", "y", "bias"))))
    rp = [E.tensor(inp2[k]) for k in names]
    ref_loss = E.fetch(programs.c2_step(E, E.tensor(inp2["X"][0]), E.tensor(inp2["labels"][0]), rp, 0.01))
    for fused in (True, False):
        assert rel_err(results[fused][0][0], ref1) <= TOL32 and rel_err(results[fused][0][1], ref_loss) <= TOL32
        for got, r in zip(results[fused][0][2:], rp):
            assert rel_err(got, E.fetch(r)) <= TOL32
    c.close()


@pytest.mark.parametrize("donatable", [True, False])
def test_in_place_updates_through_views(ctx, donatable):
    """Section 4.4: views share storage with their base as far as a program can tell.  The library
    records forward and backward sequences; the oracle really shares memory (NumPy views)."""
    E = Eager()
    r = rng(31)
    x, y = r.standard_normal((2, 3, 4), dtype=np.float32), r.standard_normal((6, 4), dtype=np.float32)
    gx = ctx.tensor(x.copy(), donatable=donatable)
    got = programs.views_program(ctx, gx, ctx.tensor(y))
    info = ctx.barrier()
    ref = programs.views_program(E, E.tensor(x.copy()), E.tensor(y))
    for g, rr, what in zip(got, ref, ("x", "v", "w", "s")):
        check(ctx, E, g, rr, TOL32, what)
    # second step on the materialised tensors: views are derived again from the new base
    got2 = programs.views_program(ctx, got[0], ctx.tensor(y))
    ref2 = programs.views_program(E, ref[0], E.tensor(y))
    for g, rr, what in zip(got2 + got[1:3], ref2 + ref[1:3], ("x", "v", "w", "s", "old v", "old w")):
        check(ctx, E, g, rr, TOL32, what + " (step 2)")


def test_windows_of_larger_tensors(ctx):
    """narrow as addressing (elementwise consumers, a contraction operand), as a copy (a result, a
    reduction operand), and the window update in place and out of place, on sizes that span tiles;
    bf16 too."""
    E = Eager()
    r = rng(32)
    a = r.standard_normal((300, 520), dtype=np.float32)
    w = r.standard_normal((128, 64), dtype=np.float32)
    u = r.standard_normal((300, 100), dtype=np.float32)

    def prog(B, a, w, u):
        left = B.narrow(a, 1, 4, 128)                   # [300, 128] at a 16-byte aligned offset
        odd = B.narrow(a, 1, 3, 128)                    # ... and at an unaligned one
        rows = B.narrow(a, 0, 7, 100)                   # a window of whole rows: dense
        e = B.add(B.tanh(left), odd)
        mm = B.matmul(left, w)
        red = B.sum(rows, axis=1)
        upd = B.slice_update(a, u, 1, 33)               # out of place: a stays as it is
        return e, mm, red, upd, rows
    got = prog(ctx, ctx.tensor(a), ctx.tensor(w), ctx.tensor(u))
    ref = prog(E, E.tensor(a), E.tensor(w), E.tensor(u))
    for g, rr, what in zip(got, ref, ("e", "mm", "red", "upd", "rows")):
        check(ctx, E, g, rr, TOL32, what)
    hb = round_to_bf16(r.standard_normal((64, 1024), dtype=np.float32))
    gh, rh = ctx.tensor(hb.copy(), dtype="bf16", donatable=True), E.tensor(hb.copy(), dtype="bf16")
    for B, t in ((ctx, gh), (E, rh)):
        win = B.view_narrow(t, 1, 256, 512)
        B.assign(win, B.mul(win, 0.5))
    ctx.barrier()
    assert "->p" in ctx.dump_plan() and " SLICE " in ctx.dump_plan()      # the window is written in place
    check(ctx, E, gh, rh, TOL16, "bf16 window in place")


def test_fallback_runs_the_eager_op_on_the_device(ctx):
    """Section 4.5: ops without a lowering (reductions over a middle axis, a custom opcode) are run
    by a registered fallback -- here the eager framework's own ops on the device memory that the
    library hands over -- after the pending trace has been evaluated; lazy ops go on from the results."""
    import torch
    E = Eager()
    seen = []

    def fb(opcode, inputs, attrs, outputs, run):
        seen.append((opcode, run))
        if opcode == 1024:                                   # running sum along the last axis
            if not run:
                outputs[0]["dtype"], outputs[0]["shape"] = inputs[0]["dtype"], inputs[0]["shape"]
                return
            ctx.device_array(outputs[0]).copy_(torch.cumsum(ctx.device_array(inputs[0]), dim=-1))
            return
        fn = {64: torch.sum, 65: torch.amax, 66: torch.mean}[opcode]
        out = ctx.device_array(outputs[0])
        out.copy_(fn(ctx.device_array(inputs[0]).float(), dim=attrs[3]).to(out.dtype))
    ctx.set_fallback(fb)
    try:
        x = rng(33).standard_normal((4, 6, 8), dtype=np.float32)
        gx = ctx.tensor(x)
        a = ctx.exp(ctx.mul(gx, 0.1))                        # pending when the first fallback op arrives
        m = ctx.sum(a, axis=1)
        c = ctx.custom_op(1024, [m])
        out = ctx.add(ctx.tanh(ctx.mul(c, 0.05)), ctx.amax(a, axis=1))
        hb = ctx.mean(ctx.cast(a, "bf16"), axis=0)           # axis 0 of a rank-3 tensor, bf16
        ra = E.exp(E.mul(E.tensor(x), 0.1))
        rm = E.sum(ra, axis=1)
        rc = E.tensor(np.cumsum(E.fetch(rm).astype(np.float64), axis=-1).astype(np.float32))
        rout = E.add(E.tanh(E.mul(rc, 0.05)), E.amax(ra, axis=1))
        check(ctx, E, m, rm, TOL32, "sum over the middle axis")
        check(ctx, E, out, rout, TOL32, "lazy ops after fallback ops")
        check(ctx, E, hb, E.mean(E.cast(ra, "bf16"), axis=0), TOL16, "bf16 mean over axis 0 of rank 3")
        assert [s for s in seen if s[0] == 1024] == [(1024, False), (1024, True)] and ctx.stats().fallback_ops >= 4
    finally:
        ctx.set_fallback(None)


def test_a_leaf_dropped_before_the_barrier_keeps_its_memory(ctx):
    """The trace names a leaf's device memory until the barrier has run; the binding keeps the owner
    of that memory alive that long even when the program drops its handle first."""
    import gc
    a = np.full((1 << 16,), 3.0, np.float32)
    b = np.full((1 << 16,), 5.0, np.float32)
    v = ctx.exp(ctx.tensor(a))          # the leaf's handle dies here
    gc.collect()
    w = ctx.tensor(b)                   # same size: the allocator would reuse a freed block
    out = ctx.fetch(v)
    assert np.allclose(out, np.exp(np.float32(3.0)), rtol=1e-6)
    assert ctx.fetch(ctx.neg(w))[0] == -5.0


ROW_SHAPES = [(4, 10), (128, 10), (33, 64), (256, 256), (8, 1000), (16, 1024), (5, 4096), (3, 1030)]


@pytest.mark.parametrize("shape", ROW_SHAPES)
def test_row_operators_f32(ctx, shape):
    E = Eager()
    r = rng(8)
    x = (r.standard_normal(shape, dtype=np.float32) * 2).astype(np.float32)
    dy = r.standard_normal(shape, dtype=np.float32)
    g = (r.random(shape[1], dtype=np.float32) + 0.5).astype(np.float32)
    b = r.standard_normal(shape[1], dtype=np.float32)
    lab = r.integers(0, shape[1], size=shape[0], dtype=np.int32)

    def prog(B, x, dy, g, b, lab):
        p = B.softmax(x)
        dp = B.softmax_grad(dy, p)
        y, mu, rs = B.layer_norm(x, g, b, eps=1e-5)
        dx = B.layer_norm_grad(dy, x, g, mu, rs)
        l = B.xent(x, lab)
        dl = B.xent_grad(x, lab, 0.25)
        return p, dp, y, mu, rs, dx, l, dl
    got = prog(ctx, *(ctx.tensor(v) for v in (x, dy, g, b, lab)))
    ref = prog(E, *(E.tensor(v) for v in (x, dy, g, b, lab)))
    for k, (gg, rr) in enumerate(zip(got, ref)):
        check(ctx, E, gg, rr, 2e-5 if k == 5 else TOL32, f"row op output {k}")
    p = ctx.fetch(got[0])
    assert np.allclose(p.sum(axis=1), 1.0, atol=1e-5)


def test_row_operators_bf16(ctx):
    E = Eager()
    r = rng(9)
    shape = (64, 256)
    x = round_to_bf16(r.standard_normal(shape, dtype=np.float32))
    dy = round_to_bf16(r.standard_normal(shape, dtype=np.float32))
    g = round_to_bf16((r.random(shape[1], dtype=np.float32) + 0.5).astype(np.float32))
    b = round_to_bf16(r.standard_normal(shape[1], dtype=np.float32))

    def prog(B, x, dy, g, b):
        p = B.softmax(x)
        dp = B.softmax_grad(dy, p)
        y, mu, rs = B.layer_norm(x, g, b)
        dx = B.layer_norm_grad(dy, x, g, mu, rs)
        return p, dp, y, dx
    got = prog(ctx, *(ctx.tensor(v, dtype="bf16") for v in (x, dy, g, b)))
    ref = prog(E, *(E.tensor(v, dtype="bf16") for v in (x, dy, g, b)))
    for gg, rr in zip(got, ref):
        assert gg.dtype == "bf16"
        check(ctx, E, gg, rr, TOL16)


GEMM_SHAPES = [(1, 1, 1), (8, 8, 8), (128, 128, 16), (130, 70, 33), (128, 784, 512), (257, 1000, 129), (128, 512, 10)]


@pytest.mark.parametrize("m,k,n", GEMM_SHAPES)
@pytest.mark.parametrize("ta,tb", [(False, False), (True, False), (False, True), (True, True)])
def test_gemm_f32(ctx, m, k, n, ta, tb):
    E = Eager()
    r = rng(10)
    a = r.standard_normal((k, m) if ta else (m, k), dtype=np.float32)
    b = r.standard_normal((n, k) if tb else (k, n), dtype=np.float32)
    check(ctx, E, ctx.matmul(ctx.tensor(a), ctx.tensor(b), ta, tb), E.matmul(E.tensor(a), E.tensor(b), ta, tb), TOL32, (m, k, n, ta, tb))


def test_gemm_identity_and_ones(ctx):
    a = rng(11).standard_normal((200, 96), dtype=np.float32)
    assert np.array_equal(ctx.fetch(ctx.matmul(ctx.tensor(a), ctx.tensor(np.eye(96, dtype=np.float32)))), a)
    ones = ctx.fetch(ctx.matmul(ctx.tensor(np.ones((150, 256), np.float32)), ctx.tensor(np.ones((256, 70), np.float32))))
    assert np.all(ones == 256)
    h = ctx.fetch(ctx.matmul(ctx.tensor(np.ones((150, 256), np.float32), dtype="bf16"),
                             ctx.tensor(np.ones((256, 70), np.float32), dtype="bf16")))
    assert np.all(h == 256)


@pytest.mark.parametrize("m,k,n", [(8, 8, 8), (128, 64, 128), (130, 70, 33), (256, 1024, 512), (100, 40, 264)])
@pytest.mark.parametrize("ta,tb", [(False, False), (True, False), (False, True), (True, True)])
def test_gemm_bf16(ctx, m, k, n, ta, tb):
    E = Eager()
    r = rng(12)
    a = round_to_bf16(r.standard_normal((k, m) if ta else (m, k), dtype=np.float32))
    b = round_to_bf16(r.standard_normal((n, k) if tb else (k, n), dtype=np.float32))
    got = ctx.matmul(ctx.tensor(a, dtype="bf16"), ctx.tensor(b, dtype="bf16"), ta, tb)
    ref = E.matmul(E.tensor(a, dtype="bf16"), E.tensor(b, dtype="bf16"), ta, tb)
    check(ctx, E, got, ref, TOL16, (m, k, n, ta, tb))
    # fp32 output of a bf16 product keeps the fp32 accumulator: far tighter than bf16 rounding
    got32 = ctx.matmul(ctx.tensor(a, dtype="bf16"), ctx.tensor(b, dtype="bf16"), ta, tb, dtype="f32")
    ref32 = E.matmul(E.tensor(a, dtype="bf16"), E.tensor(b, dtype="bf16"), ta, tb, dtype="f32")
    check(ctx, E, got32, ref32, 1e-5, (m, k, n, ta, tb))


@pytest.mark.parametrize("m,k,n,batch", [(200, 1100, 136, ()), (128, 2048, 256, ()), (70, 520, 90, (3,)), (33, 777, 50, (2, 2))])
def test_gemm_bf16_long_k_with_epilogue(ctx, m, k, n, batch):
    """Few output tiles and a long contraction: k is split over several workgroups, their partial
    products are summed in a second launch that also runs the fused chain (ragged in every
    dimension, plain and batched)."""
    E = Eager()
    r = rng(14)
    a = round_to_bf16(r.standard_normal(batch + (k, m), dtype=np.float32))       # used transposed
    b = round_to_bf16(r.standard_normal(batch + (k, n), dtype=np.float32))
    bias = round_to_bf16(r.standard_normal((n,), dtype=np.float32))
    res = round_to_bf16(r.standard_normal(batch + (m, n), dtype=np.float32))

    def prog(B):
        t = lambda v: B.tensor(v, dtype="bf16")
        return B.add(t(res), B.relu(B.add(B.matmul(t(a), t(b), True, False), t(bias))))
    got = prog(ctx)
    info = ctx.barrier()
    assert info.n_regions == 1
    check(ctx, E, got, prog(E), TOL16, (m, k, n, batch))


def test_gemm_batched_and_epilogue(ctx):
    E = Eager()
    r = rng(13)
    a = r.standard_normal((3, 4, 70, 48), dtype=np.float32)
    b = r.standard_normal((3, 4, 48, 90), dtype=np.float32)
    check(ctx, E, ctx.matmul(ctx.tensor(a), ctx.tensor(b)), E.matmul(E.tensor(a), E.tensor(b)), TOL32)
    bt = r.standard_normal((3, 4, 90, 48), dtype=np.float32)
    check(ctx, E, ctx.matmul(ctx.tensor(a), ctx.tensor(bt), False, True), E.matmul(E.tensor(a), E.tensor(bt), False, True), TOL32)
    w = r.standard_normal((48, 90), dtype=np.float32)
    bias = r.standard_normal((90,), dtype=np.float32)
    res = r.standard_normal((3, 4, 70, 90), dtype=np.float32)

    def prog(B, a, w, bias, res):
        return B.add(res, B.gelu(B.add(B.matmul(a, w), bias)))
    got = prog(ctx, *(ctx.tensor(v) for v in (a, w, bias, res)))
    info = ctx.barrier()
    assert info.n_regions == 1
    check(ctx, E, got, prog(E, *(E.tensor(v) for v in (a, w, bias, res))), TOL32)


SMALL_GEMMS = [  # m, k, n, ta, tb, batch, kernel variant (A, B fetched as whole 4-vectors along k)
    (128, 784, 512, False, False, (), "true, false"),     # a layer of the small MLP
    (128, 512, 512, False, True, (), "true, true"),
    (128, 512, 10, False, False, (), "true, false"),      # ten columns: one ragged tile
    (512, 128, 512, True, False, (), "false, false"),     # weight-gradient shape, both operands across k
    (100, 36, 72, False, True, (), "true, true"),         # k a multiple of 4, not of 8
    (100, 35, 72, False, True, (), "false, false"),       # k not a multiple of 4: element loads
    (33, 1000, 41, True, True, (), "false, true"),        # ragged everywhere, k split unevenly over the waves
    (1, 64, 1, False, False, (), "true, true"),          # (one column: k is B's contiguous dimension too)
    (70, 520, 90, False, False, (3,), "true, false"),     # batched
    (40, 96, 50, True, False, (2, 2), "false, false"),
    # a long k over few tiles: several workgroups share a tile and exchange partial tiles in the launch
    (8, 2048, 2048, False, False, (), "true, false"),     # four per tile
    (64, 2048, 512, False, True, (), "true, true"),       # eight per tile
    (33, 1500, 70, True, False, (), "false, false"),      # five per tile, ragged
    (20, 1101, 40, True, True, (), "false, false"),       # k odd: element loads, uneven slices
    (40, 1100, 50, False, False, (3,), "true, false"),    # batched
    (120, 1100, 2040, True, False, (), "false, false"),   # 256 tiles of 32 x 32: tiles of 64 x 32, two per tile, ragged
    (128, 2048, 2048, False, False, (), "true, false"),
    (64, 2048, 2048, False, False, (), "true, false"),    # 128 tiles, two per tile
]


@pytest.mark.parametrize("m,k,n,ta,tb,batch,variant", SMALL_GEMMS)
def test_gemm_f32_small_one_launch(ctx, m, k, n, ta, tb, batch, variant):
    """Small fp32 products run as ONE launch (k split over the eight waves of a workgroup -- and,
    for a long k over few tiles, over several workgroups per tile that exchange partial tiles --,
    the partial tiles added in a fixed order, the post program on the sum): the product alone,
    twice (the tickets of shared tiles must be back at zero), and with a bias, an activation, a
    residual and a second result in the same region."""
    E = Eager()
    r = rng(15)
    a = r.standard_normal(batch + ((k, m) if ta else (m, k)), dtype=np.float32)
    b = r.standard_normal(batch + ((n, k) if tb else (k, n)), dtype=np.float32)
    bias = r.standard_normal((n,), dtype=np.float32)
    res = r.standard_normal(batch + (m, n), dtype=np.float32)
    ctx.set_profiling(True)
    try:
        got = ctx.matmul(ctx.tensor(a), ctx.tensor(b), ta, tb)
        ctx.barrier()
        names = [l["kernel"] for l in ctx.last_launches()]
        assert len(names) == 1 and names[0].startswith("lt_gemm_small_kernel<") and names[0].endswith(", %s, false>" % variant), names
        check(ctx, E, got, E.matmul(E.tensor(a), E.tensor(b), ta, tb), TOL32, "product")
        again = ctx.matmul(ctx.tensor(a), ctx.tensor(b), ta, tb)
        assert np.array_equal(ctx.fetch(again), ctx.fetch(got))

        def prog(B):
            y = B.add(B.matmul(B.tensor(a), B.tensor(b), ta, tb), B.tensor(bias))
            return B.add(B.tensor(res), B.mul(B.gelu(y), 0.5)), B.relu(y)
        g1, g2 = prog(ctx)
        info = ctx.barrier()
        assert info.n_regions == 1 and info.n_launches == 1
        assert ctx.last_launches()[0]["kernel"].startswith("lt_gemm_small_kernel")
    finally:
        ctx.set_profiling(False)
    r1, r2 = prog(E)
    check(ctx, E, g1, r1, TOL32, "residual + gelu")
    check(ctx, E, g2, r2, TOL32, "relu")


@pytest.mark.parametrize("m,k,n,mean", [(512, 128, 512, False), (784, 128, 512, False), (512, 128, 10, False), (100, 77, 45, True),
                                        (33, 200, 64, False), (64, 1024, 96, True)])
def test_bias_gradient_rides_with_the_weight_gradient(ctx, m, k, n, mean):
    """dW = x^T dy and db = sum over the rows of dy, each with an in-place SGD update as its post
    program: two regions, ONE launch (the small contraction adds up the columns of the dy it
    fetches anyway and runs the column program too)."""
    E = Eager()
    r = rng(16)
    x = r.standard_normal((k, m), dtype=np.float32)
    dy = r.standard_normal((k, n), dtype=np.float32)
    w = r.standard_normal((m, n), dtype=np.float32)
    b = r.standard_normal((n,), dtype=np.float32)

    def prog(B):
        tx, tdy = B.tensor(x), B.tensor(dy)
        tw, tb = B.tensor(w.copy(), donatable=True), B.tensor(b.copy(), donatable=True)
        dw = B.matmul(tx, tdy, True, False)
        db = B.mean(tdy, 0) if mean else B.sum(tdy, 0)
        B.assign(tw, B.sub(tw, B.mul(dw, 0.01)))
        B.assign(tb, B.sub(tb, B.mul(db, 0.01)))
        return tw, tb, B.relu(db)
    ctx.set_profiling(True)
    try:
        got = prog(ctx)
        info = ctx.barrier()
        names = [l["kernel"] for l in ctx.last_launches()]
    finally:
        ctx.set_profiling(False)
    assert info.n_regions == 2 and info.n_launches == 1 and names[0].startswith("lt_gemm_small_kernel") and names[0].endswith(", true>"), (info.n_regions, names)
    for g, e in zip(got, prog(E)):
        check(ctx, E, g, e, TOL32 * max(1.0, (k / 64) ** 0.5))   # (sums of k terms: the bar of the column reductions)


def test_bias_gradient_keeps_its_own_launch_when_it_must(ctx):
    """The column program reads what the contraction writes: no riding along; same values."""
    E = Eager()
    r = rng(17)
    x = r.standard_normal((128, 96), dtype=np.float32)
    dy = r.standard_normal((128, 64), dtype=np.float32)

    def prog(B):
        tx, tdy = B.tensor(x), B.tensor(dy)
        dw = B.matmul(tx, tdy, True, False)                 # [96, 64]
        first = B.narrow(dw, 0, 0, 1)                       # its first row, [1, 64]
        return dw, B.add(B.sum(tdy, 0), B.reshape(first, (64,)))
    got = prog(ctx)
    info = ctx.barrier()
    assert info.n_launches >= 2
    for g, e in zip(got, prog(E)):
        check(ctx, E, g, e, TOL32 * 2)


def test_random_weight_and_bias_gradient_pairs(ctx):
    """Random shapes and post programs around dW = x^T dy, db = sum or mean over the rows of dy: cases
    where the column sum may share the contraction's launch and cases where it must not (one
    program reads what the other writes, the sum comes first, two sums), against the fp64 oracle."""
    shared = 0
    for seed in range(120):
        g = rng(500 + seed)
        m = int(g.choice([1, 10, 32, 33, 100, 512, 784])); n = int(g.choice([1, 4, 10, 33, 64, 130, 512]))
        k = int(g.choice([32, 33, 64, 100, 128, 500, 1024]))
        variant, mean, computed_dy = int(g.integers(0, 7)), bool(g.integers(0, 2)), bool(g.integers(0, 2))
        x = g.standard_normal((k, m)).astype(np.float32); dy0 = g.standard_normal((k, n)).astype(np.float32)
        w = g.standard_normal((m, n)).astype(np.float32); b = g.standard_normal((n,)).astype(np.float32)

        def prog(B):
            tx, tdy = B.tensor(x), B.tensor(dy0)
            tw, tb = B.tensor(w.copy(), donatable=True), B.tensor(b.copy(), donatable=True)
            dy = B.mul(B.relu(tdy), 0.5) if computed_dy else tdy
            dw = B.matmul(tx, dy, True, False)
            db = B.mean(dy, 0) if mean else B.sum(dy, 0)
            outs = []
            if variant == 0:
                B.assign(tw, B.sub(tw, B.mul(dw, 0.01))); B.assign(tb, B.sub(tb, B.mul(db, 0.01)))
            elif variant == 1:
                outs += [dw, db]
            elif variant == 2:                       # the contraction's post reads the bias that the column program updates
                outs.append(B.add(dw, tb)); B.assign(tb, B.sub(tb, B.mul(db, 0.01)))
            elif variant == 3:                       # the column program reads the weight that the contraction updates
                B.assign(tw, B.sub(tw, B.mul(dw, 0.01))); outs.append(B.add(db, B.reshape(B.narrow(tw, 0, 0, 1), (n,))))
            elif variant == 4:                       # two column sums over the same rows
                outs += [dw, db, B.sum(B.mul(dy, dy), 0)]
            elif variant == 5:                       # the column sum first
                outs += [db, B.matmul(tx, dy, True, False)]
            else:                                    # two results each
                mom = B.add(B.mul(tw, 0.9), dw); outs += [mom, B.sub(tw, B.mul(mom, 0.1))]
                mb = B.add(B.mul(tb, 0.9), db); outs += [mb, B.gelu(mb)]
            return outs + [tw, tb]
        got = prog(ctx)
        info = ctx.barrier()
        shared += info.n_launches < info.n_regions
        E = Eager("f64")
        for j, (a, r) in enumerate(zip(got, prog(E))):
            ga, ra = np.asarray(ctx.fetch(a), np.float64), np.asarray(E.fetch(r), np.float64)
            err = float(np.max(np.abs(ga - ra))) / max(float(np.max(np.abs(ra))), 1e-3)
            assert np.isfinite(ga).all() and err <= 3e-5, (seed, (m, k, n), variant, mean, computed_dy, j, err)   # (sums of up to 1024 terms)
        del got
    assert shared >= 30


def test_c2_mlp_training_teacher_forced(ctx):
    """Every step starts from the oracle's weights, so errors cannot accumulate: 1e-5 per step."""
    E = Eager()
    inp = c2_inputs(steps=3)
    names = ("W1", "b1", "W2", "b2", "W3", "b3")
    rp = [E.tensor(inp[k]) for k in names]
    for step in range(3):
        gp = [ctx.tensor(E.fetch(p).copy(), donatable=True) for p in rp]
        lg = programs.c2_step(ctx, ctx.tensor(inp["X"][step]), ctx.tensor(inp["labels"][step]), gp, 0.01)
        info = ctx.barrier()
        lr_ = programs.c2_step(E, E.tensor(inp["X"][step]), E.tensor(inp["labels"][step]), rp, 0.01)
        assert info.cache_hit == (step > 0)
        check(ctx, E, lg, lr_, TOL32, "loss")
        for g, r, k in zip(gp, rp, names):
            # compare the update itself, which is what the step computes
            check(ctx, E, g, r, TOL32, k)
    assert ctx.dump_plan().count("->p") == 6


def test_c2_mlp_training_free_running(ctx):
    E = Eager()
    steps = 20
    inp = c2_inputs(steps=steps)
    names = ("W1", "b1", "W2", "b2", "W3", "b3")
    gp = [ctx.tensor(inp[k].copy(), donatable=True) for k in names]
    rp = [E.tensor(inp[k]) for k in names]
    hits = []
    for step in range(steps):
        lg = programs.c2_step(ctx, ctx.tensor(inp["X"][step]), ctx.tensor(inp["labels"][step]), gp, 0.01)
        hits.append(ctx.barrier().cache_hit)
        lr_ = programs.c2_step(E, E.tensor(inp["X"][step]), E.tensor(inp["labels"][step]), rp, 0.01)
        assert abs(float(ctx.fetch(lg)) - float(E.fetch(lr_))) <= 1e-4 * abs(float(E.fetch(lr_)))
    assert hits[1:] == [1] * (steps - 1)       # (the first step may hit a plan cached by an earlier test)
    # Free-running, a pre-activation within rounding distance of zero can fall on different sides
    # of the ReLU in the two implementations; one flipped unit changes that step's gradient by a
    # whole column, which is ~1e-4 of a weight matrix but ~5e-3 of the (tiny, zero-initialised)
    # bias vectors.  The per-step arithmetic is pinned at 1e-5 by the teacher-forced test above.
    for g, r, k in zip(gp, rp, names):
        check(ctx, E, g, r, 1e-3 if k.startswith("W") else 2e-2, k)


def test_c5_dynamic_shapes_and_host_control_flow(ctx):
    E = Eager()
    d = 256
    inp = c5_inputs(d=d, steps=12, batches=(8, 16, 32, 136))
    gW = [ctx.tensor(w) for w in inp["W"]]; gb = [ctx.tensor(w) for w in inp["b"]]
    gWr = [ctx.tensor(w) for w in inp["Wr"]]; gbr = [ctx.tensor(w) for w in inp["br"]]
    rW = [E.tensor(w) for w in inp["W"]]; rb = [E.tensor(w) for w in inp["b"]]
    rWr = [E.tensor(w) for w in inp["Wr"]]; rbr = [E.tensor(w) for w in inp["br"]]
    seen, misses = set(), 0
    for step in range(12):
        batch = int(inp["batch"][step])
        X = c5_batch(step, batch, d)
        word = ctx.tensor(np.array([inp["word"][step]], np.int32))
        depth = 1 + int(ctx.fetch(word)[0]) % 8          # data-dependent host branch: a trace break
        assert depth == 1 + int(inp["word"][step]) % 8
        s, h = programs.c5_forward(ctx, ctx.tensor(X), gW, gb, gWr, gbr, depth)
        info = ctx.barrier()
        misses += 0 if info.cache_hit else 1
        assert info.cache_hit == ((batch, depth) in seen)
        seen.add((batch, depth))
        sr, hr = programs.c5_forward(E, E.tensor(X), rW, rb, rWr, rbr, depth)
        check(ctx, E, h, hr, TOL32, f"h step {step}")
        check(ctx, E, s, sr, TOL32, f"checksum step {step}")
        assert info.n_regions == 4 + depth + 1
    assert misses == len(seen)


@pytest.mark.parametrize("batch,depth", [(8, 1), (8, 8), (32, 4), (64, 8), (128, 8), (256, 8), (1024, 1), (1024, 8)])
def test_c5_full_width(batch, depth):
    """The configured width (d = 2048) at the smallest, a middle and the largest batch size and at
    both ends of the depth range: the 64 x 64 and the 128 x 128 fp32 contraction tiles with the
    bias + GELU (+ residual) post program, every element of h and the checksum."""
    from paper_2102_13267_amd import Context
    d = 2048
    ctx = Context(device=0, workspace_bytes=1 << 30)
    E = Eager()
    inp = c5_inputs(d=d, steps=1)
    gW = [ctx.tensor(w) for w in inp["W"]]; gb = [ctx.tensor(w) for w in inp["b"]]
    gWr = [ctx.tensor(w) for w in inp["Wr"]]; gbr = [ctx.tensor(w) for w in inp["br"]]
    X = c5_batch(batch + depth, batch, d)
    s, h = programs.c5_forward(ctx, ctx.tensor(X), gW, gb, gWr, gbr, depth)
    info = ctx.barrier()
    assert info.n_regions == 4 + depth + 1
    got_h, got_s = ctx.fetch(h), ctx.fetch(s)
    ctx.close()
    sr, hr = programs.c5_forward(E, E.tensor(X), *([E.tensor(w) for w in inp[k]] for k in ("W", "b", "Wr", "br")), depth)
    for got, ref, what in ((got_h, E.fetch(hr), "h"), (got_s, E.fetch(sr), "checksum")):
        err = rel_err(got, ref)
        note(got, ref, TOL32, err)
        assert err <= TOL32, (what, batch, depth, err)


def _c3_setup(B, mk, cfg):
    from workloads.inputs import c3_inputs
    bsz, seq, d, ffn, heads = cfg
    inp = c3_inputs(bsz, seq, d, ffn)
    keys = programs.C3_WEIGHTS + programs.C3_VECTORS
    P = {k: mk(round_to_bf16(inp[k]), "bf16", True) for k in keys}
    M = {k: mk(np.zeros_like(inp[k]), "f32", True) for k in keys}
    V = {k: mk(np.zeros_like(inp[k]), "f32", True) for k in keys}
    x, dy = mk(round_to_bf16(inp["x"]), "bf16", False), mk(round_to_bf16(inp["dy"]), "bf16", False)
    return x, dy, P, M, V, heads


@pytest.mark.parametrize("cfg", [(2, 16, 64, 128, 4), (3, 40, 192, 320, 6), (8, 256, 1024, 4096, 16)])
def test_c3_transformer_layer_forward_backward_adam(ctx, cfg):
    """bf16 activations and weights, fp32 accumulation and Adam moments; 2e-2 per tensor.
    Two steps: the second is a cache hit and runs on the updated (donated) parameters.
    The last case has the configured widths (d_model 1024, FFN 4096, 16 heads, sequences of 256) at
    a quarter of the batch, one step: every gradient and parameter through the split contractions
    with the fused Adam pass and the column reductions, as at full size."""
    E = Eager()
    g = _c3_setup(ctx, lambda a, dt, don: ctx.tensor(a, dtype=dt, donatable=don), cfg)
    r = _c3_setup(E, lambda a, dt, don: E.tensor(a, dtype=dt), cfg)
    for step in range(1 if cfg[2] >= 1024 else 2):
        yg, dxg = programs.c3_step(ctx, *g, t=step + 1)
        info = ctx.barrier()
        yr, dxr = programs.c3_step(E, *r, t=step + 1)
        assert info.cache_hit == (step > 0)
        check(ctx, E, yg, yr, TOL16, "y")
        check(ctx, E, dxg, dxr, TOL16, "dx")
        for k in programs.C3_WEIGHTS + programs.C3_VECTORS:
            if k == "bk":
                # Softmax is invariant to a shift of its row, so the key bias has an exactly zero
                # gradient: what both sides hold there is rounding noise, small against a live
                # gradient of the same shape (the query bias), and not comparable element-wise.
                live = np.max(np.abs(E.fetch(r[3]["bq"])))
                assert np.max(np.abs(E.fetch(r[3][k]))) <= 0.1 * live
                assert np.max(np.abs(ctx.fetch(g[3][k]))) <= 0.1 * live
            else:
                check(ctx, E, g[3][k], r[3][k], TOL16, f"m[{k}] step {step}")     # first moment = the gradient
                check(ctx, E, g[4][k], r[4][k], 2 * TOL16, f"v[{k}] step {step}")  # squares double the relative error
            # With zero moments Adam's first steps are sign descent: an element whose gradient is
            # pure rounding noise moves by +lr in one implementation and -lr in the other.  So the
            # parameters are held to  2.2 lr per step + one bf16 ulp  in absolute terms; the gradients
            # themselves (m, v above) carry the 2e-2 parity.
            ref_p = E.fetch(r[2][k]).astype(np.float64)
            got_p = ctx.fetch(g[2][k]).astype(np.float64)
            bound = 2.2e-3 * (step + 1) + 2.0 ** -8 * max(np.max(np.abs(ref_p)), 1e-30)   # lr = 1e-3, per step taken
            assert np.max(np.abs(got_p - ref_p)) <= bound, (k, step, np.max(np.abs(got_p - ref_p)), bound)
            strong = np.abs(E.fetch(r[3][k])) > 0.05 * np.max(np.abs(E.fetch(r[3][k])))
            if step == 0 and k != "bk" and strong.any():
                # where the first gradient is clearly non-zero the sign, hence the step, is fixed:
                # there the new parameter agrees to 2 bf16 ulps (of the value or of the lr-sized step)
                ulp = 2.0 ** -7 * np.maximum(np.abs(ref_p[strong]), 1e-3)
                assert np.all(np.abs(got_p[strong] - ref_p[strong]) <= 2 * ulp), (k, step)
    plan = ctx.dump_plan()
    assert plan.count("->p") == 48                          # 16 parameters x (p, m, v) updated in place
    assert " EW " not in plan.replace("R41 EW", "") or plan.count(" EW ") <= 2   # no stray copy kernels for the head split / merge


# ---- full sizes, in the launch configurations that bench.py times ---------------------------------
def test_c4_full_size_sampled():
    """268,435,456 parameters (the headline configuration).  The clipping coefficient needs the
    whole gradient, so the oracle reduces all of it; the Adam chain is then elementwise and is
    checked on a sample: both ends, and 2^18 positions spread over the vector."""
    from paper_2102_13267_amd import Context
    import torch
    n = 268_435_456
    ctx = Context(device=0, workspace_bytes=64 << 20)
    inp = c4_inputs(n)
    names = ("p", "g", "m", "v")
    dev = {k: torch.from_numpy(inp[k]).to("cuda:0") for k in names}
    gt = [ctx.tensor(dev[k], donatable=(k != "g")) for k in names]
    programs.c4_step(ctx, *gt, **C4_HYPER)
    info = ctx.barrier()
    assert info.n_regions == 2 and ctx.dump_plan().count("->p") == 3
    r = rng(40)
    idx = np.unique(np.concatenate([np.arange(4096), np.arange(n - 4096, n), r.integers(0, n, 1 << 18)]))
    E = Eager()
    gnorm = E.sqrt(E.sum(E.square(E.tensor(inp["g"]))))                       # the oracle over all of g
    clip = E.minimum(1.0, E.div(C4_HYPER["max_norm"], E.add(gnorm, 1e-6)))
    rs = {k: E.tensor(inp[k][idx]) for k in names}
    hyper = {k: v for k, v in C4_HYPER.items() if k != "max_norm"}
    programs.adam_update(E, rs["p"], rs["g"], rs["m"], rs["v"], clip=clip, **hyper)
    for k, t in zip(names, gt):
        if k == "g":
            continue
        got = dev[k][torch.from_numpy(idx).to("cuda:0")].cpu().numpy()     # donated: the caller's buffer holds the result
        assert ctx.device_ptr(t) == dev[k].data_ptr()
        assert rel_err(got, E.fetch(rs[k])) <= TOL32, k
    ctx.close()


C3_GEMMS = [  # (m, n, k, trans_a, trans_b, batch): the contraction shapes of the transformer layer
    (8192, 1024, 1024, False, False, ()),      # projections
    (8192, 4096, 1024, False, False, ()),      # FFN up
    (8192, 1024, 4096, False, True, ()),       # FFN down, backward w.r.t. its input
    (1024, 1024, 8192, True, False, ()),       # weight gradient: k split over workgroups
    (1024, 4096, 8192, True, False, ()),
    (256, 256, 64, False, True, (32, 16)),     # attention scores
    (256, 64, 256, False, False, (32, 16)),    # attention context (128 x 64 tiles)
    (256, 64, 256, True, False, (32, 16)),     # its gradients
]


@pytest.mark.parametrize("m,n,k,ta,tb,batch", C3_GEMMS)
def test_gemm_bf16_full_size_sampled(m, n, k, ta, tb, batch):
    """The bf16 contractions at C3's full sizes: 16 x 16 sampled outputs per (sampled) batch,
    each a k-long dot product the oracle computes on its own."""
    from paper_2102_13267_amd import Context
    import torch
    ctx = Context(device=0, workspace_bytes=1 << 30)
    g = torch.Generator(device="cuda:0").manual_seed(41)
    a = (torch.randn(*batch, *((k, m) if ta else (m, k)), device="cuda:0", generator=g) * 0.5).to(torch.bfloat16)
    b = (torch.randn(*batch, *((n, k) if tb else (k, n)), device="cuda:0", generator=g) * 0.5).to(torch.bfloat16)
    out = ctx.matmul(ctx.tensor(a, dtype="bf16"), ctx.tensor(b, dtype="bf16"), ta, tb, dtype="f32")
    got = ctx.fetch(out)
    r = rng(42)
    rows, cols = np.sort(r.choice(m, 16, replace=False)), np.sort(r.choice(n, 16, replace=False))
    picks = [()] if not batch else [tuple(int(r.integers(0, d)) for d in batch) for _ in range(4)]
    E = Eager()
    for bi in picks:
        an, bn = a[bi].float().cpu().numpy(), b[bi].float().cpu().numpy()
        asub = an[:, rows] if ta else an[rows, :]
        bsub = bn[cols, :] if tb else bn[:, cols]
        ref = E.fetch(E.matmul(E.tensor(asub, dtype="bf16"), E.tensor(bsub, dtype="bf16"), ta, tb, dtype="f32"))
        sub = got[bi][np.ix_(rows, cols)]
        assert rel_err(sub, ref) <= 1e-5, (m, n, k, ta, tb, bi)      # fp32 accumulator, fp32 output
    ctx.close()


def test_c3_full_size_batch_elements():
    """The transformer layer at its full size (batch 32, seq 256, d_model 1024, FFN 4096, 16 heads).
    A batch element's output and input gradient depend on that element alone, so the oracle runs
    the same program on single batch elements."""
    from paper_2102_13267_amd import Context
    from workloads.inputs import c3_inputs
    bsz, seq, d, ffn, heads = 32, 256, 1024, 4096, 16
    ctx = Context(device=0, workspace_bytes=8 << 30)
    inp = c3_inputs(bsz, seq, d, ffn)
    keys = programs.C3_WEIGHTS + programs.C3_VECTORS

    def setup(B, mk, sl):
        P = {k: mk(round_to_bf16(inp[k]), "bf16", True) for k in keys}
        M = {k: mk(np.zeros_like(inp[k]), "f32", True) for k in keys}
        V = {k: mk(np.zeros_like(inp[k]), "f32", True) for k in keys}
        return mk(round_to_bf16(inp["x"][sl]), "bf16", False), mk(round_to_bf16(inp["dy"][sl]), "bf16", False), P, M, V, heads
    g = setup(ctx, lambda a, dt, don: ctx.tensor(a, dtype=dt, donatable=don), slice(None))
    y, dx = programs.c3_step(ctx, *g, t=1)
    info = ctx.barrier()
    assert info.n_regions == 42
    yg, dxg = ctx.fetch(y).reshape(bsz, seq, d), ctx.fetch(dx).reshape(bsz, seq, d)
    for b in (0, 17):
        E = Eager()
        r = setup(E, lambda a, dt, don: E.tensor(a, dtype=dt), slice(b, b + 1))
        yr, dxr = programs.c3_step(E, *r, t=1)
        assert rel_err(yg[b], E.fetch(yr).reshape(seq, d)) <= TOL16, b
        assert rel_err(dxg[b], E.fetch(dxr).reshape(seq, d)) <= TOL16, b
    ctx.close()


def _many_live_values(B, x):
    """Ten values that all stay live across two chains: a program of more than eight slots."""
    u = [B.exp(B.mul(x, 0.1)), B.tanh(x), B.abs(x), B.square(x), B.neg(x), B.relu(x), B.sigmoid(x),
         B.sqrt(B.abs(x)), B.mul(x, 0.5), B.add(x, 1.0)]
    s = u[0]
    for t in u[1:]:
        s = B.add(s, t)
    m = u[0]
    for t in u[1:]:
        m = B.mul(m, B.add(B.mul(t, 0.01), 1.0))
    return B.add(s, m)


@pytest.mark.parametrize("n", [4096, (1 << 20) + 8, (1 << 22)])
def test_programs_wider_than_half_a_register_file(ctx, n):
    """Reductions and elementwise regions interpret several 4-vectors per dispatch when the program
    fits a fraction of the register file; this one does not and takes the one-at-a-time path."""
    E = Eager()
    x = (rng(77).standard_normal(n) * 0.7).astype(np.float32)
    got_s = ctx.sum(_many_live_values(ctx, ctx.tensor(x)))
    got_e = _many_live_values(ctx, ctx.tensor(x))
    ref_s = E.sum(_many_live_values(E, E.tensor(x)))
    ref_e = _many_live_values(E, E.tensor(x))
    check(ctx, E, got_e, ref_e, TOL32, "elementwise")
    check(ctx, E, got_s, ref_s, TOL32, "global sum")
    x2 = x[: (n // 1024) * 1024].reshape(-1, 1024) if n >= 1024 else x.reshape(1, -1)
    got_c = ctx.sum(_many_live_values(ctx, ctx.tensor(x2)), axis=0)
    ref_c = E.sum(_many_live_values(E, E.tensor(x2)), axis=0)
    check(ctx, E, got_c, ref_c, TOL32, "column sum")


def _stream_case(c, x_np, w_np, w2_np, p_np):
    """Independent launches with every kind of hazard between them: a wide column reduction next to
    contractions, a consumer of the reduction, five reductions sharing the scratch, and an in-place
    update of a tensor that a reduction on another stream reads."""
    x, w, w2 = c.tensor(x_np), c.tensor(w_np), c.tensor(w2_np)
    p = c.tensor(p_np.copy(), donatable=True)
    y0 = c.matmul(x, w)
    s = c.sum(c.square(x), axis=0)
    z = c.add(c.matmul(x, w2), s)
    sums = [c.sum(c.mul(x, float(k + 2)), axis=0) for k in range(5)]
    colsum = c.sum(c.abs(p), axis=0)
    c.assign(p, c.mul(p, 0.5))
    return [y0, s, z, colsum, p] + sums


def test_streams_do_not_change_results():
    """The same plan on one stream and on four: bit-identical results (the kernels, grids and
    summation orders are the same; only what runs next to what differs), three steps each so that
    events and scratch quarters are reused; the first step is also held against the oracle."""
    from paper_2102_13267_amd import Context
    g = rng(2024)
    x = g.standard_normal((4096, 1024)).astype(np.float32)
    w = (g.standard_normal((1024, 512)) * 0.03).astype(np.float32)
    w2 = (g.standard_normal((1024, 1024)) * 0.03).astype(np.float32)
    p = g.standard_normal((4096, 1024)).astype(np.float32)
    results = {}
    for n_streams in (1, 4):
        c = Context(device=0, workspace_bytes=1 << 30)
        c.set_streams(n_streams)
        steps = []
        for step in range(3):
            outs = _stream_case(c, x, w, w2, p)
            c.barrier()
            if n_streams == 4 and step == 0:
                sched = c.dump_schedule()
                assert "stream=1" in sched or "stream=2" in sched, sched
            steps.append([c.fetch(t).copy() for t in outs])
        results[n_streams] = steps
        c.close()
    for a_step, b_step in zip(results[1], results[4]):
        for a, b in zip(a_step, b_step):
            assert np.array_equal(a, b)
    E = Eager()
    ref = _stream_case(E, x, w, w2, p)
    for got, r in zip(results[4][0], ref):
        assert rel_err(got, E.fetch(r)) <= TOL32


def _random_large_trace(c, g, mats, sq, vec):
    """A random trace over large tensors (contractions, elementwise chains, row / column / global
    reductions, a row operator, in-place updates of donated buffers); returns what it keeps."""
    rows, cols = 2048, 1024
    keep = []
    for _ in range(int(g.integers(8, 14))):
        kind = int(g.integers(0, 7))
        a, b = mats[int(g.integers(0, 4))], mats[int(g.integers(0, 4))]
        if kind == 0:
            t = c.mul(c.matmul(a, sq[int(g.integers(0, 2))]), 0.03)
        elif kind == 1:
            t = c.mul(c.matmul(a, b, trans_a=True), 1e-3)
        elif kind == 2:
            t = c.tanh(c.add(c.mul(a, 0.5), b))
        elif kind == 3:
            t = c.sum(c.mul(a, b), axis=0)
        elif kind == 4:
            t = c.sum(c.square(a), axis=1)
        elif kind == 5:
            t = c.sqrt(c.sum(c.square(a)))
        else:
            t = c.softmax(a)
        if t.shape == (rows, cols) and g.random() < 0.5:
            k = int(g.integers(0, 4))
            if k < 2:
                c.assign(mats[k], t)
            else:
                mats[k] = t
        elif t.shape == (cols,) and g.random() < 0.5:
            c.assign(vec, c.add(c.mul(vec, 0.5), t))
        else:
            keep.append(t)
    return keep


@pytest.mark.parametrize("seed", range(4))
def test_random_large_traces_same_on_one_stream_and_four(seed):
    """Random traces whose launches are long enough to spread over streams, two steps each (events,
    scratch quarters and arena blocks are reused): every kept result and every buffer updated in
    place is bit-identical to the one-stream run."""
    from paper_2102_13267_amd import Context
    g0 = rng(6000 + seed)
    data = [g0.standard_normal((2048, 1024)).astype(np.float32) for _ in range(4)]
    sqd = [(g0.standard_normal((1024, 1024)) * 0.03).astype(np.float32) for _ in range(2)]
    results = {}
    for n_streams in (1, 4):
        c = Context(device=0, workspace_bytes=1 << 30)
        c.set_streams(n_streams)
        mats = [c.tensor(d.copy(), donatable=(k < 2)) for k, d in enumerate(data)]
        donated = mats[:2]
        sq = [c.tensor(d) for d in sqd]
        vec = c.tensor(np.zeros(1024, np.float32), donatable=True)
        out = []
        for step in range(2):
            keep = _random_large_trace(c, rng(7000 + seed), list(mats), sq, vec)    # the same trace both steps
            c.barrier()
            out.append([c.fetch(t).copy() for t in keep] + [c.fetch(t).copy() for t in donated] + [c.fetch(vec).copy()])
        if n_streams == 4:
            assert any(f"stream={s}" in c.dump_schedule() for s in (1, 2, 3))
        results[n_streams] = out
        c.close()
    for a_step, b_step in zip(results[1], results[4]):
        assert len(a_step) == len(b_step)
        for a, b in zip(a_step, b_step):
            assert np.array_equal(np.atleast_1d(a).view(np.uint8), np.atleast_1d(b).view(np.uint8))


def test_c3_layer_same_on_one_stream_and_four():
    """Transformer layer step at a size whose bias-gradient reductions are wide enough to leave the
    caller's stream: every output, gradient moment and parameter bit-identical to the one-stream run."""
    from paper_2102_13267_amd import Context
    from workloads.inputs import c3_inputs
    cfg = (8, 256, 1024, 2048, 16)
    bsz, seq, d, ffn, heads = cfg
    inp = c3_inputs(bsz, seq, d, ffn)
    keys = programs.C3_WEIGHTS + programs.C3_VECTORS
    results = {}
    for n_streams in (1, 4):
        c = Context(device=0, workspace_bytes=3 << 30)
        c.set_streams(n_streams)
        P = {k: c.tensor(round_to_bf16(inp[k]), dtype="bf16", donatable=True) for k in keys}
        M = {k: c.tensor(np.zeros_like(inp[k]), dtype="f32", donatable=True) for k in keys}
        V = {k: c.tensor(np.zeros_like(inp[k]), dtype="f32", donatable=True) for k in keys}
        xt, dyt = c.tensor(round_to_bf16(inp["x"]), dtype="bf16"), c.tensor(round_to_bf16(inp["dy"]), dtype="bf16")
        for step in range(2):
            y, dx = programs.c3_step(c, xt, dyt, P, M, V, heads, t=step + 1)
            c.barrier()
        if n_streams == 4:
            assert any(f"stream={s}" in c.dump_schedule() for s in (1, 2, 3))
        results[n_streams] = [c.fetch(y), c.fetch(dx)] + [c.fetch(D[k]) for D in (P, M, V) for k in keys]
        c.close()
    for a, b in zip(results[1], results[4]):
        assert np.array_equal(np.asarray(a).view(np.uint8), np.asarray(b).view(np.uint8))


@pytest.mark.parametrize("n", [8, 2048, 2056, 2052, 6 * 2048 + 24, (1 << 20) + 4])
def test_bf16_elementwise_programs(ctx, n):
    """Elementwise regions over bf16 tensors: sizes of one lane's 8 elements, one tile, a tile and a
    ragged one, a size that is not a multiple of 8 (the 4-at-a-time path), several tiles; one to
    three bf16 inputs, a device scalar, bf16 and fp32 outputs in one region."""
    E = Eager()
    g = rng(300 + n % 97)
    a, b, c = (round_to_bf16(g.standard_normal(n, dtype=np.float32)) for _ in range(3))
    s = np.array(0.75, np.float32)

    def prog(B, a, b, c, s):
        u = B.gelu(B.add(a, b))                              # bf16 in, bf16 out
        v = B.cast(B.mul(B.add(B.mul(a, c), u), s), "f32")   # three inputs, a device scalar, fp32 out
        w = B.add(a, b)                                      # the bare residual add
        return u, v, w

    got = prog(ctx, *(ctx.tensor(t, dtype="bf16") for t in (a, b, c)), ctx.tensor(s))
    ref = prog(E, *(E.tensor(t, dtype="bf16") for t in (a, b, c)), E.tensor(s))
    for gt, rt, what in zip(got, ref, "uvw"):
        check(ctx, E, gt, rt, TOL16, what)


@pytest.mark.parametrize("rows,cols", [(1, 8), (3, 24), (256, 8), (77, 1024), (5, 4104), (1300, 1032), (2600, 1032), (4096, 256), (6, 12)])
def test_bf16_elementwise_with_row_vectors(ctx, rows, cols):
    """bf16 regions that mix full tensors with row vectors (a bias, a scale): rows of 8-element
    groups go through the streamed kernel, which reads a row vector at the lane's column and
    moves the column on by the grid stride modulo the row length -- one tile, many tiles per
    workgroup ((2600, 1032) is 1311 tiles for 1024 workgroups), a ragged last tile, rows longer and shorter than a
    tile, two row vectors and no full tensor at all; (6, 12) is not whole groups of 8 and takes
    the general kernel.  In-place update of the full input among the outputs."""
    E = Eager()
    g = rng(900 + rows + cols)
    x = round_to_bf16(g.standard_normal((rows, cols), dtype=np.float32))
    y = round_to_bf16(g.standard_normal((rows, cols), dtype=np.float32))
    bias = round_to_bf16(g.standard_normal(cols, dtype=np.float32))
    scale = round_to_bf16(1.0 + 0.1 * g.standard_normal(cols, dtype=np.float32))

    def prog(B, x, y, bias, scale):
        u = B.gelu(B.add(x, bias))                       # one full tensor, one row vector
        v = B.add(B.mul(B.add(x, y), scale), bias)       # two full tensors, two row vectors
        w = B.mul(B.expand(B.add(bias, scale), (rows, cols)), 0.5)   # row vectors only
        B.assign(y, B.sub(y, B.mul(bias, 0.25)))          # in place over a full input
        return u, v, w, y

    gx, gy = ctx.tensor(x, dtype="bf16"), ctx.tensor(y.copy(), dtype="bf16", donatable=True)
    got = prog(ctx, gx, gy, ctx.tensor(bias, dtype="bf16"), ctx.tensor(scale, dtype="bf16"))
    ref = prog(E, E.tensor(x, dtype="bf16"), E.tensor(y, dtype="bf16"), E.tensor(bias, dtype="bf16"), E.tensor(scale, dtype="bf16"))
    ctx.barrier()
    for gt, rt, what in zip(got, ref, "uvwy"):
        check(ctx, E, gt, rt, TOL16, what)


@pytest.mark.parametrize("n", [4, 1024, 1028, 2048, 3072, 5 * 1024 + 8, (1 << 20) + 1024])
def test_streamed_fp32_elementwise_tile_pairs(ctx, n):
    """The streamed fp32 elementwise kernel takes two 1024-element tiles per workgroup: a single
    tile, a tile and a ragged one, an odd number of tiles (the last one is its own partner), one to
    four plain inputs, two device scalars, an in-place update among the outputs."""
    E = Eager()
    g = rng(500 + n % 89)
    arrs = [g.standard_normal(n).astype(np.float32) for _ in range(4)]
    s1, s2 = np.array(0.25, np.float32), np.array(-1.5, np.float32)

    def prog(B, a, b, c, d, s1, s2):
        one = B.tanh(a)                                            # one input
        two = B.add(B.mul(a, b), s1)                               # two inputs, one device scalar
        four = B.sub(B.mul(B.add(a, b), B.mul(c, s2)), B.mul(d, s1))   # four inputs, two device scalars
        B.assign(d, B.add(B.mul(d, 0.5), c))                       # in place
        return one, two, four, d

    lt = [ctx.tensor(x.copy(), donatable=(i == 3)) for i, x in enumerate(arrs)]
    et = [E.tensor(x.copy(), donatable=(i == 3)) for i, x in enumerate(arrs)]
    got = prog(ctx, *lt, ctx.tensor(s1), ctx.tensor(s2))
    ref = prog(E, *et, E.tensor(s1), E.tensor(s2))
    for gt, rt, what in zip(got, ref, ("one", "two", "four", "in place")):
        check(ctx, E, gt, rt, TOL32, what)


def _random_trace(B, rg, base, allow_matmul):
    """A random DAG over three inputs: well-conditioned elementwise ops, reductions over every axis
    kind, an occasional contraction, in-place updates of the inputs, dropped intermediates.
    Decisions are drawn from `rg` only, so two back ends given equal seeds build the same trace."""
    unary = ["neg", "abs", "tanh", "relu", "gelu", "square", "sigmoid"]
    binary = ["add", "sub", "mul", "maximum", "minimum"]
    vals = list(base)
    full = list(base)
    for _ in range(int(rg.integers(6, 22))):
        kind = int(rg.integers(0, 12))
        pick = lambda: full[int(rg.integers(0, len(full)))]
        if kind < 3:
            r = getattr(B, unary[int(rg.integers(0, len(unary)))])(pick())
        elif kind < 7:
            a, b = pick(), pick()
            name = binary[int(rg.integers(0, len(binary)))]
            if rg.integers(0, 3) == 0:
                r = getattr(B, name)(a, [0.0, 1.0, 0.5, -2.0][int(rg.integers(0, 4))])
            elif a.shape == b.shape or len(b.shape) == 0 or (len(a.shape) == 2 and b.shape in ((a.shape[1],), (a.shape[0], 1))):
                r = getattr(B, name)(a, b)
            else:
                continue
        elif kind < 9:
            a = pick()
            if len(a.shape) == 0:
                continue
            axis = [None, -1, 0][int(rg.integers(0, 3))]
            if axis == 0 and len(a.shape) != 2:
                axis = None
            r = getattr(B, ["sum", "amax", "mean"][int(rg.integers(0, 3))])(B.mul(a, 0.01), axis)
        elif kind == 9 and allow_matmul:
            a, b = pick(), pick()
            if len(a.shape) != 2 or a.shape != b.shape:
                continue
            r = B.mul(B.matmul(a, b, trans_a=True), 1.0 / a.shape[0])       # [cols, cols]
        elif kind >= 10:
            dst, src = vals[int(rg.integers(0, len(vals)))], pick()
            if tuple(dst.shape) != tuple(src.shape) or dst is src:
                continue
            B.assign(dst, src)
            continue
        else:
            continue
        full.append(r)
        if rg.integers(0, 3) == 0 and len(full) > 6:
            full.pop(int(rg.integers(len(vals), len(full))))
    return full


@pytest.mark.parametrize("first", [0, 100, 200])
def test_random_small_traces_with_views_and_windows(ctx, first):
    """The random traces of the plan-validity test (every broadcast kind, reductions over each axis,
    expand / reshape / permute / narrow as ops and as views with write-back, window updates,
    contractions, folding-prone scalars, dropped handles, in-place updates) on small operands with
    values: every live tensor after the barrier against the fp64 oracle.  Bar: 1e-5 plus twenty
    times the distance of the fp32 oracle from the fp64 one (a division by a near-zero product
    amplifies rounding in any implementation; for most tensors that distance is ~1e-7).  The scale
    of a comparison has a floor of 1e-2: a result that is itself rounding-sized (GELU of a large
    negative sum) is held to an absolute 1e-7."""
    from test_plan_validity import random_trace
    for seed in range(first, first + 100):
        g = rng(50000 + seed)
        data = []

        def mk(shape, dtype="f32", donatable=False):
            data.append((g.standard_normal(shape) * 0.5).astype(np.float32))
            return ctx.tensor(data[-1].copy(), donatable=donatable)
        # a trace with an op pattern that has no lowering would stay pending in the shared context:
        # such seeds are found on the null device first and left out
        from paper_2102_13267_amd import Context, LtError
        dry = Context(device=None)
        keep = random_trace(seed)(dry, lambda shape, dtype="f32", donatable=False: dry.from_device(0, "f32", shape, donatable))
        try:
            dry.barrier()
        except LtError as e:
            assert e.status == 5 and "internal" not in str(e), (seed, e)
            continue
        finally:
            del keep
        got = random_trace(seed)(ctx, mk)
        ctx.barrier()
        E, E64 = Eager(), Eager("f64")
        it, it64 = iter(data), iter(data)
        ref = random_trace(seed)(E, lambda shape, dtype="f32", donatable=False: E.tensor(next(it).copy(), donatable=donatable))
        ref64 = random_trace(seed)(E64, lambda shape, dtype="f32", donatable=False: E64.tensor(next(it64).copy(), donatable=donatable))
        assert len(got) == len(ref) == len(ref64)
        for k, (a, b, c) in enumerate(zip(got, ref, ref64)):
            ga, rb, rc = (np.asarray(x, np.float64) for x in (ctx.fetch(a), E.fetch(b), E64.fetch(c)))
            assert ga.shape == rb.shape, (seed, k)
            fin = np.isfinite(rb) & np.isfinite(rc) & (np.abs(rc) < 1e30)     # (exp and div chains overflow fp32 now and then)
            assert np.isfinite(ga[fin]).all(), (seed, k)
            if fin.any():
                scale = max(float(np.max(np.abs(rc[fin]))), 1e-2)
                # how far fp32 arithmetic in the recorded order is from the exact result: a division
                # by a near-zero product amplifies rounding in any implementation
                cond = float(np.max(np.abs(rb[fin] - rc[fin]))) / scale
                tol = TOL32 + 20.0 * cond
                err = float(np.max(np.abs(ga[fin] - rc[fin]))) / scale
                note(ga[fin], rc[fin], tol, err)
                assert err <= tol, (seed, k, err, cond)
        del got, ref, ref64


@pytest.mark.parametrize("shape,trials", [((8, 16), 12), ((100, 257), 8), ((1024, 1024), 6), ((4096, 1024), 4)])
def test_random_traces_numeric(ctx, shape, trials):
    """Random traces, the same on both sides, every live tensor compared after the barrier.  The
    larger shapes reach the streamed kernels, the several-vectors-per-dispatch interpreter paths
    and (4096 x 1024: column reductions of 16 MiB) the side streams."""
    for trial in range(trials):
        seed = 9000 + 31 * trial + shape[0]
        g = rng(seed)
        arrs = [g.standard_normal(shape).astype(np.float32) * 0.5, g.standard_normal(shape).astype(np.float32) * 0.5,
                g.standard_normal(shape[1]).astype(np.float32)]
        E = Eager()
        lt = [ctx.tensor(a.copy(), donatable=(i == 0)) for i, a in enumerate(arrs)]
        et = [E.tensor(a.copy(), donatable=(i == 0)) for i, a in enumerate(arrs)]
        got = _random_trace(ctx, rng(seed + 1), lt, allow_matmul=shape[0] >= 100)
        ref = _random_trace(E, rng(seed + 1), et, allow_matmul=shape[0] >= 100)
        assert len(got) == len(ref)
        ctx.barrier()
        for k, (a, b) in enumerate(zip(got, ref)):
            ga, rb = ctx.fetch(a), E.fetch(b)
            err = rel_err(ga, rb)
            note(ga, rb, TOL32, err)
            assert err <= TOL32, (shape, trial, k, err)
        del got, ref, lt, et


def test_epilogue_member_numbered_before_the_anchor(ctx):
    """`anchor(...) - 0.5 * v`: operands are numbered last to first, so the product that only the
    epilogue reads gets a smaller canonical number than the reduction / contraction it joins."""
    E = Eager()
    g = rng(77)
    a, w, r = (g.standard_normal(s).astype(np.float32) for s in ((96, 40), (40, 24), (96, 24)))
    x, v, c = g.standard_normal((96, 40)).astype(np.float32), g.standard_normal(96).astype(np.float32), g.standard_normal(40).astype(np.float32)

    def prog(B, a, w, r, x, v, c):
        y = B.add(B.matmul(a, w), B.mul(r, 0.5))
        z = B.sub(B.sum(x, axis=1), B.mul(v, 0.5))
        u = B.sub(B.sum(x, axis=0), B.mul(c, 0.25))
        t = B.sub(B.sum(B.square(x)), B.mul(B.sum(v), 2.0))
        return y, z, u, t

    got = prog(ctx, *(ctx.tensor(t) for t in (a, w, r, x, v, c)))
    ref = prog(E, *(E.tensor(t) for t in (a, w, r, x, v, c)))
    info = ctx.barrier()
    assert info.n_regions <= 5
    for gt, rt, what in zip(got, ref, "yzut"):
        check(ctx, E, gt, rt, TOL32, what)


@pytest.mark.parametrize("rows,cols", [(128, 10), (1, 1), (5, 3), (1000, 7), (64, 64), (1023, 64), (300, 33), (4, 61), (130, 12)])
def test_column_reductions_of_narrow_matrices(ctx, rows, cols):
    """Axis-0 reductions of small matrices of at most 64 columns take a path of their own (a
    thread per column and row residue, four rows per interpreter dispatch, one workgroup): one
    column, fewer rows than a dispatch takes, a column count that does not divide the workgroup,
    the largest column count, more rows than threads; sum / max / mean; a prologue with a row
    vector, a column vector and a scalar; an epilogue; bf16 and int inputs."""
    E = Eager()
    g = rng(1300 + rows * 7 + cols)
    x = g.standard_normal((rows, cols)).astype(np.float32)
    y = round_to_bf16(g.standard_normal((rows, cols), dtype=np.float32))
    rv = g.standard_normal(cols).astype(np.float32)
    cv = g.standard_normal((rows, 1)).astype(np.float32)
    k = g.integers(-5, 6, (rows, cols)).astype(np.int32)

    def prog(B, x, y, rv, cv, k):
        s = B.sum(x, axis=0)                                                     # the bare operand
        m = B.amax(B.mul(B.add(x, rv), B.expand(cv, (rows, cols))), axis=0)      # row and column vectors in the prologue
        a = B.sub(B.mean(B.mul(B.tanh(x), B.cast(y, "f32")), axis=0), B.mul(rv, 0.5))   # bf16 input, an epilogue
        i = B.sum(B.mul(B.cast(k, "f32"), 2.0), axis=0)                          # integer input
        return s, m, a, i

    got = prog(ctx, ctx.tensor(x), ctx.tensor(y, dtype="bf16"), ctx.tensor(rv), ctx.tensor(cv), ctx.tensor(k))
    ref = prog(E, E.tensor(x), E.tensor(y, dtype="bf16"), E.tensor(rv), E.tensor(cv), E.tensor(k))
    tol = 2e-5 * max(1.0, rows ** 0.5 / 8)   # (partial sums of `rows` terms against max|ref| of a cancelling sum)
    for gt, rt, what in zip(got, ref, ("sum", "max", "mean", "int")):
        check(ctx, E, gt, rt, tol, what)


@pytest.mark.parametrize("rows,cols,dtype", [(8, 256, "f32"), (67, 512, "f32"), (64, 1024, "bf16"), (521, 768, "bf16"),
                                              (2048, 1024, "bf16"), (300, 260, "f32"), (130, 250, "bf16")])
def test_column_reductions_with_per_row_inputs(ctx, rows, cols, dtype):
    """Column sums whose program reads per-row vectors next to whole tensors (the weight gradient
    of a layer norm): row counts below, at and between multiples of what the waves of a workgroup
    fetch per trip, one and two whole inputs, one and two per-row inputs, fp32 and bf16; the last
    two shapes (cols not a multiple of 256, of 4) take the general path."""
    E = Eager()
    g = rng(700 + rows + cols)
    conv = round_to_bf16 if dtype == "bf16" else (lambda t: t)
    dy, x = (conv(g.standard_normal((rows, cols), dtype=np.float32)) for _ in range(2))
    mu, rs = g.standard_normal(rows, dtype=np.float32), (g.random(rows, dtype=np.float32) + 0.5)

    def prog(B, dy, x, mu, rs):
        mu2, rs2 = B.reshape(mu, (rows, 1)), B.reshape(rs, (rows, 1))
        xhat = B.mul(B.sub(x, mu2), rs2)
        dgamma = B.sum(B.mul(dy, xhat), axis=0)              # two whole inputs, two per-row inputs
        centred = B.sum(B.sub(x, mu2), axis=0)               # one whole input, one per-row input
        scaled = B.amax(B.mul(B.mul(dy, x), rs2), axis=0)    # another reduction, per-row input last
        return dgamma, centred, scaled

    got = prog(ctx, ctx.tensor(dy, dtype=dtype), ctx.tensor(x, dtype=dtype), ctx.tensor(mu), ctx.tensor(rs))
    ref = prog(E, E.tensor(dy, dtype=dtype), E.tensor(x, dtype=dtype), E.tensor(mu), E.tensor(rs))
    tol = TOL16 if dtype == "bf16" else 2e-5 * max(1.0, rows ** 0.5 / 8)
    for gt, rt, what in zip(got, ref, ("dgamma", "centred", "scaled")):
        check(ctx, E, gt, rt, tol, what)
