"""lt_barrier_static (-m gpu): the barrier whose scratch lives in the library's static device array,
called through the C ABI, against lt_barrier on the same traces -- two calls in a row, the second on
a smaller input, so that what the first call left in the shared array would show."""
import numpy as np
import pytest

from oracle.numeric import Eager, round_to_bf16
from workloads import programs
from workloads.inputs import C4_HYPER, c1_inputs

pytestmark = pytest.mark.gpu


def rel_err(got, ref):
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    return float(np.max(np.abs(got - ref))) / max(float(np.max(np.abs(ref))), 1e-30)


def run_c1(ctx, barrier, rows, cols):
    inp = c1_inputs(rows, cols)
    out = programs.c1_trace(ctx, *(ctx.tensor(inp[k]) for k in ("x", "y", "bias")))
    info = barrier()
    assert info.n_regions == 2
    return ctx.fetch(out), inp


def run_c4(ctx, barrier, n):
    r = np.random.Generator(np.random.PCG64(77))
    arrs = [(r.standard_normal(n, dtype=np.float32) * 1e-2).astype(np.float32) for _ in range(4)]
    arrs[3] = np.abs(arrs[3])
    ts = [ctx.tensor(a.copy(), donatable=True) for a in arrs]
    programs.c4_step(ctx, *ts, **C4_HYPER)
    barrier()
    return [ctx.fetch(t) for t in (ts[0], ts[2], ts[3])], arrs


def run_gemm(ctx, barrier, m, k, n):
    r = np.random.Generator(np.random.PCG64(78))
    a = round_to_bf16(r.standard_normal((k, m), dtype=np.float32))
    b = round_to_bf16(r.standard_normal((k, n), dtype=np.float32))
    bias = r.standard_normal((n,), dtype=np.float32)
    out = ctx.add(ctx.matmul(ctx.tensor(a, dtype="bf16"), ctx.tensor(b, dtype="bf16"), trans_a=True, dtype="f32"), ctx.tensor(bias))
    colsum = ctx.sum(out, axis=0)
    barrier()
    return [ctx.fetch(out), ctx.fetch(colsum)], (a, b, bias)


def test_static_barrier_matches_the_barrier_and_the_oracle():
    from paper_2102_13267_amd import Context, LtError
    ctx = Context(device=0, workspace_bytes=256 << 20)
    ref_ctx = Context(device=0, workspace_bytes=256 << 20)
    E = Eager()
    # two calls in a row per kind of trace, the second smaller (and ragged)
    for rows, cols in ((1024, 1024), (300, 516)):
        got, inp = run_c1(ctx, ctx.barrier_static, rows, cols)
        want, _ = run_c1(ref_ctx, ref_ctx.barrier, rows, cols)
        assert np.array_equal(got, want)                  # same plan, same kernels, same bits
        ref = E.fetch(programs.c1_trace(E, *(E.tensor(inp[k]) for k in ("x", "y", "bias"))))
        assert rel_err(got, ref) <= 1e-5 and np.max(np.abs(got)) == 1.0
    for n in ((1 << 20) + 3, 1000):
        got, arrs = run_c4(ctx, ctx.barrier_static, n)
        want, _ = run_c4(ref_ctx, ref_ctx.barrier, n)
        rs = [E.tensor(a) for a in arrs]
        programs.c4_step(E, *rs, **C4_HYPER)
        for g, w, r in zip(got, want, (rs[0], rs[2], rs[3])):
            assert np.array_equal(g, w)
            assert rel_err(g, E.fetch(r)) <= 1e-5
    for m, k, n in ((256, 4096, 128), (100, 520, 72)):     # split over k: partial products in the scratch
        got, (a, b, bias) = run_gemm(ctx, ctx.barrier_static, m, k, n)
        want, _ = run_gemm(ref_ctx, ref_ctx.barrier, m, k, n)
        ref = E.add(E.matmul(E.tensor(a, dtype="bf16"), E.tensor(b, dtype="bf16"), trans_a=True, dtype="f32"), E.tensor(bias))
        for g, w, r in zip(got, want, (ref, E.sum(ref, axis=0))):
            assert np.array_equal(g, w)
            assert rel_err(g, E.fetch(r)) <= 1e-5
    # fp32, a long k over few tiles: the workgroups of a tile exchange partial tiles and take tickets in
    # the static array (tickets of the first call are back at zero for the second)
    for m, k, n in ((16, 2048, 512), (8, 1300, 70)):
        r = np.random.Generator(np.random.PCG64(79))
        a = r.standard_normal((m, k), dtype=np.float32); b = r.standard_normal((k, n), dtype=np.float32)
        bias = r.standard_normal((n,), dtype=np.float32)
        prog = lambda B: B.relu(B.add(B.matmul(B.tensor(a), B.tensor(b)), B.tensor(bias)))
        got_t = prog(ctx); ctx.barrier_static()
        want_t = prog(ref_ctx); ref_ctx.barrier()
        got = ctx.fetch(got_t)
        assert np.array_equal(got, ref_ctx.fetch(want_t))
        assert rel_err(got, E.fetch(prog(E))) <= 1e-5
    # a plan whose temporaries exceed the array is refused before anything runs; lt_barrier still runs it
    x = ctx.tensor(np.ones((1 << 22,), np.float32))
    y = ctx.exp(x)                                         # 16 MiB temporary (y feeds two regions)
    s = ctx.mul(y, ctx.sum(y))
    del y
    with pytest.raises(LtError) as e:
        ctx.barrier_static()
    assert e.value.status == 6 and "static scratch" in str(e.value)
    ctx.barrier()
    assert np.allclose(ctx.fetch(s)[:4], np.e * np.e * (1 << 22), rtol=1e-5)
    ctx.close()
    ref_ctx.close()
