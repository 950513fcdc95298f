"""The plans of the library (null device) and of the structural oracle, put through a checker that
shares nothing with either lowering (tests/plan_check.py): whatever the two agree on must also be a
partition that computes the trace.  No GPU."""
import numpy as np
import pytest

from oracle.structural import Tracer
from paper_2102_13267_amd import Context
from plan_check import PlanError, check_plan
from workloads import programs
from workloads.inputs import C4_HYPER, c3_inputs


def lib_plan(ctx):
    info = ctx.barrier()
    return ctx.dump_key(), info.n_nodes, ctx.dump_plan()


def both(build):
    """Run `build(B, mk)` on the library's null device and on the oracle; check both plans."""
    ctx = Context()
    keep = build(ctx, lambda shape, dtype="f32", donatable=False: ctx.tensor(
        np.zeros(shape, {"s32": np.int32}.get(dtype, np.float32)), dtype=dtype, donatable=donatable))
    key, n, plan = lib_plan(ctx)
    res = check_plan(key, n, plan)
    T = Tracer()
    keep2 = build(T, lambda shape, dtype="f32", donatable=False: T.tensor(shape, dtype, donatable=donatable))
    ref = T.barrier()
    check_plan(ref["bytes"], ref["n_nodes"], ref["plan"])
    del keep, keep2
    return key, n, plan, res


def c1(B, mk):
    return programs.c1_trace(B, mk((1024, 1024)), mk((1024, 1024)), mk((1024,)))


def c2(B, mk):
    dims = (784, 512, 512, 10)
    params = []
    for i in range(3):
        params += [mk((dims[i], dims[i + 1]), donatable=True), mk((dims[i + 1],), donatable=True)]
    return programs.c2_step(B, mk((128, 784)), mk((128,), "s32"), params, 0.01), params


def c3(B, mk):
    bsz, seq, d, ffn, heads = 2, 16, 64, 128, 4
    inp = c3_inputs(bsz, seq, d, ffn)
    keys = programs.C3_WEIGHTS + programs.C3_VECTORS
    W = {k: mk(inp[k].shape, "bf16", True) for k in keys}
    M = {k: mk(inp[k].shape, "f32", True) for k in keys}
    V = {k: mk(inp[k].shape, "f32", True) for k in keys}
    return programs.c3_step(B, mk(inp["x"].shape, "bf16"), mk(inp["dy"].shape, "bf16"), W, M, V, heads), W, M, V


def c4(B, mk):
    ts = [mk((1 << 17,), donatable=True) for _ in range(4)]
    programs.c4_step(B, *ts, **C4_HYPER)
    return ts


def c5(B, mk):
    d = 64
    return programs.c5_forward(B, mk((16, d)), [mk((d, d)) for _ in range(4)], [mk((d,)) for _ in range(4)],
                               [mk((d, d)) for _ in range(8)], [mk((d,)) for _ in range(8)], 5)


@pytest.mark.parametrize("build", [c1, c2, c3, c4, c5])
def test_plans_of_the_five_configurations_are_valid(build):
    both(build)


def random_trace(seed):
    """Elementwise ops with every broadcast kind, reductions over each axis, views (expand, reshape,
    permute), contractions, folding-prone scalars, dropped handles and in-place updates."""
    def build(B, mk):
        rg = np.random.Generator(np.random.PCG64(seed))
        base = [mk((8, 16), donatable=bool(rg.integers(0, 2))) for _ in range(3)] + [mk((16,), donatable=True), mk((8, 1))]
        pool = list(base)
        sq = [mk((16, 16)), mk((16, 8))]
        unary = ["neg", "abs", "exp", "tanh", "relu", "gelu", "square", "sigmoid"]
        binary = ["add", "sub", "mul", "div", "maximum", "minimum"]
        for _ in range(int(rg.integers(4, 30))):
            kind = int(rg.integers(0, 17))
            pick = lambda: pool[int(rg.integers(0, len(pool)))]
            try:
                if kind < 3:
                    r = getattr(B, unary[int(rg.integers(0, len(unary)))])(pick())
                elif kind < 7:
                    name = binary[int(rg.integers(0, len(binary)))]
                    if rg.integers(0, 3) == 0:
                        r = getattr(B, name)(pick(), [0.0, 1.0, 0.5, 2.0][int(rg.integers(0, 4))])
                    else:
                        r = getattr(B, name)(pick(), pick())
                elif kind < 9:
                    a = pick()
                    axis = [None, -1, 0][int(rg.integers(0, 3))]
                    if len(a.shape) != 2 and axis == 0:
                        axis = None
                    if len(a.shape) == 0:
                        continue
                    r = getattr(B, ["sum", "amax", "mean"][int(rg.integers(0, 3))])(a, axis)
                elif kind == 9:
                    a = pick()
                    if len(a.shape) != 2:
                        continue
                    r = B.permute(a, (1, 0))
                elif kind == 10:
                    a = pick()
                    if len(a.shape) != 2:
                        continue
                    r = B.reshape(a, (a.shape[1], a.shape[0])) if rg.integers(0, 2) else B.reshape(a, (a.shape[0] * a.shape[1],))
                elif kind == 11:
                    a = pick()
                    if a.shape not in ((16,), (8, 1)):
                        continue
                    r = B.expand(a, (8, 16))
                elif kind == 12:
                    a = pick()
                    if a.shape == (8, 16):
                        r = B.matmul(a, sq[int(rg.integers(0, 2))])
                    elif a.shape == (16, 8):
                        r = B.matmul(a, a, trans_b=True)
                    else:
                        continue
                elif kind == 13:
                    a = pick()
                    if a.shape != (8, 16):
                        continue
                    r = B.narrow(a, 1, int(rg.integers(0, 3)) * 4, 8) if rg.integers(0, 2) else B.narrow(a, 0, 2, 4)
                elif kind == 14:
                    a, u = pick(), pick()
                    if a.shape != (8, 16) or u.shape != (8, 1):
                        continue
                    r = B.slice_update(a, u, 1, int(rg.integers(0, 16)))
                elif kind == 15:
                    a = pick()                      # an in-place update through a view of one of the inputs
                    dst = base[int(rg.integers(0, 3))]
                    if a.shape != (8, 16):
                        continue
                    v = B.view_narrow(dst, 0, 2, 4) if rg.integers(0, 2) else B.view_permute(dst, (1, 0))
                    B.assign(v, B.narrow(a, 0, 0, 4) if v.shape == (4, 16) else B.permute(a, (1, 0)))
                    del v
                    continue
                else:
                    dst, src = base[int(rg.integers(0, len(base)))], pick()
                    if dst.shape != src.shape or dst is src:
                        continue
                    B.assign(dst, src)
                    continue
            except (ValueError, AssertionError):
                continue
            except Exception as e:              # the library's shape errors
                if type(e).__name__ != "LtError":
                    raise
                continue
            pool.append(r)
            if rg.integers(0, 3) == 0 and len(pool) > 8:
                pool.pop(int(rg.integers(len(base), len(pool))))
        return pool
    return build


@pytest.mark.parametrize("seed", range(400))
def test_random_traces_give_valid_plans(seed):
    ctx = Context()
    keep = random_trace(seed)(ctx, lambda shape, dtype="f32", donatable=False: ctx.tensor(np.zeros(shape, np.float32), donatable=donatable))
    try:
        key, n, plan = lib_plan(ctx)
    except Exception as e:
        # (an "internal: ..." message is a mistake of the lowering, never a reason to skip)
        if type(e).__name__ == "LtError" and e.status == 5 and "internal" not in str(e):
            pytest.skip("the trace has an op pattern without a lowering: " + str(e))
        raise
    check_plan(key, n, plan)
    del keep


def mutate(plan, fn):
    lines = plan.splitlines()
    fn(lines)
    return "\n".join(lines)


def test_the_checker_rejects_planted_mistakes():
    """Each mutation of a valid plan breaks one property; the checker must name every one."""
    key, n, plan, _ = both(c4)
    lines = plan.splitlines()
    assert len(lines) == 2 and "->p" in lines[1]
    bad = []
    bad.append("\n".join(reversed(lines)))                                           # consumer before producer
    bad.append(lines[0])                                                             # a region dropped
    bad.append(plan.replace("->p3", "->pX").replace("->p2", "->p3").replace("->pX", "->p2"))   # in place over another parameter
    bad.append(plan.replace("->p2", "->p0"))                                         # ... over one that was not offered
    m = lines[1].split("members=[")[1].split("]")[0].split(",")
    bad.append(plan.replace("members=[" + ",".join(m), "members=[" + ",".join(m[1:])))   # a member dropped
    i = lines[1].split("inputs=[")[1].split("]")[0].split(",")
    bad.append(plan.replace("inputs=[" + ",".join(i), "inputs=[" + ",".join(i[:-1])))    # an input dropped
    o = lines[1].split("outputs=[")[1].split("]")[0].split(",")
    bad.append(plan.replace("outputs=[" + ",".join(o) + "]", "outputs=[" + ",".join(o[:-1]) + "]").replace("," + o[-1] + "->p", ",0.0->p"))
    bad.append(plan + "\n" + lines[1].replace("R1", "R2"))                           # members in two regions
    for k, b in enumerate(bad):
        with pytest.raises(PlanError):
            check_plan(key, n, b)
    # the alias case of section 4.3: writing `a` in place while b = a * 1 is alive
    ctx = Context()
    a = ctx.tensor(np.zeros((16,), np.float32), donatable=True)
    b = ctx.mul(a, 1.0)
    ctx.assign(a, ctx.add(a, 1.0))
    key, n, plan = lib_plan(ctx)
    check_plan(key, n, plan)
    with pytest.raises(PlanError):
        check_plan(key, n, plan.replace("inplace=[]", "inplace=[" + plan.split("outputs=[")[1].split("]")[0] + "->p0]"))
    # a permutation fused with the producer of its operand
    ctx = Context()
    x, w = ctx.tensor(np.zeros((16, 8), np.float32)), ctx.tensor(np.zeros((8, 16), np.float32))
    mm = ctx.matmul(x, w)
    s = ctx.add(mm, ctx.permute(mm, (1, 0)))
    del mm
    key, n, plan = lib_plan(ctx)
    check_plan(key, n, plan)
    fused = "R0 MM anchor=2 members=[2,3,4] inputs=[1.0,0.0] outputs=[4.0] inplace=[]"
    with pytest.raises(PlanError):
        check_plan(key, n, fused)
    # an elementwise region over two shapes
    ctx = Context()
    u = ctx.exp(ctx.tensor(np.zeros((4, 8), np.float32)))
    v = ctx.exp(ctx.tensor(np.zeros((8,), np.float32)))
    key, n, plan = lib_plan(ctx)
    check_plan(key, n, plan)
    with pytest.raises(PlanError):
        check_plan(key, n, "R0 EW anchor=- members=[1,3] inputs=[0.0,2.0] outputs=[1.0,3.0] inplace=[]")
