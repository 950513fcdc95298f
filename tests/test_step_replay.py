"""A captured step run again without tracing (section 7 of the paper: tracing can be skipped when
the user guarantees the same computation).  Host bookkeeping on the null device; on the GPU the
replayed steps against the same steps traced, bit for bit, and against the eager oracle."""
import numpy as np
import pytest

from paper_2102_13267_amd import Context, LtError
from workloads import programs
from workloads.inputs import c2_inputs

NAMES = ("W1", "b1", "W2", "b2", "W3", "b3")


# ---- host logic (null device) ------------------------------------------------------------------

def _mlp_null(ctx, batch=16):
    shapes = {"W1": (32, 24), "b1": (24,), "W2": (24, 24), "b2": (24,), "W3": (24, 10), "b3": (10,)}
    params = [ctx.from_device(0, "f32", shapes[k], donatable=True) for k in NAMES]
    X = ctx.from_device(0, "f32", (batch, 32))
    labels = ctx.from_device(0, "s32", (batch,))
    return params, X, labels


def test_capture_needs_a_barrier():
    ctx = Context(device=None)
    with pytest.raises(LtError):
        ctx.capture_step()


def test_replay_bookkeeping_on_the_null_device():
    ctx = Context(device=None)
    params, X, labels = _mlp_null(ctx)
    loss = programs.c2_step(ctx, X, labels, params, 0.01)
    info = ctx.barrier()
    plan = ctx.dump_plan()
    step = ctx.capture_step()
    assert step.scalars and set(step.scalars) <= {0.01, 1.0 / 16}   # one per use of the learning rate
    before = ctx.stats()
    r = step.replay()
    after = ctx.stats()
    assert after.replays == before.replays + 1
    assert after.barriers == before.barriers                 # nothing was cut, hashed or looked up
    assert after.nodes_recorded == before.nodes_recorded     # nothing was recorded
    assert after.regions_launched == before.regions_launched + info.n_regions
    assert r.n_regions == info.n_regions and r.n_launches == info.n_launches and r.cache_hit == 1
    assert ctx.dump_plan() == plan
    # the results are plain data again: the next traced step sees them as leaves, and hits the cache
    loss2 = programs.c2_step(ctx, X, labels, params, 0.01)
    assert ctx.barrier().cache_hit == 1
    assert loss.shape == () and loss2.shape == ()
    # wrong number of scalars
    with pytest.raises(LtError):
        step.replay(scalars=step.scalars + [1.0])
    step.replay(scalars=step.scalars)


def test_replay_refuses_a_pending_trace_and_released_inputs():
    ctx = Context(device=None)
    params, X, labels = _mlp_null(ctx)
    loss = programs.c2_step(ctx, X, labels, params, 0.01)
    ctx.barrier()
    step = ctx.capture_step()
    t = ctx.add(params[1], 1.0)          # a pending trace
    with pytest.raises(LtError) as e:
        step.replay()
    assert "pending" in str(e.value)
    ctx.barrier()
    del t
    step.replay()
    del X                                 # an input of the step goes away
    with pytest.raises(LtError) as e:
        step.replay()
    assert "released" in str(e.value)
    assert loss is not None


def test_capture_refuses_a_step_whose_input_was_released():
    ctx = Context(device=None)
    a = ctx.from_device(0, "f32", (8, 8))
    b = ctx.add(a, 2.0)
    del a                                 # (the leaf keeps its buffer until the barrier)
    ctx.barrier()
    with pytest.raises(LtError) as e:
        ctx.capture_step()
    assert "released" in str(e.value)
    assert b is not None


def test_capture_refuses_donation_to_another_tensor():
    ctx = Context(device=None)
    a = ctx.from_device(0, "f32", (64, 64), donatable=True)
    keep = ctx.mul(a, 3.0)
    other = ctx.from_device(0, "f32", (64, 64))
    ctx.assign(a, other)                  # a's old buffer is free for the taking; the result goes to `keep`
    ctx.barrier()
    if "->p" in ctx.dump_plan():
        with pytest.raises(LtError) as e:
            ctx.capture_step()
        assert "another tensor" in str(e.value) or "scratch" in str(e.value)
    assert keep is not None


def test_replay_after_the_cache_was_cleared():
    ctx = Context(device=None)
    params, X, labels = _mlp_null(ctx)
    loss = programs.c2_step(ctx, X, labels, params, 0.01)
    ctx.barrier()
    step = ctx.capture_step()
    ctx.set_fusion(False)
    with pytest.raises(LtError) as e:
        step.replay()
    assert "cleared" in str(e.value)
    assert loss is not None


def test_rebind_rules_on_the_null_device():
    ctx = Context(device=None)
    a = ctx.from_device(0, "f32", (4, 4))
    b = ctx.add(a, 1.0)
    with pytest.raises(LtError):          # the pending trace reads a
        ctx._check(ctx._lib.lt_tensor_rebind(ctx._h, a.tid, 0))
    ctx.barrier()
    ctx._check(ctx._lib.lt_tensor_rebind(ctx._h, a.tid, 0))
    with pytest.raises(LtError):          # b is a result: library memory
        ctx._check(ctx._lib.lt_tensor_rebind(ctx._h, b.tid, 0))


# ---- on the GPU ----------------------------------------------------------------------------------

@pytest.fixture()
def gctx():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    c = Context(device=0, workspace_bytes=256 << 20)
    yield c
    c.close()


@pytest.mark.gpu
@pytest.mark.parametrize("graphs", [False, True])
def test_replayed_steps_equal_traced_steps_bit_for_bit(gctx, graphs):
    """Twelve SGD steps of the MLP: traced every step, against one traced step and eleven replays
    with the batch tensors re-pointed.  Same plan, same kernels, same order: identical bits.  The
    traced run is compared with the oracle elsewhere; here the replayed one is too.  With graphs
    on, the batches are copied into fixed input tensors instead, so that addresses come back and
    steps run as HIP graphs -- with fetches (synchronisation and eager work) between them."""
    import torch
    from oracle.numeric import Eager
    steps = 12
    inp = c2_inputs(steps=steps)
    Xs = [torch.from_numpy(inp["X"][i]).cuda() for i in range(steps)]
    Ls = [torch.from_numpy(inp["labels"][i]).cuda() for i in range(steps)]

    def traced():
        ctx = gctx
        params = [ctx.tensor(inp[k].copy(), donatable=True) for k in NAMES]
        losses = []
        for i in range(steps):
            loss = programs.c2_step(ctx, ctx.tensor(Xs[i]), ctx.tensor(Ls[i]), params, 0.01)
            ctx.barrier()
            losses.append(float(ctx.fetch(loss)))
        return [ctx.fetch(p).copy() for p in params], losses

    def replayed():
        ctx = gctx
        params = [ctx.tensor(inp[k].copy(), donatable=True) for k in NAMES]
        X, L = ctx.tensor(Xs[0].clone()), ctx.tensor(Ls[0].clone())
        loss = programs.c2_step(ctx, X, L, params, 0.01)
        ctx.barrier()
        losses = [float(ctx.fetch(loss))]
        step = ctx.capture_step()
        recorded = ctx.stats().nodes_recorded
        ctx.set_graphs(graphs)
        before = ctx.stats()
        for i in range(1, steps):
            if graphs:
                X._keep.copy_(Xs[i])
                L._keep.copy_(Ls[i])
            else:
                ctx.rebind(X, Xs[i])
                ctx.rebind(L, Ls[i])
            step.replay(blocking=(i % 2 == 0))
            losses.append(float(ctx.fetch(loss)))
        after = ctx.stats()
        ctx.set_graphs(False)
        assert after.nodes_recorded == recorded
        assert after.replays - before.replays == steps - 1
        if graphs:
            # the results alternate between two places of the workspace: two graphs, each built
            # when its addresses came back
            assert 1 <= after.graphs_built - before.graphs_built <= 4
            assert after.graph_launches - before.graph_launches >= steps - 1 - 4
        else:
            assert after.graph_launches == before.graph_launches
        return [ctx.fetch(p).copy() for p in params], losses

    pt, lt_ = traced()
    pr, lr_ = replayed()
    assert lt_ == lr_
    for a, b, k in zip(pt, pr, NAMES):
        assert np.array_equal(a, b), k
    # and against the oracle (the tolerances of the free-running comparison of the traced steps)
    E = Eager()
    rp = [E.tensor(inp[k]) for k in NAMES]
    for i in range(steps):
        lo = programs.c2_step(E, E.tensor(inp["X"][i]), E.tensor(inp["labels"][i]), rp, 0.01)
        assert abs(lr_[i] - float(E.fetch(lo))) <= 1e-4 * abs(float(E.fetch(lo)))
    for g, r, k in zip(pr, rp, NAMES):
        ref = E.fetch(r)
        tol = 1e-3 if k.startswith("W") else 2e-2
        assert np.max(np.abs(g - ref)) <= tol * max(1e-30, np.max(np.abs(ref))), k


@pytest.mark.gpu
def test_replay_with_new_scalars(gctx):
    """The scalars of a step are inputs of the replay: y = a * s + t with other s and t."""
    ctx = gctx
    a_np = np.linspace(-2, 2, 4096, dtype=np.float32).reshape(64, 64)
    a = ctx.tensor(a_np)
    y = ctx.add(ctx.mul(a, 3.5), -0.25)
    ctx.barrier()
    step = ctx.capture_step()
    assert sorted(step.scalars) == [-0.25, 3.5]
    new = [7.0 if v == 3.5 else 0.5 for v in step.scalars]
    step.replay(scalars=new)
    got = ctx.fetch(y)
    want = (a_np * np.float32(7.0) + np.float32(0.5)).astype(np.float32)
    assert np.max(np.abs(got - want)) <= 1e-6 * np.max(np.abs(want))
    step.replay()
    got = ctx.fetch(y)
    want = (a_np * np.float32(3.5) + np.float32(-0.25)).astype(np.float32)
    assert np.max(np.abs(got - want)) <= 1e-6 * np.max(np.abs(want))


@pytest.mark.gpu
def test_traced_steps_as_graphs(gctx):
    """Barriers whose plan and addresses come back run as HIP graphs too: an in-place Adam-like
    update traced every step, with and without graphs, bit for bit."""
    ctx = gctx
    rng = np.random.default_rng(5)
    p0 = rng.standard_normal((256, 384)).astype(np.float32)
    g0 = rng.standard_normal((256, 384)).astype(np.float32)

    def run(graphs):
        ctx.set_graphs(graphs)
        p = ctx.tensor(p0.copy(), donatable=True)
        m = ctx.tensor(np.zeros_like(p0), donatable=True)
        g = ctx.tensor(g0)
        norms = []
        before = ctx.stats()
        for i in range(10):
            nm = ctx.add(ctx.mul(m, 0.9), ctx.mul(g, 0.1))
            npar = ctx.sub(p, ctx.mul(nm, 0.05))
            n = ctx.sum(ctx.mul(npar, npar))
            ctx.assign(m, nm)
            ctx.assign(p, npar)
            ctx.barrier(blocking=(i % 3 == 0))
            norms.append(float(ctx.fetch(n)))
        after = ctx.stats()
        ctx.set_graphs(False)
        return ctx.fetch(p).copy(), ctx.fetch(m).copy(), norms, after.graph_launches - before.graph_launches

    pa, ma, na, ga = run(False)
    pb, mb, nb, gb = run(True)
    assert ga == 0 and gb >= 4
    assert na == nb
    assert np.array_equal(pa, pb) and np.array_equal(ma, mb)


@pytest.mark.gpu
def test_transformer_layer_steps_replayed_with_the_step_number_as_scalars(gctx):
    """Four Adam steps of the small transformer layer, traced (t = 1 .. 4), against two traced steps
    and two replays in which the two scalars that depend on t (the bias corrections) are
    replaced: parameters and moments bit for bit."""
    import torch
    from workloads.inputs import c3_inputs
    ctx = gctx
    bsz, seq, d, ffn, heads = 2, 16, 64, 128, 4
    inp = c3_inputs(bsz, seq, d, ffn)
    keys = programs.C3_WEIGHTS + programs.C3_VECTORS
    bf = lambda a: torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()

    def setup():
        P = {k: ctx.tensor(bf(inp[k]), dtype="bf16", donatable=True) for k in keys}
        M = {k: ctx.tensor(np.zeros_like(inp[k]), dtype="f32", donatable=True) for k in keys}
        V = {k: ctx.tensor(np.zeros_like(inp[k]), dtype="f32", donatable=True) for k in keys}
        return ctx.tensor(bf(inp["x"]), dtype="bf16"), ctx.tensor(bf(inp["dy"]), dtype="bf16"), P, M, V, heads

    def state(g):
        return [np.asarray(ctx.fetch(g[j][k])).copy() for j in (2, 3, 4) for k in keys]

    g = setup()
    for t in range(1, 5):
        held = programs.c3_step(ctx, *g, t=t)
        ctx.barrier()
    traced = state(g)
    g = setup()
    for t in (1, 2):          # (at t = 1 the bias corrections equal 1 - beta: captured at t = 2, where they can be told apart)
        held = programs.c3_step(ctx, *g, t=t)
        ctx.barrier()
    step = ctx.capture_step()
    base = step.scalars
    c1, c2 = 1.0 - 0.9 ** 2, 1.0 - 0.999 ** 2
    assert c1 in base and c2 in base
    for t in range(3, 5):
        step.replay(scalars=[1.0 - 0.9 ** t if v == c1 else 1.0 - 0.999 ** t if v == c2 else v for v in base])
    for a, b in zip(traced, state(g)):
        assert np.array_equal(a, b)
    assert held is not None


@pytest.mark.gpu
def test_shared_tile_contraction_replayed_as_graphs(gctx):
    """h <- relu(h W + b) with 8 rows against a 2048 x 512 weight: several workgroups per tile exchange
    partial tiles and take tickets inside the launch; the tickets are reset by the kernel itself, so
    the step can run again and again as a HIP graph.  Against the same steps launched one by one."""
    ctx = gctx
    rng = np.random.default_rng(9)
    h0 = rng.standard_normal((8, 2048)).astype(np.float32)
    w = (rng.standard_normal((2048, 2048)) * 0.03).astype(np.float32)
    b = rng.standard_normal((2048,)).astype(np.float32)

    def run(graphs):
        h = ctx.tensor(h0.copy(), donatable=True)
        W, bias = ctx.tensor(w), ctx.tensor(b)
        ctx.assign(h, ctx.relu(ctx.add(ctx.matmul(h, W), bias)))
        ctx.barrier()
        step = ctx.capture_step()
        ctx.set_graphs(graphs)
        before = ctx.stats().graph_launches
        outs = []
        for i in range(8):
            step.replay(blocking=bool(i & 1))
            outs.append(ctx.fetch(h).copy())
        launched = ctx.stats().graph_launches - before
        ctx.set_graphs(False)
        return outs, launched

    eager, n0 = run(False)
    graphed, n1 = run(True)
    assert n0 == 0 and n1 >= 3
    for a, g in zip(eager, graphed):
        assert np.array_equal(a, g)
    ref = h0.astype(np.float64)
    for i in range(9):
        ref = np.maximum(ref @ w.astype(np.float64) + b, 0.0)
    assert np.max(np.abs(graphed[-1] - ref)) <= 1e-4 * np.max(np.abs(ref))   # nine chained products


def _random_steps(ctx, seed, steps, replay_from, graphs):
    """`steps` steps of the random stateful trace `seed` (the generator of the plan-validity test)
    on the same tensors: traced, or replayed from step `replay_from` on; HIP graphs on or off.
    Returns every input and every live result after every step."""
    from test_plan_validity import random_trace
    rg = np.random.Generator(np.random.PCG64(9000 + seed))
    made, calls = [], [0]

    def mk(shape, dtype="f32", donatable=False):
        k = calls[0]
        calls[0] += 1
        if k == len(made):
            made.append(ctx.tensor((rg.standard_normal(shape) * 0.5).astype(np.float32), donatable=donatable))
        return made[k]

    snaps, step, live = [], None, None
    try:
        for s in range(steps):
            if step is None:
                calls[0] = 0
                live = None
                live = random_trace(seed)(ctx, mk)
                ctx.set_graphs(graphs)
                ctx.barrier(blocking=bool(s % 3))
                if replay_from is not None and s + 1 == replay_from:
                    step = ctx.capture_step()
            else:
                step.replay(blocking=bool(s & 1))
            ctx.set_graphs(False)      # (the fetches below are eager work between the graph launches)
            snaps.append([np.asarray(ctx.fetch(t)).copy() for t in made + [t for t in live if t not in made]])
            ctx.set_graphs(graphs)
    finally:
        ctx.set_graphs(False)
    return snaps


def _compare_random_steps(ctx, seeds, steps, first, second):
    compared = 0
    for seed in seeds:
        try:
            a = _random_steps(ctx, seed, steps, *first)
            b = _random_steps(ctx, seed, steps, *second)
        except LtError as e:
            if e.status in (5, 6) and "internal" not in str(e):
                continue                      # no lowering for the pattern, or the step cannot be captured
            raise
        for s, (x, y) in enumerate(zip(a, b)):
            assert len(x) == len(y)
            for k, (u, v) in enumerate(zip(x, y)):
                assert np.array_equal(u, v, equal_nan=True), (seed, s, k)
        compared += 1
    return compared


@pytest.mark.gpu
def test_random_stateful_steps_replayed_equal_traced(gctx):
    """Random traces with in-place updates of their inputs, run as four traced steps, against two
    traced steps, a capture and two replays: every input and every live result after every step,
    bit for bit.  The capture is taken at the second step, when updated inputs already sit in
    library memory (the steady state)."""
    assert _compare_random_steps(gctx, range(60), 4, (None, False), (2, False)) >= 40


@pytest.mark.gpu
def test_random_stateful_steps_as_graphs_equal_eager_launches(gctx):
    """The same traces for ten steps, traced and replayed, with HIP graphs on against off: a
    graph is built when a plan meets the same addresses again and launched from then on, with
    fetches (eager work and synchronisation) between the launches."""
    before = gctx.stats().graph_launches
    assert _compare_random_steps(gctx, range(60, 100), 10, (None, False), (None, True)) >= 25
    assert _compare_random_steps(gctx, range(100, 140), 10, (2, False), (2, True)) >= 25
    assert gctx.stats().graph_launches - before >= 200


def test_capture_refuses_a_step_that_bound_plain_data():
    """t2 <- t3 with t3 plain data only makes t2 a second name of t3's buffer: no node records it,
    so a replay could not repeat it (t2 would keep naming the buffer of the captured step)."""
    ctx = Context(device=None)
    t2 = ctx.from_device(0, "f32", (8, 16), donatable=True)
    t3 = ctx.from_device(0, "f32", (8, 16), donatable=True)
    ctx.assign(t2, t3)
    ctx.assign(t3, ctx.add(t3, 1.0))
    ctx.barrier()
    with pytest.raises(LtError) as e:
        ctx.capture_step()
    assert e.value.status == 5 and "plain data" in str(e.value)
    # the next step without such an assignment can be captured
    ctx.assign(t3, ctx.add(t3, 1.0))
    ctx.barrier()
    ctx.capture_step().free()
    assert t2 is not None
