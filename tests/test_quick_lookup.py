"""Hashing while recording (section 7 of the paper): the record-time fingerprint finds the plan of
a trace seen before without the canonical walk; whatever changes the canonical key must change
the fingerprint too.  (Every context of this suite runs in checking mode: see conftest.py.)"""
import numpy as np
import pytest

from paper_2102_13267_amd import Context
from workloads import programs

NAMES = ("W1", "b1", "W2", "b2", "W3", "b3")
SHAPES = {"W1": (32, 24), "b1": (24,), "W2": (24, 24), "b2": (24,), "W3": (24, 10), "b3": (10,)}


def _mlp(ctx, batch=16):
    params = [ctx.from_device(0, "f32", SHAPES[k], donatable=True) for k in NAMES]
    return params, ctx.from_device(0, "f32", (batch, 32)), ctx.from_device(0, "s32", (batch,))


@pytest.mark.parametrize("mode", [1, 2])
def test_repeated_steps_are_found_by_fingerprint(mode):
    ctx = Context(device=None)
    ctx.set_quick_lookup(mode)
    params, X, L = _mlp(ctx)
    infos = []
    for _ in range(5):
        loss = programs.c2_step(ctx, X, L, params, 0.01)
        infos.append(ctx.barrier())
    st = ctx.stats()
    assert [i.cache_hit for i in infos] == [0, 1, 1, 1, 1]
    assert st.quick_hits == 4 and st.cache_hits == 4 and st.cache_misses == 1
    # the reported hash, key length and node count are the canonical ones either way
    assert len({(i.hash, i.key_bytes, i.n_nodes, i.n_regions) for i in infos}) == 1
    assert loss is not None


def test_same_answers_with_and_without_the_fingerprint():
    out = []
    for mode in (0, 1):
        ctx = Context(device=None)
        ctx.set_quick_lookup(mode)
        params, X, L = _mlp(ctx)
        rows = []
        for _ in range(3):
            loss = programs.c2_step(ctx, X, L, params, 0.01)
            i = ctx.barrier()
            rows.append((i.hash, i.key_bytes, i.cache_hit, i.n_nodes, i.n_roots, i.n_regions, ctx.dump_plan(), bytes(ctx.dump_key())))
        out.append(rows)
        assert ctx.stats().quick_hits == (2 if mode else 0)
        assert loss is not None
    assert out[0] == out[1]


def test_what_changes_the_key_changes_the_fingerprint():
    """Same recorded ops, different canonical form: a result dropped before the barrier (other
    roots), a second handle on an input's buffer (alias class), an input that is donatable and
    given up (donation pattern), a donor that another tensor still names.  Checking mode would
    fail the barrier if the fingerprint sent any of them to the first one's plan."""
    ctx = Context(device=None)
    ctx.set_quick_lookup(2)

    def step(drop=False, alias=False, donate=False, keep_donor=False):
        a = ctx.from_device(0, "f32", (64, 64), donatable=donate)
        b = ctx.from_device(0, "f32", (64, 64))
        c = ctx.from_device(0, "f32", (64, 64))
        if alias:
            ctx.assign(c, a)                  # c is a second tensor on a's buffer: same ops, two leaves on one buffer
        other = ctx.mul(c, 3.0)
        u = ctx.add(ctx.mul(a, b), 2.0)
        v = ctx.tanh(u)
        if donate:
            ctx.assign(a, v)                  # a gives its buffer up: v may be written over it
        if drop:
            del other
        if alias and not keep_donor:
            del c                             # (the leaf made from c keeps reading the buffer)
        info = ctx.barrier()
        return info.hash, info.cache_hit, ctx.dump_plan()

    seen = {}
    for kw in (dict(), dict(drop=True), dict(alias=True, keep_donor=True), dict(donate=True), dict(donate=True, alias=True, keep_donor=True),
               dict(donate=True, alias=True)):
        h, hit, plan = step(**kw)
        assert not hit, kw                    # each variant is a trace of its own
        seen[tuple(sorted(kw.items()))] = (h, plan)
        h2, hit2, plan2 = step(**kw)          # and is found again, by fingerprint
        assert hit2 and h2 == h and plan2 == plan, kw
    assert len({h for h, _ in seen.values()}) == len(seen)
    assert ctx.stats().quick_hits == len(seen)


def test_dynamic_scalars_and_buffers_do_not_enter_the_fingerprint():
    ctx = Context(device=None)
    hashes = []
    for lr in (0.01, 0.02, 0.5):
        a = ctx.from_device(0, "f32", (8, 8))
        y = ctx.mul(a, lr)
        i = ctx.barrier()
        hashes.append((i.hash, i.cache_hit))
    assert hashes[0][0] == hashes[1][0] == hashes[2][0]
    assert [h for _, h in hashes] == [0, 1, 1] and ctx.stats().quick_hits == 2
    a = ctx.from_device(0, "f32", (8, 8))
    y = ctx.mul(a, 1.0)                       # a special scalar: another graph (section 4.1)
    i = ctx.barrier()
    assert not i.cache_hit and i.hash != hashes[0][0]
    assert y is not None


def test_fusion_switch_forgets_the_fingerprints():
    ctx = Context(device=None)
    a = ctx.from_device(0, "f32", (8, 8))
    y = ctx.tanh(ctx.mul(a, 0.5))
    ctx.barrier()
    ctx.set_fusion(False)
    y = ctx.tanh(ctx.mul(a, 0.5))
    i = ctx.barrier()
    assert not i.cache_hit and i.n_regions == 2
    assert y is not None
