"""Stream schedule of a plan (host logic, null device): which launches leave the caller's stream,
and that every hazard between launches on different streams is covered by an event."""
import re

import numpy as np
import pytest

from paper_2102_13267_amd import Context

LINE = re.compile(r"L(\d+) (\w+) R(\d+) stream=(\d) slot=(\d) record=([01]) waits=\[([\d,]*)\] reads=\[([\w,]*)\] writes=\[([\w,]*)\]")


def parse(text):
    out = []
    for ln in text.splitlines():
        m = LINE.fullmatch(ln)
        assert m, ln
        i, kind, region, stream, slot, record, waits, reads, writes = m.groups()
        out.append(dict(i=int(i), kind=kind, region=int(region), stream=int(stream), slot=int(slot), record=int(record),
                        waits=[int(w) for w in waits.split(",") if w],
                        reads=set(r for r in reads.split(",") if r), writes=set(w for w in writes.split(",") if w)))
    return out


def invariants(sched):
    for k, l in enumerate(sched):
        assert l["i"] == k and 0 <= l["stream"] <= 3 and 0 <= l["slot"] <= 3
        for w in l["waits"]:
            assert w < k, "a launch waits only for earlier launches"
            assert sched[w]["stream"] != l["stream"], "same-stream order needs no event"
            assert sched[w]["record"] == 1, "a launch that is waited for records an event"
    for l in sched:
        if l["record"]:
            assert any(l["i"] in m["waits"] for m in sched), "no event without a waiter"


def ordered_before(sched):
    """before[j][s] = the last launch of stream s known to have finished when launch j starts
    (-1: none): its own stream's predecessor, what that one knew, and what each event it waits for
    brings along."""
    before = []
    last_on = {}
    for l in sched:
        know = dict(before[last_on[l["stream"]]]) if l["stream"] in last_on else {}
        if l["stream"] in last_on:
            know[l["stream"]] = last_on[l["stream"]]
        for w in l["waits"]:
            for s, k in list(before[w].items()) + [(sched[w]["stream"], w)]:
                know[s] = max(know.get(s, -1), k)
        before.append(know)
        last_on[l["stream"]] = l["i"]
    return before


def hazards_are_ordered(sched):
    """Every pair of launches that touch the same storage, at least one of them writing it, and
    every pair of reductions that share a scratch quarter, run in plan order."""
    before = ordered_before(sched)
    for j, lj in enumerate(sched):
        for i in range(j):
            li = sched[i]
            clash = (li["writes"] & (lj["reads"] | lj["writes"])) or (li["reads"] & lj["writes"])
            scratch = li["kind"] in ("COL", "ALL") and lj["kind"] in ("COL", "ALL") and li["slot"] == lj["slot"]
            if clash or scratch:
                assert before[j].get(li["stream"], -1) >= i, (i, j, clash, li, lj)


def f32(ctx, shape):
    return ctx.tensor(np.zeros(shape, np.float32), dtype="f32")


def test_small_plans_stay_on_the_callers_stream():
    ctx = Context()
    x, w = f32(ctx, (64, 32)), f32(ctx, (32, 32))
    outs = [ctx.sum(x, axis=0), ctx.matmul(x, w), ctx.sum(ctx.square(x), axis=0), ctx.tanh(x)]
    ctx.barrier()
    sched = parse(ctx.dump_schedule())
    invariants(sched)
    assert len(sched) == 4 and all(l["stream"] == 0 and not l["waits"] for l in sched)


def test_wide_column_reductions_move_and_their_consumers_wait():
    """y0 = x w; s = column sums of x^2 (16 MiB read: a side stream); z = x w2 + s: the contraction
    whose epilogue reads s has to be ordered behind the reduction."""
    ctx = Context()
    x, w, w2 = f32(ctx, (4096, 1024)), f32(ctx, (1024, 1024)), f32(ctx, (1024, 1024))
    y0 = ctx.matmul(x, w)
    s = ctx.sum(ctx.square(x), axis=0)
    z = ctx.add(ctx.matmul(x, w2), s)
    ctx.barrier()
    plan = ctx.dump_plan().splitlines()
    sched = parse(ctx.dump_schedule())
    invariants(sched)
    kinds = [l["kind"] for l in sched]
    assert kinds.count("COL") == 1
    col = next(l for l in sched if l["kind"] == "COL")
    assert col["stream"] > 0
    # z's contraction reads s in its post program (the second launch, when k is split over workgroups)
    reader = [l for l in sched if l["kind"] in ("MM", "SPLITPOST") and set(l["reads"]) & set(col["writes"])][-1]
    assert reader["i"] > col["i"] and "inputs=" in plan[reader["region"]]
    # ordered behind the reduction: the same stream, an event of the reduction, or an event of a
    # later launch of the reduction's stream
    assert reader["stream"] == col["stream"] or col["i"] in reader["waits"] or any(
        sched[w]["stream"] == col["stream"] and w >= col["i"] for w in reader["waits"])
    del y0, z


def test_reductions_in_flight_use_different_scratch_quarters():
    ctx = Context()
    x = f32(ctx, (8192, 1024))
    big = ctx.matmul(x, f32(ctx, (1024, 1024)))
    sums = [ctx.sum(ctx.mul(x, float(k + 2)), axis=0) for k in range(5)]
    ctx.barrier()
    sched = parse(ctx.dump_schedule())
    invariants(sched)
    cols = [l for l in sched if l["kind"] == "COL"]
    assert len(cols) == 5
    assert [l["slot"] for l in cols] == [0, 1, 2, 3, 0]
    # the fifth reuses the first one's quarter: same stream and later, or an event
    a, e = cols[0], cols[4]
    assert a["stream"] == e["stream"] or a["i"] in e["waits"] or any(
        m["stream"] == a["stream"] and m["i"] >= a["i"] for m in (sched[w] for w in e["waits"]))
    del big, sums


def test_in_place_update_waits_for_every_reader_on_other_streams():
    """p is read by a column reduction on a side stream and then overwritten in place: the writer
    waits for the reader (write-after-read across streams)."""
    ctx = Context()
    p = ctx.tensor(np.zeros((8192, 1024), np.float32), dtype="f32", donatable=True)
    warm = ctx.matmul(p, f32(ctx, (1024, 256)))
    colsum = ctx.sum(ctx.abs(p), axis=0)
    ctx.assign(p, ctx.mul(p, 0.5))
    ctx.barrier()
    sched = parse(ctx.dump_schedule())
    invariants(sched)
    col = next(l for l in sched if l["kind"] == "COL")
    writer = next(l for l in sched if l["kind"] == "EW")
    assert writer["i"] > col["i"]
    assert col["stream"] == writer["stream"] or col["i"] in writer["waits"]
    del warm, colsum


@pytest.mark.parametrize("seed", range(12))
def test_random_large_traces_keep_every_hazard_in_order(seed):
    """Random traces over tensors large enough for their launches to leave the caller's stream:
    contractions, elementwise chains, row / column / global reductions, in-place updates of
    donated buffers.  Whatever the schedule, conflicting launches must stay ordered."""
    g = np.random.Generator(np.random.PCG64(4000 + seed))
    ctx = Context()
    rows, cols = 4096, 1024
    mats = [ctx.tensor(np.zeros((rows, cols), np.float32), dtype="f32", donatable=(k < 2)) for k in range(4)]
    sq = [f32(ctx, (cols, cols)) for _ in range(2)]
    vec = ctx.tensor(np.zeros((cols,), np.float32), dtype="f32", donatable=True)
    keep = []
    for _ in range(int(g.integers(8, 16))):
        kind = int(g.integers(0, 7))
        a, b = mats[int(g.integers(0, 4))], mats[int(g.integers(0, 4))]
        if kind == 0:
            t = ctx.matmul(a, sq[int(g.integers(0, 2))])
        elif kind == 1:
            t = ctx.matmul(a, b, trans_a=True)
        elif kind == 2:
            t = ctx.tanh(ctx.add(ctx.mul(a, 0.5), b))
        elif kind == 3:
            t = ctx.sum(ctx.mul(a, b), axis=0)
        elif kind == 4:
            t = ctx.sum(ctx.square(a), axis=1)
        elif kind == 5:
            t = ctx.sqrt(ctx.sum(ctx.square(a)))
        else:
            t = ctx.softmax(a)
        if t.shape == (rows, cols) and g.random() < 0.5:
            k = int(g.integers(0, 4))
            if k < 2:
                ctx.assign(mats[k], t)                       # in place: donated
            else:
                mats[k] = t                                  # the old tensor dies: its storage may be reused
        elif t.shape == (cols,) and g.random() < 0.5:
            ctx.assign(vec, ctx.add(vec, t))
        else:
            keep.append(t)
    ctx.barrier()
    sched = parse(ctx.dump_schedule())
    invariants(sched)
    hazards_are_ordered(sched)
    assert any(l["stream"] > 0 for l in sched) or len(sched) < 3
    del keep


def test_hazard_check_sees_a_missing_event():
    """The checker itself: with the events of a schedule that needs them taken away, it objects."""
    ctx = Context()
    x, w2 = f32(ctx, (4096, 1024)), f32(ctx, (1024, 1024))
    y0 = ctx.matmul(x, f32(ctx, (1024, 1024)))               # one stream
    s = ctx.sum(ctx.square(x), axis=0)                       # another
    z = ctx.add(ctx.matmul(y0, w2), s)                       # reads both: an event, whichever stream it takes
    ctx.barrier()
    sched = parse(ctx.dump_schedule())
    hazards_are_ordered(sched)
    assert any(l["waits"] for l in sched)
    for l in sched:
        l["waits"] = []
    with pytest.raises(AssertionError):
        hazards_are_ordered(sched)
    del y0, z


def test_set_streams_argument_checks():
    ctx = Context()
    ctx.set_streams(1)
    ctx.set_streams(4)
    for bad in (0, 5, -1):
        with pytest.raises(Exception):
            ctx.set_streams(bad)
