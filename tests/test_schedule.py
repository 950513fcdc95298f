"""Stream schedule of a plan (host logic, null device): which launches leave the caller's stream,
and that every hazard between launches on different streams is covered by an event."""
import re

import numpy as np
import pytest

from paper_2102_13267_amd import Context

LINE = re.compile(r"L(\d+) (\w+) R(\d+) stream=(\d) slot=(\d) record=([01]) waits=\[([\d,]*)\]")


def parse(text):
    out = []
    for ln in text.splitlines():
        m = LINE.fullmatch(ln)
        assert m, ln
        i, kind, region, stream, slot, record, waits = m.groups()
        out.append(dict(i=int(i), kind=kind, region=int(region), stream=int(stream), slot=int(slot), record=int(record),
                        waits=[int(w) for w in waits.split(",") if w]))
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
    reader = [l for l in sched if l["kind"] == "MM"][-1]     # z's contraction: its epilogue reads s
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


def test_set_streams_argument_checks():
    ctx = Context()
    ctx.set_streams(1)
    ctx.set_streams(4)
    for bad in (0, 5, -1):
        with pytest.raises(Exception):
            ctx.set_streams(bad)
