"""Pins for the structural oracle (no GPU): the IR listings printed in the
paper, published hash vectors, and invariants of the canonical form."""
import itertools

import numpy as np
import pytest

import figures
from conftest import ROOT, read_golden
from oracle import structural as S
from oracle.structural import Tracer
from workloads import programs


@pytest.mark.parametrize("name", ["fig1", "fig2", "fig3"])
def test_paper_figures_reproduced(name):
    """Figures 1(a), 2(b) and 3 of the paper, node for node."""
    T = Tracer("CPU:0")
    keep = getattr(figures, name)(T, lambda shape: T.tensor(shape))
    assert T.dump_ir() == read_golden(name + "_ir.txt")
    del keep


def test_fnv1a64_published_vectors():
    for line in read_golden("fnv1a64_vectors.txt").splitlines():
        text, hexval = line.rsplit(" ", 1)
        assert S.fnv1a64(text.strip('"').encode()) == int(hexval, 16)


def _hash_of(build):
    T = Tracer()
    keep = build(T)
    r = T.barrier()
    del keep
    return r["hash"], r["bytes"]


def _simple(T, scalar=0.5, shape=(4, 8), dtype="f32", swap=False, op="sub"):
    a, b = T.tensor(shape, dtype), T.tensor(shape, dtype)
    lhs, rhs = T.mul(a, scalar), b
    if swap:
        lhs, rhs = rhs, lhs
    return [getattr(T, op)(lhs, rhs)], (a, b)


def test_hash_invariants_special_scalars():
    """Section 4.1: only 0 and 1 are part of the graph; other scalars are
    parameters.  0.5 -> 0.7 keeps the hash, 0.5 -> 1.0 changes it (the
    spurious recompilation the paper admits), -0.0 is not special."""
    h05, _ = _hash_of(lambda T: _simple(T, 0.5))
    h07, _ = _hash_of(lambda T: _simple(T, 0.7))
    h10, _ = _hash_of(lambda T: _simple(T, 1.0))
    h00, _ = _hash_of(lambda T: _simple(T, 0.0))
    hm0, _ = _hash_of(lambda T: _simple(T, -0.0))
    assert h05 == h07 == hm0
    assert len({h05, h10, h00}) == 3


def test_hash_sensitive_to_structure():
    base, _ = _hash_of(lambda T: _simple(T))
    assert base == _hash_of(lambda T: _simple(T))[0]                 # same trace twice
    assert base != _hash_of(lambda T: _simple(T, shape=(4, 9)))[0]    # a dim
    assert base != _hash_of(lambda T: _simple(T, dtype="bf16"))[0]    # a dtype
    assert base != _hash_of(lambda T: _simple(T, op="div"))[0]        # an opcode
    assert base != _hash_of(lambda T: _simple(T, swap=True))[0]       # operand order


def test_hash_ignores_buffers_but_not_sharing():
    def two(T, share):
        a = T.tensor((3, 3))
        b = a if share else T.tensor((3, 3))
        return [T.add(a, b)], (a, b)
    assert _hash_of(lambda T: two(T, True))[0] != _hash_of(lambda T: two(T, False))[0]
    assert _hash_of(lambda T: two(T, False))[0] == _hash_of(lambda T: two(T, False))[0]


def test_canonical_string_is_injective_on_small_dags():
    """Brute force: every DAG of <= 3 binary ops over 2 leaves; two traces get
    the same byte string iff they are structurally the same program."""
    ops = ["add", "sub"]
    seen = {}
    for n_ops in (1, 2, 3):
        choices = []
        for k in range(n_ops):
            avail = 2 + k
            choices.append(list(itertools.product(ops, range(avail), range(avail))))
        for combo in itertools.product(*choices):
            T = Tracer()
            vals = [T.tensor((2,)), T.tensor((2,))]
            for (op, i, j) in combo:
                vals.append(getattr(T, op)(vals[i], vals[j]))
            root = vals[-1]
            leaves = vals[:2]
            del vals
            # structural identity of the reachable expression, leaves by first use
            def expr(T, t):
                names = {}
                def go(n):
                    node = T.nodes[n]
                    if node.op == S.DEVICE_DATA:
                        return ("leaf", id(node.buffer))
                    return (node.op,) + tuple(go(c) for c, _ in node.ins)
                tree = go(t.node)
                flat = repr(tree)
                for k, ident in enumerate(dict.fromkeys(
                        int(tok) for tok in __import__("re").findall(r"'leaf', (\d+)", flat))):
                    flat = flat.replace(str(ident), f"L{k}")
                return flat
            sig = expr(T, root)
            # node sharing matters too: count distinct reachable nodes
            order, _ = T.canonical_order([(root.node, 0)])
            sig = (sig, len(order))
            blob = T.barrier()["bytes"]
            if blob in seen:
                assert seen[blob] == sig
            seen.setdefault(blob, sig)
            del root, leaves
    sigs = list(seen.values())
    assert len(set(sigs)) == len(sigs)        # equal signature => equal bytes


def test_c1_cache_sequence_and_two_regions():
    T = Tracer()
    x, y, b = T.tensor((1024, 1024)), T.tensor((1024, 1024)), T.tensor((1024,))
    hits, plans = [], []
    for _ in range(10):
        out = programs.c1_trace(T, x, y, b)
        r = T.barrier()
        hits.append(int(r["cache_hit"]))
        plans.append(r["plan"])
        del out
    assert hits == [0] + [1] * 9
    assert len(set(plans)) == 1
    lines = plans[0].splitlines()
    assert len(lines) == 2 and lines[0].startswith("R0 ROW") and lines[1].startswith("R1 ALL")


def test_c4_is_one_reduction_and_one_elementwise_pass_in_place():
    from workloads.inputs import C4_HYPER
    T = Tracer()
    n = 1 << 20
    p, g, m, v = (T.tensor((n,), donatable=True) for _ in range(4))
    for step in range(3):
        programs.c4_step(T, p, g, m, v, **C4_HYPER)
        r = T.barrier()
        lines = r["plan"].splitlines()
        assert [l.split()[1] for l in lines] == ["ALL", "EW"]
        assert lines[1].count("->p") == 3                       # p, m, v written in place
        assert r["cache_hit"] == (step > 0)


def test_c2_cache_hit_from_second_step_and_updates_in_place():
    T = Tracer()
    dims = (784, 512, 512, 10)
    params = []
    for i in range(3):
        params += [T.tensor((dims[i], dims[i + 1]), donatable=True), T.tensor((dims[i + 1],), donatable=True)]
    hits = []
    for step in range(4):
        X, lab = T.tensor((128, 784)), T.tensor((128,), "s32")
        loss = programs.c2_step(T, X, lab, params, 0.01)
        r = T.barrier()
        hits.append(int(r["cache_hit"]))
        assert r["plan"].count("->p") == 6
        del loss, X, lab
    assert hits == [0, 1, 1, 1]


def test_aliasing_counter_examples_of_section_4_3():
    """(i) a += 1 then two reads: the second read must not re-apply the update
    (after the barrier the handle is plain data, nothing is pending).
    (ii) b = a + 2; a += 1: b is in the same graph, and the region computing
    b must run before a's buffer is overwritten."""
    T = Tracer()
    a = T.tensor((16,), donatable=True)
    T.assign(a, T.add(a, 1.0))
    r1 = T.barrier()
    assert r1["plan"].count("->p0") == 1
    r2 = T.barrier()
    assert r2["n_nodes"] == 0 and r2["plan"] == ""
    b = T.add(a, 2.0)
    T.assign(a, T.add(a, 1.0))
    r3 = T.barrier()
    lines = r3["plan"].splitlines()
    # either one fused region (reads a once, writes both) or b's region first
    writer = [k for k, l in enumerate(lines) if "->p" in l]
    assert len(writer) == 1
    for k, l in enumerate(lines):
        if k > writer[0]:
            assert "inputs=[]" in l or "0.0" not in l.split("inputs=")[1].split("]")[0]
    del b


def test_donation_refused_while_another_handle_sees_the_buffer():
    T = Tracer()
    a = T.tensor((16,), donatable=True)
    keep = T.scalar(0.0)
    T.assign(keep, a)                       # a second handle bound to a's buffer
    T.assign(a, T.add(a, 1.0))
    assert "->p" not in T.barrier()["plan"]
    del keep


def test_a_live_alias_of_the_destination_forbids_its_update_in_place():
    """b = a * 1 folds to a's buffer itself (section 4.1); a += 1 in the same step must then leave
    that buffer alone, or b would show the new value (section 4.3, second condition)."""
    T = Tracer()
    a = T.tensor((16,), donatable=True)
    b = T.mul(a, 1.0)
    T.assign(a, T.add(a, 1.0))
    assert "->p" not in T.barrier()["plan"]
    del b
    # without the alias the same update is in place
    T.assign(a, T.add(a, 1.0))
    assert "->p0" in T.barrier()["plan"]


def test_two_leaves_on_one_buffer_are_part_of_the_key():
    """A second handle on a buffer (made by assign) gives a second device_data leaf; whether two
    leaves alias decides what may be written in place, so it must change the hash."""
    def run(aliased):
        T = Tracer()
        x = T.tensor((8, 8), donatable=True)
        w = T.scalar(0.0)
        if aliased:
            T.assign(w, x)
        else:
            w = T.tensor((8, 8), donatable=True)
        r = T.add(T.permute(w, (1, 0)), x)
        T.assign(x, r)
        del w, r
        return T.barrier()
    plain, aliased = run(False), run(True)
    assert plain["hash"] != aliased["hash"]
    assert "->p" in plain["plan"] and "->p" not in aliased["plan"]


def test_fusion_never_builds_a_cyclic_region_graph():
    """s feeds a global max, and the result divides s again: the divide must
    not be pulled back into the row-reduction region (that would be a cycle)."""
    T = Tracer()
    x = T.tensor((64, 32))
    s = T.sum(x, axis=1)
    out = T.div(s, T.amax(T.abs(s)))
    del s
    lines = T.barrier()["plan"].splitlines()
    assert [l.split()[1] for l in lines] == ["ROW", "ALL"]
    del out


def test_region_caps_split_long_chains():
    T = Tracer()
    x = T.tensor((128,))
    h = x
    for k in range(80):
        h = T.add(T.mul(h, 0.5), x)
    lines = T.barrier()["plan"].splitlines()
    assert len(lines) >= 5
    for l in lines:
        members = l.split("members=[")[1].split("]")[0].split(",")
        inputs = [s for s in l.split("inputs=[")[1].split("]")[0].split(",") if s]
        assert len(members) + len(inputs) <= S.MAX_SLOTS
    del h
