"""Validity checker for a lowered plan (test infrastructure; shares nothing with either lowering).

Input: the canonical byte string of a cut trace (what `lt_dump_key` returns: the program), the number
of nodes in it, and the region list (`lt_dump_plan`: the partition).  The checker does not decide
WHICH partition is right -- any partition that passes computes the trace's values, because every
property below is what makes running the regions one after the other equal to running the recorded
ops one by one (section 3 of the paper), with the special scalars 0 and 1 folded away (section 4.1)
and in-place updates only where nothing can observe the old value (section 4.3):

  1. every node that a result depends on is computed exactly once: it is a member of exactly one
     region, or a leaf, or a pure view (expand / reshape / a permutation feeding contractions) that
     its consumers resolve into addressing;
  2. what a region's members read from outside is declared as its inputs, each of which is, seen
     through views, a caller's buffer or a declared output of a region that runs EARLIER in the list
     (so the region graph is acyclic and the list is a schedule of it);
  3. every result of the trace is a leaf or a declared output of its region; outputs are members;
  4. a region's members share the iteration space its kernel walks: one shape for an elementwise
     region; for a reduction the reduced tensor's shape before the anchor and the anchor's shape
     (or, for a global reduction, one small finaliser shape) after it; the product's shape after a
     contraction; fixed row operators stand alone;
  5. a permutation never sits in one region with the producer of its operand (it reads other
     positions than it writes) -- except as the output layout of a bare contraction whose product
     nothing else reads;
  6. the caps of a region hold (inputs, outputs, inputs + members);
  7. an in-place entry `v->pK` writes a region output of parameter K's dtype and shape; K is claimed
     once; no later region reads K, no other result is K itself, and inside the writing region K is
     read only position by position (a direct operand of an elementwise member, not through a view,
     not by the anchor, not by a permutation).
"""
from __future__ import annotations

import struct

DEVICE_DATA, SCALAR_PARAM, CONSTANT = 1, 2, 3
ADD, SUB, MUL, DIV = 32, 33, 34, 35
EXPAND, RESHAPE, PERMUTE, NARROW, SLICE_UPDATE = 48, 49, 50, 51, 52
SUM, AMAX, MEAN = 64, 65, 66
LAYER_NORM = 82
MATMUL = 96
A_VALUE, A_AXIS, A_DIM0 = 1, 3, 16
MAX_INPUTS, MAX_OUTPUTS, MAX_SLOTS, MAX_FINALISER = 8, 8, 32, 65536


class PlanError(AssertionError):
    pass


def need(cond, msg):
    if not cond:
        raise PlanError(msg)


class N:
    __slots__ = ("op", "dtype", "shape", "attrs", "ins", "ordinal", "alias")


def parse_key(key: bytes, n_nodes: int):
    """-> (nodes, roots) with roots = [(node, slot, donor ordinal or None)]."""
    pos = 0

    def take(fmt):
        nonlocal pos
        v = struct.unpack_from("<" + fmt, key, pos)
        pos += struct.calcsize("<" + fmt)
        return v if len(v) > 1 else v[0]
    nodes = []
    for _ in range(n_nodes):
        n = N()
        n.op, n.dtype, rank = take("HBB")
        n.shape = tuple(take("q") for _ in range(rank))
        n.attrs = {}
        for _ in range(take("B")):
            k, isf = take("HB")
            n.attrs[k] = take("d") if isf else take("q")
        n.ins = [tuple(take("IB")) for _ in range(take("B"))]
        n.ordinal = n.alias = None
        if n.op == DEVICE_DATA:
            n.ordinal, n.alias = take("II")       # alias: ordinal of the first leaf on the same buffer
        elif n.op == SCALAR_PARAM:
            n.ordinal = take("I")
        nodes.append(n)
    roots = []
    for _ in range(take("I")):
        node, slot, donor = take("IBI")
        roots.append((node, slot, None if donor == 0xFFFFFFFF else donor))
    need(pos == len(key), "key has trailing bytes")
    return nodes, roots


def parse_plan(text: str):
    regions = []
    for line in text.splitlines():
        if not line.strip():
            continue
        head, rest = line.split(" members=[")
        _, kind, anchor = head.split()
        members, rest = rest.split("] inputs=[")
        inputs, rest = rest.split("] outputs=[")
        outputs, rest = rest.split("] inplace=[")
        inplace = rest.rstrip("]")
        val = lambda s: tuple(int(x) for x in s.split("."))
        regions.append({
            "kind": kind,
            "anchor": None if anchor == "anchor=-" else int(anchor.split("=")[1]),
            "members": [int(m) for m in members.split(",") if m],
            "inputs": [val(s) for s in inputs.split(",") if s],
            "outputs": [val(s) for s in outputs.split(",") if s],
            "inplace": [(val(s.split("->p")[0]), int(s.split("->p")[1])) for s in inplace.split(",") if s],
        })
    return regions


def check_plan(key: bytes, n_nodes: int, plan_text: str):
    nodes, roots = parse_key(key, n_nodes)
    regions = parse_plan(plan_text)

    def out_shape(v):
        n = nodes[v[0]]
        return n.shape[:-1] if n.op == LAYER_NORM and v[1] > 0 else n.shape

    def out_dtype(v):
        n = nodes[v[0]]
        return 0 if n.op == LAYER_NORM and v[1] > 0 else n.dtype

    # ---- the special scalars 0 and 1 (section 4.1): x*1, 1*x, x+0, 0+x, x-0, x/1 are x -------------
    def const_value(v):
        v = resolve(v)
        n = nodes[v[0]]
        if n.op == CONSTANT:
            return n.attrs[A_VALUE]
        if n.op in (EXPAND, RESHAPE):
            return const_value(n.ins[0])
        return None

    def resolve(v):
        while v[1] == 0:
            n = nodes[v[0]]
            ops = n.ins
            keep = None
            if n.op == ADD and len(ops) == 3 and const_value(ops[2]) == 1:
                ops = ops[:2]
            if n.op == MUL and len(ops) == 2:
                keep = 0 if const_value(ops[1]) == 1 else 1 if const_value(ops[0]) == 1 else None
                if keep == 0 and not same(ops[0], n):
                    keep = 1 if const_value(ops[0]) == 1 else None
            elif n.op == ADD and len(ops) == 2:
                keep = 0 if const_value(ops[1]) == 0 else 1 if const_value(ops[0]) == 0 else None
                if keep == 0 and not same(ops[0], n):
                    keep = 1 if const_value(ops[0]) == 0 else None
            elif n.op == SUB and const_value(ops[1]) == 0:
                keep = 0
            elif n.op == DIV and const_value(ops[1]) == 1:
                keep = 0
            if keep is None or not same(ops[keep], n):
                return v
            v = resolve(ops[keep])
        return v

    def same(v, n):
        w = resolve(v)
        return out_shape(w) == n.shape and out_dtype(w) == n.dtype

    def operands(i):
        n = nodes[i]
        ops = n.ins
        if n.op == ADD and len(ops) == 3 and const_value(ops[2]) == 1:
            ops = ops[:2]
        return [resolve(v) for v in ops]

    def is_immediate(v):
        n = nodes[v[0]]
        if n.op in (CONSTANT, SCALAR_PARAM):
            return True
        return n.op in (EXPAND, RESHAPE) and is_immediate(operands(v[0])[0])

    # ---- region membership -------------------------------------------------------------------------
    region_of = {}
    for k, r in enumerate(regions):
        need(r["members"] == sorted(set(r["members"])), f"R{k}: members not sorted / unique")
        for m in r["members"]:
            need(m not in region_of, f"node {m} is a member of two regions")
            need(nodes[m].op not in (DEVICE_DATA, SCALAR_PARAM, CONSTANT), f"R{k}: leaf {m} as member")
            region_of[m] = k
    produced = {}
    for k, r in enumerate(regions):
        for v in r["outputs"]:
            need(v[0] in r["members"], f"R{k}: output {v} is not computed by the region")
            produced[v] = k

    def is_view_node(i):
        return i not in region_of and nodes[i].op in (EXPAND, RESHAPE, PERMUTE, NARROW)

    def base(v):
        while is_view_node(v[0]):
            v = operands(v[0])[0]
        return v

    root_vals = [resolve((n, s)) for (n, s, _) in roots]
    # 1. liveness: everything a result depends on is a leaf, a view or a member of one region
    live, stack = set(), [v[0] for v in root_vals]
    while stack:
        i = stack.pop()
        if i in live:
            continue
        live.add(i)
        stack.extend(v[0] for v in operands(i))
    for i in sorted(live):
        n = nodes[i]
        if n.op in (DEVICE_DATA, SCALAR_PARAM, CONSTANT) or i in region_of:
            continue
        need(n.op in (EXPAND, RESHAPE, PERMUTE, NARROW), f"live node {i} (op {n.op}) is computed by no region")
        if n.op == PERMUTE:
            users = [j for j in live if any(v[0] == i for v in operands(j))]
            need(users and all(nodes[j].op == MATMUL for j in users), f"permutation {i} outside every region feeds a non-contraction")
    for i in region_of:
        need(i in live, f"dead node {i} is a member of a region")

    # 3. results
    for v in root_vals:
        if nodes[v[0]].op in (DEVICE_DATA, SCALAR_PARAM, CONSTANT):
            continue
        need(v in produced, f"result {v} is not a declared output of any region")

    for k, r in enumerate(regions):
        members = set(r["members"])
        # 2. what the members read
        reads = []
        for m in r["members"]:
            for v in operands(m):
                if v[0] in members or is_immediate(v):
                    continue
                if v not in reads:
                    reads.append(v)
        need(sorted(reads) == sorted(r["inputs"]), f"R{k}: declared inputs {r['inputs']} differ from what the members read {reads}")
        for v in r["inputs"]:
            b = base(v)
            if nodes[b[0]].op == DEVICE_DATA:
                continue
            need(b in produced, f"R{k}: input {v} (base {b}) is produced by no region")
            need(produced[b] < k, f"R{k}: input {v} is produced by the later region R{produced[b]}")
        # values needed outside must be declared outputs
        for m in r["members"]:
            n_out = 3 if nodes[m].op == LAYER_NORM else 1
            for s in range(n_out):
                v = (m, s)
                ext = v in root_vals or any(v in operands(j) for j in live if j not in members)
                need(ext == (v in r["outputs"]), f"R{k}: value {v} escapes={ext} but declared={v in r['outputs']}")
        # 5. permutations
        for m in r["members"]:
            layout = r["kind"] == "MM" and operands(m)[0] == (r["anchor"], 0) and len(members) == 2 and (r["anchor"], 0) not in r["outputs"]
            if nodes[m].op == PERMUTE and not layout:   # (a contraction may write its product in a permuted layout)
                need(operands(m)[0][0] not in members, f"R{k}: permutation {m} shares the region with its operand's producer")
        # 6. caps
        need(len(r["inputs"]) <= MAX_INPUTS and len(r["outputs"]) <= MAX_OUTPUTS, f"R{k}: too many inputs or outputs")
        need(len(r["inputs"]) + len(r["members"]) <= MAX_SLOTS, f"R{k}: more than {MAX_SLOTS} slots")
        # 4. iteration spaces
        a = r["anchor"]
        if r["kind"] == "EW":
            need(a is None, f"R{k}: elementwise region with an anchor")
            shapes = {nodes[m].shape for m in r["members"]}
            need(len(shapes) == 1, f"R{k}: elementwise members of different shapes {shapes}")
            for m in r["members"]:
                need(nodes[m].op < SUM and nodes[m].op != SLICE_UPDATE, f"R{k}: member {m} is not elementwise")
        else:
            need(a in members, f"R{k}: anchor {a} is not a member")
            an = nodes[a]
            before = set()
            stack = [a]
            while stack:                       # members the anchor depends on
                for v in operands(stack.pop()):
                    if v[0] in members and v[0] not in before:
                        before.add(v[0])
                        stack.append(v[0])
            after = members - before - {a}
            for m in members - {a}:
                need(nodes[m].op < SUM and nodes[m].op != SLICE_UPDATE, f"R{k}: member {m} next to the anchor is not elementwise")
            if r["kind"] == "SLICE":
                need(an.op == SLICE_UPDATE and len(members) == 1, f"R{k}: a window update stands alone")
            elif r["kind"] == "MM":
                need(an.op == MATMUL and not before, f"R{k}: contraction region with a prologue")
                # a permutation OF THE PRODUCT is its output layout and closes the region; a
                # permutation of another region's value is an ordinary strided read
                perms = [m for m in after if nodes[m].op == PERMUTE and operands(m)[0][0] == a]
                if perms:
                    need(len(after) == 1, f"R{k}: a layout permutation must be the contraction's only follower")
                else:
                    need(all(nodes[m].shape == an.shape for m in after), f"R{k}: post members differ from the product's shape")
            elif an.op in (SUM, AMAX, MEAN):
                in_shape = out_shape(operands(a)[0])
                axis = an.attrs.get(A_AXIS)
                want = "ALL" if (axis is None or len(in_shape) <= 1) else "ROW" if axis == len(in_shape) - 1 else "COL" if axis == 0 else None
                need(want == r["kind"], f"R{k}: reduction over axis {axis} of {in_shape} labelled {r['kind']}")
                need(all(nodes[m].shape == in_shape for m in before), f"R{k}: prologue members differ from the reduced tensor's shape")
                fin = {nodes[m].shape for m in after if nodes[m].shape != an.shape}
                if fin:
                    need(r["kind"] == "ALL" and len(fin) == 1, f"R{k}: post members of shapes {fin} after an anchor of shape {an.shape}")
                    (fs,) = fin
                    cnt = 1
                    for d in fs:
                        cnt *= d
                    need(len(fs) >= 1 and cnt <= MAX_FINALISER, f"R{k}: finaliser of {cnt} elements")
            else:
                need(r["kind"] == "ROW" and len(members) == 1, f"R{k}: a fixed row operator stands alone")
        # 7. in-place updates
        for (v, p) in r["inplace"]:
            need(v in r["outputs"], f"R{k}: in-place value {v} is not an output")
            leaf = [i for i, n in enumerate(nodes) if n.op == DEVICE_DATA and n.ordinal == p]
            need(len(leaf) == 1, f"R{k}: parameter {p} does not exist")
            leaf = leaf[0]
            cls = nodes[leaf].alias

            def is_donor(w):
                return nodes[w[0]].op == DEVICE_DATA and nodes[w[0]].alias == cls
            need(nodes[leaf].shape == out_shape(v) and nodes[leaf].dtype == out_dtype(v), f"R{k}: {v}->p{p} changes shape or dtype")
            need(any(resolve((n, s)) == v and d == p for (n, s, d) in roots), f"R{k}: {v}->p{p} was not offered by the cut")
            for j, w in enumerate(root_vals):
                need(not is_donor(w), f"R{k}: parameter {p} is overwritten while result {j} is that parameter itself")
            for k2 in range(k + 1, len(regions)):
                for w in regions[k2]["inputs"]:
                    need(not is_donor(base(w)), f"R{k}: parameter {p} is overwritten before R{k2} reads it")
            for m in r["members"]:
                for w in operands(m):
                    if w[0] in members or is_immediate(w) or not is_donor(base(w)):
                        continue
                    if m == a and nodes[m].op == SLICE_UPDATE and w == (leaf, 0) and w == operands(m)[0] and not is_donor(base(operands(m)[1])):
                        continue        # a window update rewrites part of its own base: the rest stays as it is
                    need(w == (leaf, 0) and m != a and nodes[m].op not in (PERMUTE, EXPAND, RESHAPE, NARROW) and nodes[m].shape == nodes[leaf].shape,
                         f"R{k}: parameter {p} is overwritten by a region that reads it out of position (member {m})")
    claimed = [p for r in regions for (_, p) in r["inplace"]]
    need(len(claimed) == len(set(claimed)), "a parameter is written in place twice")
    return {"regions": len(regions), "live": len(live)}
