"""Reference planner: queries -> operator-level frontiers and gradient indices.

TEST INFRASTRUCTURE ONLY -- the product path never imports this file.

The paper groups, at every scheduling step, the ready operators of one type
from all queries into one batch [Sec. 4.1 "Dynamic Scheduling", "Batched
Execution"; Alg. 1], splits intersections/unions into classes of equal input
count [Sec. 4.3, Eq. C_k], and pre-computes the gather/scatter offsets of the
entity embeddings [Sec. 4.2 "Efficient Tensor Indexing"].  It does not fix an
order or a numbering, so a canonical one is fixed here (the HIP library's
planner must reproduce it bit for bit):

 1. Unions are removed by disjunctive normal form; branches keep input order.
 2. Nodes get global ids in (query, branch, depth-first post-order) order.
 3. level(anchor) = 0, level(op) = 1 + max level of its inputs (level-synchronous
    schedule), or level(op) = the step of the Max-Fillness loop in which the
    operator runs (see max_fillness_steps); a Max-Fillness step is one group.
 4. A group is the set of operator nodes with the same (level, type, number
    of inputs); groups are ordered by level, then type (projection <
    intersection < negation), then input count; members by global id.
 5. Output slots are numbered type-major: all projections first, then all
    intersections, then all negations; inside a type in group order.  The
    gradient row of anchor number a (anchors counted in global-id order) is
    n_slots + a.
 6. Rows of the per-type MLP buffers: projection and negation members use
    their rank inside the type; intersection group g with n members and k
    inputs owns n*k rows from int_row_base(g), input j of member i at
    base + j*n + i.
 7. Gradient index of a table = stable sort of its contributions by row id.
    Relation table: one contribution per projection (in projection-slot
    order), its source being the gradient row of the projection's input.
    Entity table: anchors (anchor order), then one per query for the positive,
    then B*K for the negatives in row-major order.
 8. Storage rows of a forward-only pass with outputs reclaimed as soon as their consumer has
    run: see forward_rows.
"""
import numpy as np

from .model import OP_ANCHOR, OP_PROJ, OP_INTER, OP_NEG, Unsupported, dnf, query_tree

_TYPE_OF = {"p": OP_PROJ, "i": OP_INTER, "n": OP_NEG}


def _class_of(node):
    """Pool of an operator: projections, intersections by input count (C_2, C_3, ...), negations."""
    return (node["type"], len(node["ins"]))


def max_fillness_steps(nodes, b_max=0):
    """The scheduling loop of Alg. 1 on the forward operators, in the paper's notation.

    R: operators that became ready in this cycle; P[tau]: pool (queue) of ready operators of
    class tau; rho(tau) = |P[tau]| / B_max [Sec. 4.1, Eq. for the fillness ratio]; tau* =
    argmax rho; PopBatch takes the first min(|P[tau*]|, B_max) entries.  Canonical choices the
    paper leaves open: R is filed into the pools in node order; ties of rho go to the
    first class in the order projection < intersection (by input count) < negation; b_max = 0
    means no bound; the loop continues until all pools are empty.
    Returns ({operator id: step, 1-based}, peak number of live operator outputs under eager
    reference counting [Sec. 4.3]: an output is freed when its consumer has run, outputs
    without a consumer -- the roots -- stay).
    """
    ops = [g for g, n in enumerate(nodes) if n["type"] != OP_ANCHOR]
    consumer = {}
    for g in ops:
        for c in nodes[g]["ins"]:
            consumer[c] = g
    unmet = {g: sum(1 for c in nodes[g]["ins"] if nodes[c]["type"] != OP_ANCHOR) for g in ops}
    classes = sorted(set(_class_of(nodes[g]) for g in ops))
    P = {tau: [] for tau in classes}
    R = [g for g in ops if unmet[g] == 0]
    step, t, live, peak = {}, 0, 0, 0
    while True:
        for v in sorted(R):
            P[_class_of(nodes[v])].append(v)
        R = []
        if not any(P.values()):
            break
        tau_star = max(classes, key=lambda tau: (len(P[tau]), -classes.index(tau)))
        k = len(P[tau_star]) if b_max == 0 else min(len(P[tau_star]), b_max)
        batch, P[tau_star] = P[tau_star][:k], P[tau_star][k:]
        t += 1
        live += len(batch)
        peak = max(peak, live)
        for o in batch:
            step[o] = t
            live -= sum(1 for c in nodes[o]["ins"] if nodes[c]["type"] != OP_ANCHOR)
            succ = consumer.get(o)
            if succ is not None:
                unmet[succ] -= 1
                if unmet[succ] == 0:
                    R.append(succ)
    return step, peak


def level_peak_live(nodes):
    """Peak of live operator outputs when all operators of one depth are one step."""
    ops = [g for g, n in enumerate(nodes) if n["type"] != OP_ANCHOR]
    live = peak = 0
    for l in sorted(set(nodes[g]["level"] for g in ops)):
        now = [g for g in ops if nodes[g]["level"] == l]
        live += len(now)
        peak = max(peak, live)
        live -= sum(1 for g in now for c in nodes[g]["ins"] if nodes[c]["type"] != OP_ANCHOR)
    return peak


def build_plan(batch, schedule="level", b_max=0):
    """Returns a dict of int32 numpy arrays / ints describing the canonical plan.

    schedule: "level" (one step per depth) or "max_fill" (Alg. 1 with B_max = b_max)."""
    nodes = []            # per global id: dict(type, arg, ins, level, query)
    roots = []            # per query: list of root gids
    for q in range(batch.B):
        branches = dnf(query_tree(batch.query_nodes(q)))
        qroots = []
        for br in branches:
            if br[0] == "e":
                raise Unsupported("a query must contain at least one operator")

            def visit(t):
                if t[0] == "e":
                    nodes.append(dict(type=OP_ANCHOR, arg=t[1], ins=[], level=0))
                elif t[0] == "p":
                    c = visit(t[2])
                    nodes.append(dict(type=OP_PROJ, arg=t[1], ins=[c], level=nodes[c]["level"] + 1))
                else:
                    cs = [visit(c) for c in t[1:]]
                    nodes.append(dict(type=_TYPE_OF[t[0]], arg=0, ins=cs,
                                      level=1 + max(nodes[c]["level"] for c in cs)))
                return len(nodes) - 1

            qroots.append(visit(br))
        roots.append(qroots)

    if schedule == "max_fill":
        step, peak_live = max_fillness_steps(nodes, b_max)
        for g, t in step.items():
            nodes[g]["level"] = t
    else:
        assert schedule == "level"
        peak_live = level_peak_live(nodes)

    ops = [g for g, n in enumerate(nodes) if n["type"] != OP_ANCHOR]
    anchors = [g for g, n in enumerate(nodes) if n["type"] == OP_ANCHOR]

    def gkey(g):
        n = nodes[g]
        return (n["level"], n["type"], len(n["ins"]))

    # slots: type-major
    slot_order = sorted(ops, key=lambda g: (nodes[g]["type"], nodes[g]["level"], len(nodes[g]["ins"]), g))
    slot = {g: s for s, g in enumerate(slot_order)}
    n_slots = len(ops)
    anchor_idx = {g: a for a, g in enumerate(anchors)}
    n_type = [sum(1 for g in ops if nodes[g]["type"] == t) for t in (OP_PROJ, OP_INTER, OP_NEG)]
    type_base = {OP_PROJ: 0, OP_INTER: n_type[0], OP_NEG: n_type[0] + n_type[1]}

    keys = sorted(set(gkey(g) for g in ops))
    members = {k: [] for k in keys}
    for g in ops:                                  # ops is in global-id order
        members[gkey(g)].append(g)

    g_level, g_type, g_nin, g_n, g_out, g_mlp, g_ref, g_rel = [], [], [], [], [], [], [], []
    in_ref, in_gslot, rel = [], [], []
    int_rows = 0
    for k in keys:
        mem = members[k]
        level, typ, nin = k
        n = len(mem)
        g_level.append(level)
        g_type.append(typ)
        g_nin.append(nin)
        g_n.append(n)
        g_out.append(slot[mem[0]])
        g_ref.append(len(in_ref))
        if typ == OP_INTER:
            g_mlp.append(int_rows)
            int_rows += n * nin
        else:
            g_mlp.append(slot[mem[0]] - type_base[typ])
        g_rel.append(len(rel) if typ == OP_PROJ else -1)
        for j in range(nin):
            for g in mem:
                c = nodes[g]["ins"][j]
                if nodes[c]["type"] == OP_ANCHOR:
                    in_ref.append(-1 - nodes[c]["arg"])
                    in_gslot.append(n_slots + anchor_idx[c])
                else:
                    in_ref.append(slot[c])
                    in_gslot.append(slot[c])
        if typ == OP_PROJ:
            rel.extend(nodes[g]["arg"] for g in mem)

    n_levels = max(g_level) if g_level else 0
    lvl_off = [0] * (n_levels + 2)
    for l in g_level:
        lvl_off[l + 1] += 1
    lvl_off = list(np.cumsum(lvl_off))            # groups of level l: [lvl_off[l], lvl_off[l+1])

    root_off, root_slot = [0], []
    for qroots in roots:
        root_slot.extend(slot[g] for g in qroots)
        root_off.append(len(root_slot))

    # relation gradient index: projections in slot order
    proj = slot_order[: n_type[0]]
    rkeys = np.asarray([nodes[g]["arg"] for g in proj], np.int64)
    rsrc_all = []
    for g in proj:
        c = nodes[g]["ins"][0]
        rsrc_all.append(n_slots + anchor_idx[c] if nodes[c]["type"] == OP_ANCHOR else slot[c])
    r_uniq, r_seg_off, r_order = segment_index(rkeys)
    r_src = np.asarray(rsrc_all, np.int32)[r_order] if len(proj) else np.zeros(0, np.int32)

    i32 = lambda x: np.asarray(x, np.int32)
    return dict(
        n_groups=len(keys), n_levels=n_levels, n_slots=n_slots, n_anchor=len(anchors),
        n_proj=n_type[0], n_inter=n_type[1], n_neg=n_type[2], n_int_rows=int_rows,
        n_roots=len(root_slot), peak_live=peak_live,
        lvl_off=i32(lvl_off),
        g_level=i32(g_level), g_type=i32(g_type), g_nin=i32(g_nin), g_n=i32(g_n),
        g_out_base=i32(g_out), g_mlp_base=i32(g_mlp), g_ref_off=i32(g_ref), g_rel_off=i32(g_rel),
        in_ref=i32(in_ref), in_gslot=i32(in_gslot), rel=i32(rel),
        root_off=i32(root_off), root_slot=i32(root_slot),
        anchor_ent=i32([nodes[g]["arg"] for g in anchors]),
        r_uniq=i32(r_uniq), r_seg_off=i32(r_seg_off), r_src=i32(r_src),
    )


def forward_rows(plan):
    """Rows of a forward-only pass under eager reference counting [Sec. 4.3, Reclaim(T): a tensor
    is reclaimed as soon as every operator that consumes it has run; Alg. 1, DecrementRefCounts].

    A forward-only pass (scoring, ranking) needs an operator's output only until its consumer has
    run, so outputs share storage rows.  Canonical assignment (the HIP library's planner must
    reproduce it bit for bit): the plan's steps in order; in a step every output takes, in group and
    member order, the lowest free row (a new row if none is free); when the step has run, the rows
    of the outputs it consumed are free again.  Roots have no consumer and keep their rows.
    Returns (f_row [n_slots]: row of every output slot, number of rows used, and per operator type
    (projection, intersection, negation) the most MLP rows any one step needs)."""
    import heapq
    n_slots, L = int(plan["n_slots"]), int(plan["n_levels"])
    f_row = np.full(n_slots, -1, np.int64)
    free, n_rows = [], 0
    step_rows = np.zeros(3, np.int64)
    lo = plan["lvl_off"]
    for l in range(1, L + 1):
        groups = range(int(lo[l]), int(lo[l + 1]))
        rows_now = np.zeros(3, np.int64)
        for g in groups:
            n, k, t = int(plan["g_n"][g]), int(plan["g_nin"][g]), int(plan["g_type"][g])
            rows_now[{OP_PROJ: 0, OP_INTER: 1, OP_NEG: 2}[t]] += n * (k if t == OP_INTER else 1)
            for i in range(n):
                if free:
                    row = heapq.heappop(free)
                else:
                    row, n_rows = n_rows, n_rows + 1
                f_row[int(plan["g_out_base"][g]) + i] = row
        for g in groups:
            n, k, ro = int(plan["g_n"][g]), int(plan["g_nin"][g]), int(plan["g_ref_off"][g])
            for ref in plan["in_ref"][ro:ro + k * n]:
                if ref >= 0:
                    heapq.heappush(free, int(f_row[ref]))
        step_rows = np.maximum(step_rows, rows_now)
    return f_row.astype(np.int32), n_rows, step_rows.astype(np.int32)


def segment_index(keys):
    """Stable grouping of contributions by key: (unique keys ascending,
    segment offsets [U+1], contribution order)."""
    keys = np.asarray(keys, np.int64)
    order = np.argsort(keys, kind="stable")
    sk = keys[order]
    if sk.shape[0] == 0:
        return np.zeros(0, np.int64), np.zeros(1, np.int64), order
    head = np.ones(sk.shape[0], bool)
    head[1:] = sk[1:] != sk[:-1]
    starts = np.flatnonzero(head)
    return sk[starts], np.concatenate([starts, [sk.shape[0]]]), order


def entity_index(plan, pos, negs):
    """Entity-table gradient index for one step: contributions are
    [anchors | positives | negatives row-major]; returns int32
    (uniq ids, seg_off, src = contribution numbers in segment order)."""
    keys = np.concatenate([np.asarray(plan["anchor_ent"], np.int64),
                           np.asarray(pos, np.int64),
                           np.asarray(negs, np.int64).reshape(-1)])
    u, off, order = segment_index(keys)
    return u.astype(np.int32), off.astype(np.int32), order.astype(np.int32)
