"""Pins of the reference planner: per-template operator census (closed form from
the 14 query shapes), structural invariants of operator-level scheduling
(every operator exactly once, only after its inputs; groups homogeneous in type
and input count), and brute-force checks of the gradient indices."""
import numpy as np
import pytest

import workloads as wl
from oracle import model as om
from oracle import plan as oplan

P, I, N = om.OP_PROJ, om.OP_INTER, om.OP_NEG

# template -> (anchors, roots, {(level, type, nin): count})
CENSUS = {
    "1p": (1, 1, {(1, P, 1): 1}),
    "2p": (1, 1, {(1, P, 1): 1, (2, P, 1): 1}),
    "3p": (1, 1, {(1, P, 1): 1, (2, P, 1): 1, (3, P, 1): 1}),
    "2i": (2, 1, {(1, P, 1): 2, (2, I, 2): 1}),
    "3i": (3, 1, {(1, P, 1): 3, (2, I, 3): 1}),
    "ip": (2, 1, {(1, P, 1): 2, (2, I, 2): 1, (3, P, 1): 1}),
    "pi": (2, 1, {(1, P, 1): 2, (2, P, 1): 1, (3, I, 2): 1}),
    "2u": (2, 2, {(1, P, 1): 2}),
    "up": (2, 2, {(1, P, 1): 2, (2, P, 1): 2}),
    "2in": (2, 1, {(1, P, 1): 2, (2, N, 1): 1, (3, I, 2): 1}),
    "3in": (3, 1, {(1, P, 1): 3, (2, N, 1): 1, (3, I, 3): 1}),
    "inp": (2, 1, {(1, P, 1): 2, (2, N, 1): 1, (3, I, 2): 1, (4, P, 1): 1}),
    "pin": (2, 1, {(1, P, 1): 2, (2, P, 1): 1, (2, N, 1): 1, (3, I, 2): 1}),
    "pni": (2, 1, {(1, P, 1): 2, (2, P, 1): 1, (3, N, 1): 1, (4, I, 2): 1}),
}


@pytest.fixture(scope="module")
def kg():
    return wl.make_kg(400, 12, 4000, 2.1, 11)


def census_of(plan):
    return {(int(l), int(t), int(k)): int(n) for l, t, k, n in
            zip(plan["g_level"], plan["g_type"], plan["g_nin"], plan["g_n"])}


@pytest.mark.parametrize("name", sorted(CENSUS))
def test_single_template_census(kg, name):
    qb = wl.make_batch(kg, 5, {name: 1.0}, 3)
    plan = oplan.build_plan(qb)
    anchors, roots, groups = CENSUS[name]
    assert plan["n_anchor"] == 5 * anchors
    assert plan["n_roots"] == 5 * roots
    assert census_of(plan) == {k: 5 * v for k, v in groups.items()}


def test_mixed_batch_census_is_the_sum_over_templates(kg):
    qb = wl.make_batch(kg, 200, {n: 1.0 for n in CENSUS}, 4)
    plan = oplan.build_plan(qb)
    want, anchors, roots = {}, 0, 0
    for name in qb.names:
        a, r, g = CENSUS[name]
        anchors += a
        roots += r
        for k, v in g.items():
            want[k] = want.get(k, 0) + v
    assert census_of(plan) == want
    assert plan["n_anchor"] == anchors and plan["n_roots"] == roots
    assert plan["n_levels"] == 4
    # the 14-template mean the scope table quotes: 27/14 anchors, 37/14 projections per query
    tot = {n: CENSUS[n] for n in CENSUS}
    assert sum(a for a, _, _ in tot.values()) == 27
    assert sum(v for _, _, g in tot.values() for (l, t, k), v in g.items() if t == P) == 37


def check_invariants(qb, plan, asap=True):
    S, A = plan["n_slots"], plan["n_anchor"]
    G = plan["n_groups"]
    level_of_slot = np.full(S, -1)
    type_of_slot = np.full(S, -1)
    seen = np.zeros(S, int)
    keys = []
    mlp_rows = {P: [], I: [], N: []}
    for g in range(G):
        l, t, k, n = (int(plan[x][g]) for x in ("g_level", "g_type", "g_nin", "g_n"))
        keys.append((l, t, k))
        ob = int(plan["g_out_base"][g])
        seen[ob:ob + n] += 1
        level_of_slot[ob:ob + n] = l
        type_of_slot[ob:ob + n] = t
        mb = int(plan["g_mlp_base"][g])
        mlp_rows[t].extend(range(mb, mb + n * (k if t == I else 1)))
    assert keys == sorted(keys) and len(set(keys)) == G          # ordered, one group per key
    assert np.all(seen == 1)                                     # every operator exactly once
    assert np.all(np.diff(type_of_slot) >= 0)                    # slots are type-major
    for t, n in ((P, plan["n_proj"]), (N, plan["n_neg"]), (I, plan["n_int_rows"])):
        assert sorted(mlp_rows[t]) == list(range(n))
    consumers = np.zeros(S + A, int)
    for g in range(G):
        l, t, k, n = (int(plan[x][g]) for x in ("g_level", "g_type", "g_nin", "g_n"))
        ro = int(plan["g_ref_off"][g])
        refs = plan["in_ref"][ro:ro + k * n].reshape(k, n)
        gs = plan["in_gslot"][ro:ro + k * n].reshape(k, n)
        lv = np.where(refs >= 0, level_of_slot[np.maximum(refs, 0)], 0)
        assert np.all(lv < l)                                        # inputs run in earlier steps
        if asap:
            assert np.all(lv.max(axis=0) == l - 1)                   # ASAP levels
        assert np.all(gs[refs >= 0] == refs[refs >= 0])
        assert np.all(gs[refs < 0] >= S)
        assert np.array_equal(plan["anchor_ent"][gs[refs < 0] - S], -1 - refs[refs < 0])
        np.add.at(consumers, gs.reshape(-1), 1)
        if t == P:
            assert k == 1 and plan["g_rel_off"][g] >= 0
        else:
            assert plan["g_rel_off"][g] == -1
    for s in plan["root_slot"]:
        consumers[s] += 1
    assert np.all(consumers == 1)                                # trees: one consumer each
    assert plan["root_off"][0] == 0 and plan["root_off"][-1] == plan["n_roots"]
    lo = plan["lvl_off"]
    assert lo[0] == 0 and lo[1] == 0 and lo[-1] == G
    for l in range(1, plan["n_levels"] + 1):
        assert np.all(plan["g_level"][lo[l]:lo[l + 1]] == l)


def test_plan_invariants_mixed(kg):
    qb = wl.make_batch(kg, 300, {n: 1.0 for n in CENSUS}, 9)
    check_invariants(qb, oplan.build_plan(qb))


@pytest.mark.parametrize("schedule,b_max", [("level", 0), ("max_fill", 0), ("max_fill", 7)])
def test_plan_values_through_refs_match_per_query_execution(kg, schedule, b_max):
    """Executing the plan's groups step by step with the oracle's operators gives,
    at every root slot, the per-query branch embedding -- whatever the schedule."""
    qb = wl.make_batch(kg, 40, {n: 1.0 for n in CENSUS}, 10)
    plan = oplan.build_plan(qb, schedule, b_max)
    p = wl.make_params(400, 12, 8, 16, 5)
    M = om.Model(p, 12.0)
    Pm = M.P
    A = np.zeros((plan["n_slots"], 8))
    for g in range(plan["n_groups"]):
        t, k, n = (int(plan[x][g]) for x in ("g_type", "g_nin", "g_n"))
        ro, ob = int(plan["g_ref_off"][g]), int(plan["g_out_base"][g])
        refs = plan["in_ref"][ro:ro + k * n].reshape(k, n)
        for i in range(n):
            xs = [A[r] if r >= 0 else Pm["E"][-1 - r] for r in refs[:, i]]
            if t == P:
                r = int(plan["rel"][int(plan["g_rel_off"][g]) + i])
                A[ob + i] = om.mlp_forward(xs[0] + Pm["R"][r], Pm["W1"], Pm["b1"], Pm["W2"], Pm["b2"])[0]
            elif t == N:
                A[ob + i] = om.mlp_forward(xs[0], Pm["V1"], Pm["c1"], Pm["V2"], Pm["c2"])[0]
            else:
                att = np.stack([om.mlp_forward(x, Pm["U1"], Pm["u1"], Pm["U2"], Pm["u2"])[0] for x in xs])
                w = np.exp(att - att.max(0))
                w /= w.sum(0)
                A[ob + i] = (w * np.stack(xs)).sum(0)
    for q in range(qb.B):
        br = om.dnf(qb.tree(q))
        slots = plan["root_slot"][plan["root_off"][q]:plan["root_off"][q + 1]]
        assert len(br) == len(slots)
        for b, s in zip(br, slots):
            np.testing.assert_allclose(A[s], om.forward(b, M)[0], rtol=1e-12, atol=1e-14)


# ---------------------------------------------------------------- Max-Fillness schedule (Alg. 1)
def test_max_fillness_hand_worked_schedule():
    """Three queries worked by hand.  Node ids: q0 = p(p(e)): e0 p1 p2; q1 = i(p(e), p(e)):
    e3 p4 e5 p6 i7; q2 = n(p(e)): e8 p9 n10.
    Unbounded: cycle 1 files p1 p4 p6 p9 -> step 1 runs all four projections; then p2, i7, n10
    are ready, one per pool: the tie goes projection, intersection, negation (steps 2, 3, 4).
    B_max = 3: step 1 takes the first three of the pool (p1 p4 p6), p9 stays; p2 and i7 become
    ready; the projection pool [p9, p2] is the fullest -> step 2; then n10 is ready next to i7:
    step 3 intersection, step 4 negation.
    Live outputs (an output dies when its consumer has run, roots stay): unbounded 4, then
    +1 (5, the peak) -1, +1 -2, +1 -1; bounded 3, then +2 (5) -1, +1 -2, +1 -1."""
    trees = [("p", 1, ("p", 0, ("e", 1))), ("i", ("p", 2, ("e", 2)), ("p", 3, ("e", 3))), ("n", ("p", 4, ("e", 4)))]
    qb = wl.batch_from_trees(trees, [5, 6, 7])
    for b_max, want_n, want_rel in ((0, [4, 1, 1, 1], [[0, 2, 3, 4], [1]]), (3, [3, 2, 1, 1], [[0, 2, 3], [1, 4]])):
        plan = oplan.build_plan(qb, "max_fill", b_max)
        assert list(plan["g_level"]) == [1, 2, 3, 4] and plan["n_levels"] == 4
        assert list(plan["g_type"]) == [P, P, I, N]
        assert list(plan["g_n"]) == want_n
        assert list(plan["rel"][:want_n[0]]) == want_rel[0]
        assert list(plan["rel"][want_n[0]:]) == want_rel[1]
        assert plan["peak_live"] == 5
    # the level-synchronous order of the same batch: 4 projections, then p + i + n together
    lvl = oplan.build_plan(qb)
    assert list(lvl["g_level"]) == [1, 2, 2, 2] and lvl["peak_live"] == 7


def test_forward_rows_hand_worked():
    """The three queries above, outputs reclaimed when their consumer has run.  Output slots are
    type-major: unbounded p1 p4 p6 p9 = 0..3, p2 = 4, i7 = 5, n10 = 6.  Step 1 fills rows 0..3; step 2
    (p2) finds no free row: row 4, then p1's row 0 is free; step 3 (i7) takes row 0 and frees rows 1
    and 2 (p4, p6); step 4 (n10) takes row 1: five rows, the peak of live outputs.
    B_max = 3: step 1 p1 p4 p6 = slots and rows 0..2; step 2 runs p2 (slot 3) and p9 (slot 4) into
    rows 3 and 4 and frees row 0; step 3 i7 -> row 0, frees 1 and 2; step 4 n10 -> row 1.
    Level-synchronous: p2, i7 and n10 run in one step beside their inputs: seven rows, no reuse."""
    trees = [("p", 1, ("p", 0, ("e", 1))), ("i", ("p", 2, ("e", 2)), ("p", 3, ("e", 3))), ("n", ("p", 4, ("e", 4)))]
    qb = wl.batch_from_trees(trees, [5, 6, 7])
    for b_max in (0, 3):
        plan = oplan.build_plan(qb, "max_fill", b_max)
        f_row, n_rows, step_rows = oplan.forward_rows(plan)
        assert list(f_row) == [0, 1, 2, 3, 4, 0, 1] and n_rows == 5 == plan["peak_live"]
        assert list(step_rows) == ([4, 2, 1] if b_max == 0 else [3, 2, 1])
    f_row, n_rows, step_rows = oplan.forward_rows(oplan.build_plan(qb))
    assert list(f_row) == list(range(7)) and n_rows == 7 and list(step_rows) == [4, 2, 1]


@pytest.mark.parametrize("schedule,b_max", [("level", 0), ("max_fill", 0), ("max_fill", 7)])
def test_forward_rows_no_row_is_read_after_it_was_reassigned(kg, schedule, b_max):
    """Replaying the steps with one value cell per row: every input row still holds the output it is
    read for, every root's row holds the root at the end, the rows used equal the peak of live
    outputs, and executing the plan through these rows gives the per-query embeddings."""
    qb = wl.make_batch(kg, 60, {n: 1.0 for n in CENSUS}, 12)
    plan = oplan.build_plan(qb, schedule, b_max)
    f_row, n_rows, step_rows = oplan.forward_rows(plan)
    assert n_rows == plan["peak_live"] and f_row.min() == 0 and f_row.max() == n_rows - 1
    p = wl.make_params(400, 12, 8, 16, 5)
    M = om.Model(p, 12.0)
    Pm = M.P
    holder = np.full(n_rows, -1)
    A = np.zeros((n_rows, 8))
    lo = plan["lvl_off"]
    rows_seen = np.zeros(3, int)
    for l in range(1, plan["n_levels"] + 1):
        new = {}
        rows_now = np.zeros(3, int)
        for g in range(lo[l], lo[l + 1]):
            t, k, n = (int(plan[x][g]) for x in ("g_type", "g_nin", "g_n"))
            rows_now[[P, I, N].index(t)] += n * (k if t == I else 1)
            ro, ob = int(plan["g_ref_off"][g]), int(plan["g_out_base"][g])
            refs = plan["in_ref"][ro:ro + k * n].reshape(k, n)
            for i in range(n):
                for r in refs[:, i]:
                    assert r < 0 or holder[f_row[r]] == r, "row reassigned before its reader ran"
                xs = [A[f_row[r]] if r >= 0 else Pm["E"][-1 - r] for r in refs[:, i]]
                if t == P:
                    rr = int(plan["rel"][int(plan["g_rel_off"][g]) + i])
                    y = om.mlp_forward(xs[0] + Pm["R"][rr], Pm["W1"], Pm["b1"], Pm["W2"], Pm["b2"])[0]
                elif t == N:
                    y = om.mlp_forward(xs[0], Pm["V1"], Pm["c1"], Pm["V2"], Pm["c2"])[0]
                else:
                    att = np.stack([om.mlp_forward(x, Pm["U1"], Pm["u1"], Pm["U2"], Pm["u2"])[0] for x in xs])
                    w = np.exp(att - att.max(0))
                    w /= w.sum(0)
                    y = (w * np.stack(xs)).sum(0)
                new[ob + i] = y
        for s_, y in new.items():          # the outputs of a step are written when its inputs have been read
            assert holder[f_row[s_]] == -1 or holder[f_row[s_]] not in plan["root_slot"]
            holder[f_row[s_]] = s_
            A[f_row[s_]] = y
        rows_seen = np.maximum(rows_seen, rows_now)
    assert list(rows_seen) == list(step_rows)
    for q in range(qb.B):
        br = om.dnf(qb.tree(q))
        slots = plan["root_slot"][plan["root_off"][q]:plan["root_off"][q + 1]]
        for b, s_ in zip(br, slots):
            assert holder[f_row[s_]] == s_
            np.testing.assert_allclose(A[f_row[s_]], om.forward(b, M)[0], rtol=1e-12, atol=1e-14)


CLASS_ORDER = [(P, 1)] + [(I, k) for k in range(2, 9)] + [(N, 1)]


@pytest.mark.parametrize("b_max", [0, 1, 5, 50])
def test_max_fillness_invariants_and_greedy_choice(kg, b_max):
    """Every step is one class of at most B_max operators whose inputs ran earlier, and -- replaying
    the plan -- the class that ran was the fullest pool of that cycle (ties to the first class),
    cut at B_max."""
    qb = wl.make_batch(kg, 120, {n: 1.0 for n in CENSUS}, 31)
    plan = oplan.build_plan(qb, "max_fill", b_max)
    check_invariants(qb, plan, asap=False)
    S, G = plan["n_slots"], plan["n_groups"]
    assert G == plan["n_levels"] and list(plan["g_level"]) == list(range(1, G + 1))   # one group per step
    step = np.zeros(S, int)
    cls = [None] * S
    ready_at = np.ones(S, int)
    for g in range(G):
        t, k, n = (int(plan[x][g]) for x in ("g_type", "g_nin", "g_n"))
        ob, ro = int(plan["g_out_base"][g]), int(plan["g_ref_off"][g])
        assert b_max == 0 or n <= b_max
        step[ob:ob + n] = g + 1
        for i in range(n):
            cls[ob + i] = (t, k)
    for g in range(G):
        t, k, n = (int(plan[x][g]) for x in ("g_type", "g_nin", "g_n"))
        ob, ro = int(plan["g_out_base"][g]), int(plan["g_ref_off"][g])
        refs = plan["in_ref"][ro:ro + k * n].reshape(k, n)
        for i in range(n):
            ins = [step[r] for r in refs[:, i] if r >= 0]
            ready_at[ob + i] = 1 + max(ins) if ins else 1
    for t in range(1, G + 1):
        waiting = [s for s in range(S) if ready_at[s] <= t <= step[s]]
        count = {c: sum(1 for s in waiting if cls[s] == c) for c in CLASS_ORDER}
        best = max(CLASS_ORDER, key=lambda c: (count[c], -CLASS_ORDER.index(c)))
        ran = (int(plan["g_type"][t - 1]), int(plan["g_nin"][t - 1]))
        assert ran == best, (t, ran, best, count)
        assert int(plan["g_n"][t - 1]) == (count[best] if b_max == 0 else min(count[best], b_max))
    if b_max == 1:
        assert G == S
    # an unbounded step never leaves ready operators of its class behind
    if b_max == 0:
        for t in range(1, G + 1):
            assert not any(ready_at[s] <= t < step[s] and cls[s] == cls[np.flatnonzero(step == t)[0]] for s in range(S))
    # reclamation can only help: never more live outputs than operators
    assert 0 < plan["peak_live"] <= S


def test_max_fillness_single_chain_templates(kg):
    """Ten 3p chains are 30 projections in one pool.  Unbounded, a step drains the pool, so
    the steps are the three depths.  With B_max = 4 the single pool is never empty before the
    end (every step of 4 makes up to 4 successors ready): 7 steps of 4 and one of 2, and the
    first come first served order mixes depths inside a step."""
    qb = wl.make_batch(kg, 10, {"3p": 1.0}, 3)
    assert list(oplan.build_plan(qb, "max_fill", 0)["g_n"]) == [10, 10, 10]
    plan = oplan.build_plan(qb, "max_fill", 4)
    assert list(plan["g_n"]) == [4] * 7 + [2]
    # step 3 holds the last two first-hop projections (anchor inputs) and two second hops
    ro = int(plan["g_ref_off"][2])
    assert sorted(int(r) < 0 for r in plan["in_ref"][ro:ro + 4]) == [False, False, True, True]


def brute_index(keys):
    uniq = sorted(set(int(k) for k in keys))
    off, src = [0], []
    for u in uniq:
        src.extend(i for i, k in enumerate(keys) if int(k) == u)
        off.append(len(src))
    return uniq, off, src


def test_gradient_indices_against_brute_force(kg):
    qb = wl.make_batch(kg, 30, {n: 1.0 for n in CENSUS}, 12)
    plan = oplan.build_plan(qb)
    negs = wl.make_negatives(400, 30, 6, 13)
    negs[:, 0] = negs[0, 0]                      # one entity hit by every query
    u, off, src = oplan.entity_index(plan, qb.pos, negs)
    keys = list(plan["anchor_ent"]) + list(qb.pos) + list(negs.reshape(-1))
    bu, boff, bsrc = brute_index(keys)
    assert list(u) == bu and list(off) == boff and list(src) == bsrc
    # relation index: one contribution per projection, source = gradient row of its input
    S = plan["n_slots"]
    rel_of_proj, src_of_proj = [None] * plan["n_proj"], [None] * plan["n_proj"]
    for g in range(plan["n_groups"]):
        if plan["g_type"][g] != P:
            continue
        n, ob, ro, rl = (int(plan[x][g]) for x in ("g_n", "g_out_base", "g_ref_off", "g_rel_off"))
        for i in range(n):
            rel_of_proj[ob + i] = int(plan["rel"][rl + i])
            src_of_proj[ob + i] = int(plan["in_gslot"][ro + i])
    bu, boff, bsrc = brute_index(rel_of_proj)
    assert list(plan["r_uniq"]) == bu and list(plan["r_seg_off"]) == boff
    assert list(plan["r_src"]) == [src_of_proj[i] for i in bsrc]
    assert all(0 <= s < S + plan["n_anchor"] for s in plan["r_src"])


def test_unsupported_and_degenerate():
    bad = wl.batch_from_trees([("i", ("u", ("p", 0, ("e", 1)), ("p", 1, ("e", 2))), ("p", 0, ("e", 3)))], [0])
    with pytest.raises(om.Unsupported):
        oplan.build_plan(bad)
    with pytest.raises(om.Unsupported):
        oplan.build_plan(wl.batch_from_trees([("e", 3)], [0]))
    empty = oplan.build_plan(wl.batch_from_trees([], []))
    assert empty["n_groups"] == 0 and empty["n_slots"] == 0 and list(empty["root_off"]) == [0]
    # a union of three branches under two projections
    q = ("p", 5, ("p", 4, ("u", ("p", 0, ("e", 1)), ("p", 1, ("e", 2)), ("p", 2, ("e", 3)))))
    pl = oplan.build_plan(wl.batch_from_trees([q], [0]))
    assert pl["n_roots"] == 3 and pl["n_proj"] == 9 and pl["n_levels"] == 3
    assert list(pl["rel"]) == [0, 1, 2, 4, 4, 4, 5, 5, 5]
