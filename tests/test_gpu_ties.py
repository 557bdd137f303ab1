"""Inputs that sit exactly on a kink of the model (needs an MI355X).

The other GPU cases keep a margin from every kink, because within fp32 rounding of one two
correct implementations may decide differently.  Exactly on a kink nothing is left to rounding:
the stated rules decide -- relu'(0) = 0, sign(0) = 0, equal branch distances -> the lowest
branch, equal distances in a ranking -> the lower entity id -- and the library must take the
same decisions as the oracle.  The inputs here are built so that the kink values are exact in
both precisions (zeros that come from zero weights, bit-identical rows)."""
import numpy as np
import pytest

import workloads as wl
from oracle import model as om
from oracle import plan as oplan
from oracle import rank as orank
from tests import parity as par

pytestmark = pytest.mark.gpu

_say = par.say


def _proj(rng, N, R, depth=1):
    t = ("e", int(rng.integers(N)))
    for _ in range(depth):
        t = ("p", int(rng.integers(R)), t)
    return t


def test_union_of_identical_branches_gradient_goes_to_the_first():
    """Both branches of a union are the same sub-query: their embeddings and distances are bit-identical,
    every candidate ties, the lower branch wins (strict `<`), the second branch gets no gradient."""
    _say("ties: unions whose branches are identical (2u, up, 3-way), mixed with ordinary queries")
    rng = np.random.default_rng(71)
    N, R, d, h = 400, 7, 48, 96
    trees = []
    for i in range(40):
        b = _proj(rng, N, R, 1 + i % 2)
        kind = i % 4
        if kind == 0:
            trees.append(("u", b, b))
        elif kind == 1:
            trees.append(("p", int(rng.integers(R)), ("u", b, b)))
        elif kind == 2:
            trees.append(("u", b, b, b))
        else:
            trees.append(("i", _proj(rng, N, R), _proj(rng, N, R, 2)))
    pos = [int(rng.integers(N)) for _ in trees]
    case = par.Case(N, R, d, h, 0, 7, 6.0, seed=72, trees=trees, pos=pos, exact_kinks=True)
    eng = par.check_forward_backward(case)
    # the library's own statement of the rule: the gradient rows of all but the first branch are zero
    plan = eng.plan(case.qb)
    eng.forward_backward(plan, case.neg_dev())
    g = eng.grads()
    pe = plan.export()
    n_checked = 0
    for q in range(case.B):
        if case.qb.tree(q)[0] == "i":
            continue
        slots = pe["root_slot"][pe["root_off"][q]:pe["root_off"][q + 1]]
        assert len(slots) >= 2
        assert np.array_equal(g["act"][slots[0]], g["act"][slots[1]])          # bit-identical branches
        assert np.any(g["dact"][slots[0]] != 0.0)
        for s in slots[1:]:
            assert not np.any(g["dact"][s]), "query %d: a later branch of a tie received gradient" % q
        n_checked += 1
    assert n_checked == 30
    plan.free()
    par.check_train_steps(case, steps=1)


def test_dead_hidden_units_and_zero_differences():
    """Hidden units with zero weights and zero bias in every MLP (pre-activation exactly 0: no
    gradient through them, relu'(0) = 0), and one coordinate in which every projection output and
    every entity row hold the same value (difference exactly 0: sign(0) = 0, no gradient to either
    side from any pair)."""
    _say("ties: dead hidden units (relu'(0) = 0); a coordinate where y == E[e] exactly (sign(0) = 0)")
    N, R, d, h = 500, 9, 40, 56
    dead = {"W1": ("b1", "W2", [3, 17, 55]), "V1": ("c1", "V2", [0, 31]), "U1": ("u1", "U2", [8, 40])}
    coord, beta = 5, np.float32(0.0625)

    def edit(P):
        for wa, (ba, wb, units) in dead.items():
            P[wa][units, :] = 0.0
            P[ba][units] = 0.0
        # projection outputs: coordinate `coord` is b2[coord] exactly (zero row of W2)
        P["W2"][coord, :] = 0.0
        P["b2"][coord] = beta
        P["E"][:, coord] = beta

    # every root is a projection, so every root embedding holds beta in that coordinate
    mix = {n: 1.0 for n in ("1p", "2p", "3p", "ip", "inp", "2u", "up")}
    case = par.Case(N, R, d, h, 60, 6, 5.0, mix=mix, seed=81, exact_kinks=True, params_edit=edit)
    assert any(n == "inp" for n in case.qb.names) and any(n == "ip" for n in case.qb.names)
    eng = par.check_forward_backward(case)
    plan = eng.plan(case.qb)
    eng.forward_backward(plan, case.neg_dev())
    g = eng.grads()
    pe = plan.export()
    for wa, (ba, wb, units) in dead.items():
        assert not np.any(g[wa][units, :]), wa + ": gradient through a unit with relu'(0)"
        assert not np.any(g[ba][units]), ba
        assert not np.any(g[wb][:, units]), wb + ": a dead unit's output is 0, so is its weight gradient"
    # sign(0) = 0: the roots get nothing in that coordinate; entity rows get only what arrives
    # through anchors (pairs contribute exactly 0)
    roots = pe["root_slot"]
    assert np.all(g["act"][roots][:, coord] == beta)
    assert not np.any(g["dact"][roots][:, coord])
    _, _, G, _ = case.oracle_grads()
    anchors = set(int(a) for a in pe["anchor_ent"])
    only_pairs = np.array([int(e) not in anchors for e in g["e_uniq"]])
    assert only_pairs.sum() > 50
    assert not np.any(g["gE"][only_pairs][:, coord])
    for e in g["e_uniq"][only_pairs]:
        assert G.rows["E"][int(e)][coord] == 0.0
    plan.free()
    par.check_train_steps(case, steps=2)


def test_ranking_ties_go_to_the_lower_entity_id():
    """Every entity has a twin with a bit-identical row (id + N/2): all-entity top-k must list the
    lower id first and, where only one of the two fits, return the lower; a twin at the same
    distance is not strictly closer, so filtered ranks do not count it."""
    _say("ties: twin entity rows in the all-entity top-k (k = 1, 5, 10) and in filtered ranks")
    import torch
    N, R, d, h, half = 1000, 12, 32, 64, 500

    def edit(P):
        P["E"][half:] = P["E"][:half]

    case = par.Case(N, R, d, h, 48, 4, 8.0, seed=91, params_edit=edit)
    M = case.model()
    eng = case.engine()
    plan = eng.plan(case.qb)
    full = [case.distances_all(case.qb, q, M) for q in range(case.B)]
    for k in (1, 5, 10):
        ids, dist = eng.rank_all(plan, k)
        torch.cuda.synchronize()
        ids, dist = ids.cpu().numpy(), dist.cpu().numpy()
        for q in range(case.B):
            assert np.array_equal(full[q][:half], full[q][half:])              # the oracle sees the twins too
            want_ids, want_d = orank.topk_all(case.qb, q, M, k, case.distances_all)
            par.assert_close(dist[q], want_d, "top-%d distances q%d" % (k, q))
            got = list(ids[q])
            for j, e in enumerate(got):
                if e >= half:      # an upper twin is listed only right after its lower twin, at the same distance
                    assert j > 0 and got[j - 1] == e - half and dist[q][j] == dist[q][j - 1], (k, q, got)
            if got[-1] < half and k > 1:
                assert got[-1] + half not in got
            # wherever fp32 keeps the oracle's order of the distinct rows, the ids are the oracle's exactly
            lower = np.sort(full[q][:half])
            if np.all(np.diff(lower[:k + 1]) > 1e-5 * lower[k]):
                assert got == list(want_ids), (k, q, got, list(want_ids))
    # filtered ranks: answers whose twin is not listed
    rng = np.random.default_rng(5)
    lists = []
    for q in range(case.B):
        near = np.argsort(full[q][:half], kind="stable")[:8]
        ans = [int(a) + (half if rng.random() < 0.5 else 0) for a in rng.choice(near, 3, replace=False)]
        lists.append(ans + [int(x) for x in rng.choice(half, 2, replace=False) if int(x) not in ans and int(x) + half not in ans])
    off = np.concatenate([[0], np.cumsum([len(l) for l in lists])]).astype(np.int32)
    flat = np.asarray([a for l in lists for a in l], np.int32)
    dev = lambda x: torch.from_numpy(x).cuda()
    ranks, adist, _ = eng.rank_answers(plan, dev(off), dev(flat), None)
    ranks, adist = ranks.cpu().numpy(), adist.cpu().numpy()
    exact = 0
    for q in range(case.B):
        a = np.asarray(lists[q], np.int64)
        want, d_ref = orank.filtered_ranks(case.qb, q, a, M, case.distances_all)
        got = ranks[off[q]:off[q + 1]]
        other = np.ones(N, bool)
        other[a] = False
        for j, e in enumerate(a):
            twin = (int(e) + half) % N
            assert other[twin]                                                 # the twin competes, at equal distance
            d_other = full[q][other]
            # no third entity within fp32 rounding of the answer's distance: the rank is decided, and a
            # library that counted the twin as closer would be off by one
            near_tie = np.sum(np.abs(d_other - d_ref[j]) <= 1e-5 * d_ref[j])
            if near_tie == 1:
                assert got[j] == want[j], "q%d answer %d: rank %d, oracle %d" % (q, e, got[j], want[j])
                exact += 1
    _say("filtered ranks with twins: %d of %d answers decided exactly" % (exact, len(flat)))
    assert exact >= 0.8 * len(flat)
    plan.free()
