"""Pins of the box-family oracle against things that are not the oracle: hand-worked
numbers, closed forms, invariants, torch autograd.  All CPU, all small."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import box as ob
from oracle import model as om

HP = dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, gamma=12.0, alpha=0.25)


def tiny(seed=0, N=50, R=6, d=8, h=16, B=12, K=4, T=400, mix=None):
    kg = wl.make_kg(N, R, T, 2.1, seed)
    qb = wl.make_batch(kg, B, mix or {n: 1.0 for n in wl.EPFO9}, seed + 1)
    negs = wl.make_negatives(N, B, K, seed + 2)
    return kg, qb, negs, wl.make_box_params(N, R, d, h, seed + 3)


def test_distance_hand_worked():
    """centre (1, 2, 0), offset (0.5, 0, 1), entity (2, 2.5, 0.5): |e-c| = (1, .5, .5); outside parts
    (.5, .5, 0) sum to 1; inside parts (.5, 0, .5) sum to 1; alpha = 1/4 -> 1.25."""
    C = np.array([[1.0, 2.0, 0.0]])
    O = np.array([[0.5, 0.0, 1.0]])
    e = np.array([[2.0, 2.5, 0.5]])
    assert ob.box_distance(C, O, e, 0.25)[0, 0] == pytest.approx(1.25, abs=1e-15)
    s, win = ob.score(C, O, e, 12.0, 0.25)
    assert s[0] == pytest.approx(10.75, abs=1e-15) and win[0] == 0


def test_1p_closed_form_and_relu_on_relation_offsets():
    _, _, _, p = tiny(d=6, h=5)
    a, t = 3, 7
    r = int(np.argmax((p["Ro"] < 0).any(axis=1)))        # a relation with a negative raw offset
    nodes = [(om.OP_ANCHOR, a, []), (om.OP_PROJ, r, [0])]
    M = ob.BoxModel(p, 12.0, 0.25)
    c, o, _ = ob.forward(om.query_tree(nodes), M)
    P = M.P
    np.testing.assert_allclose(c, P["E"][a] + P["R"][r], rtol=0, atol=0)
    np.testing.assert_allclose(o, np.where(P["Ro"][r] > 0, P["Ro"][r], 0.0), rtol=0, atol=0)
    assert (P["Ro"][r] < 0).any() and (o >= 0).all()
    _, s = ob.query_step(nodes, t, [1, 2], M, 1)
    diff = np.abs(P["E"][t] - c)
    want = 12.0 - np.maximum(diff - o, 0).sum() - 0.25 * np.minimum(diff, o).sum()
    assert s[0] == pytest.approx(want, rel=1e-14)


def test_zero_offsets_give_the_l1_distance_and_inside_points_the_scaled_one():
    rng = np.random.default_rng(0)
    C, e = rng.standard_normal((2, 7)), rng.standard_normal((5, 7))
    d0 = ob.box_distance(C, np.zeros_like(C), e, 0.3)
    np.testing.assert_allclose(d0, np.abs(C[:, None] - e[None]).sum(-1), rtol=1e-14)
    big = np.full_like(C, 100.0)
    np.testing.assert_allclose(ob.box_distance(C, big, e, 0.3), 0.3 * d0, rtol=1e-14)
    # alpha = 1 makes inside and outside the same: the distance is the L1 distance for any offsets
    O = np.abs(rng.standard_normal(C.shape))
    np.testing.assert_allclose(ob.box_distance(C, O, e, 1.0), d0, rtol=1e-14)


def test_intersection_of_identical_boxes_and_permutation_invariance():
    _, _, _, p = tiny(d=6, h=5)
    M = ob.BoxModel(p, 12.0, 0.25)
    one = ("p", 1, ("e", 4))
    c1, o1, _ = ob.forward(one, M)
    c, o, _ = ob.forward(("i", one, one, one), M)
    np.testing.assert_allclose(c, c1, rtol=1e-13)
    g, _ = om.mlp_forward(o1, M.P["V1"], M.P["c1"], M.P["V2"], M.P["c2"])
    np.testing.assert_allclose(o, o1 / (1.0 + np.exp(-g)), rtol=1e-13)
    assert (o <= o1 + 1e-15).all()                       # an intersection never grows a box
    two = ("p", 3, ("p", 0, ("e", 9)))
    ca, oa, _ = ob.forward(("i", one, two), M)
    cb, obb, _ = ob.forward(("i", two, one), M)
    np.testing.assert_allclose(ca, cb, rtol=1e-13)
    np.testing.assert_allclose(oa, obb, rtol=1e-13)


def test_union_takes_the_closest_branch_and_negation_is_refused():
    _, _, _, p = tiny(d=6, h=5)
    M = ob.BoxModel(p, 12.0, 0.25)
    n2u = [(0, 4, []), (1, 1, [0]), (0, 9, []), (1, 3, [2]), (om.OP_UNION, 0, [1, 3])]
    _, s = ob.query_step(n2u, 5, [1, 2, 3], M, 1)
    _, sa = ob.query_step(n2u[:2], 5, [1, 2, 3], M, 1)
    _, sb = ob.query_step(n2u[2:4][:1] + [(1, 3, [0])], 5, [1, 2, 3], M, 1)
    np.testing.assert_allclose(s, np.maximum(sa, sb), rtol=1e-14)
    with pytest.raises(om.Unsupported):
        ob.query_step([(0, 4, []), (1, 1, [0]), (om.OP_NEG, 0, [1])], 5, [1], M, 1)


def test_distances_to_all_entities_by_explicit_loops_and_against_the_training_scores():
    _, qb, negs, p = tiny(seed=5, N=40, B=9, K=3)
    M = ob.BoxModel(p, 12.0, 0.25)
    E = M.P["E"]
    for i in range(qb.B):
        got = ob.distances_all(qb, i, M, chunk=7)
        boxes = [ob.forward(b, M)[:2] for b in om.dnf(qb.tree(i))]
        for e in range(E.shape[0]):
            best = np.inf
            for c, o in boxes:
                tot = 0.0
                for j in range(E.shape[1]):
                    a = abs(E[e, j] - c[j])
                    tot += (a - o[j] if a > o[j] else 0.0) + 0.25 * min(a, o[j])
                best = min(best, tot)
            assert got[e] == pytest.approx(best, rel=1e-12)
        _, s = ob.query_step(qb.query_nodes(i), int(qb.pos[i]), negs[i], M, qb.B)
        np.testing.assert_allclose(12.0 - got[np.concatenate([[qb.pos[i]], negs[i]])], s, rtol=1e-13)


def _torch_loss(qb, negs, P, gamma, alpha):
    """Independent re-statement with torch ops + autograd (per query, fp64)."""
    def ev(t):
        if t[0] == "e":
            return P["E"][t[1]], torch.zeros_like(P["E"][0])
        if t[0] == "p":
            c, o = ev(t[2])
            return c + P["R"][t[1]], o + torch.relu(P["Ro"][t[1]])
        boxes = [ev(c) for c in t[1:]]
        cs = torch.stack([b[0] for b in boxes])
        os_ = torch.stack([b[1] for b in boxes])
        att = torch.relu(cs @ P["U1"].T + P["u1"]) @ P["U2"].T + P["u2"]
        hid = torch.relu(os_ @ P["V1"].T + P["c1"]).mean(0)          # mean of the hidden layer, then the linear layer
        gate = torch.sigmoid(P["V2"] @ hid + P["c2"])
        return (torch.softmax(att, 0) * cs).sum(0), os_.min(0).values * gate

    total = 0.0
    for i in range(qb.B):
        boxes = [ev(b) for b in om.dnf(qb.tree(i))]
        C = torch.stack([b[0] for b in boxes])
        O = torch.stack([b[1] for b in boxes])
        cand = torch.tensor(np.concatenate([[qb.pos[i]], negs[i]]), dtype=torch.long)
        a = (P["E"][cand][None] - C[:, None, :]).abs()
        dist = (torch.relu(a - O[:, None, :]).sum(-1) + alpha * torch.minimum(a, O[:, None, :]).sum(-1)).min(0).values
        s = gamma - dist
        total = total + (-torch.nn.functional.logsigmoid(s[0])
                         - torch.nn.functional.logsigmoid(-s[1:]).mean()) / (2 * qb.B)
    return total


@pytest.mark.parametrize("seed", [0, 1])
def test_loss_and_all_gradients_against_torch_autograd(seed):
    _, qb, negs, p = tiny(seed=seed, B=27, K=5)
    a = int(qb.arg[0])                                   # one entity as anchor, positive and negative
    qb.pos[3] = a
    negs[5, 2] = a
    negs[5, 3] = a
    M = ob.BoxModel(p, 12.0, 0.25)
    loss, G, _ = ob.batch_loss_and_grads(qb, negs, M)
    P = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in p.items()}
    tl = _torch_loss(qb, negs, P, 12.0, 0.25)
    tl.backward()
    assert loss == pytest.approx(float(tl.detach()), rel=1e-12)
    assert set(G.dense) == {"U1", "u1", "U2", "u2", "V1", "c1", "V2", "c2"}
    for k in G.dense:
        assert np.abs(G.dense[k]).max() > 0, k
        np.testing.assert_allclose(G.dense[k], P[k].grad.numpy(), rtol=1e-9, atol=1e-14, err_msg=k)
    for tname in ob.TABLES:
        np.testing.assert_allclose(G.table_dense(tname, p[tname].shape), P[tname].grad.numpy(),
                                   rtol=1e-9, atol=1e-14, err_msg=tname)
    rels = set(int(qb.arg[n]) for n in range(len(qb.op)) if qb.op[n] == om.OP_PROJ)
    assert set(G.rows["R"]) == rels == set(G.rows["Ro"])


def test_adam_first_step_moves_touched_rows_by_lr_and_leaves_the_rest():
    _, qb, negs, p = tiny(seed=2, B=10, K=3)
    P = om.to_f64(p)
    before = {k: v.copy() for k, v in P.items()}
    state = {k: [np.zeros_like(v), np.zeros_like(v)] for k, v in P.items()}
    _, G = ob.train_step(qb, negs, P, state, 1, HP)
    for table in ob.TABLES:
        touched = sorted(G.rows[table])
        rest = np.setdiff1d(np.arange(P[table].shape[0]), touched)
        assert np.array_equal(P[table][rest], before[table][rest])
        g = np.stack([G.rows[table][i] for i in touched])
        step = P[table][touched] - before[table][touched]
        big = np.abs(g) > 1e-5
        np.testing.assert_allclose(step[big], -HP["lr"] * np.sign(g[big]), rtol=1e-3)
        assert (state[table][0][rest] == 0).all()
    for k, g in G.dense.items():
        big = np.abs(g) > 1e-5
        np.testing.assert_allclose((P[k] - before[k])[big], -HP["lr"] * np.sign(g[big]), rtol=1e-3)
