"""Pins of the CPU oracle against things that are not the oracle: closed forms,
invariants, finite differences, torch autograd / torch optimisers, brute force.
All CPU, all small."""
import math

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import model as om
from oracle import rank as orank

HP = dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, gamma=12.0)


def tiny(seed=0, N=50, R=6, d=8, h=16, B=10, K=4, T=400, mix=None, d_sem=0):
    kg = wl.make_kg(N, R, T, 2.1, seed)
    mix = mix or {n: 1.0 for n in wl.configs.ALL14}
    qb = wl.make_batch(kg, B, mix, seed + 1)
    negs = wl.make_negatives(N, B, K, seed + 2)
    params = wl.make_params(N, R, d, h, seed + 3, d_sem=d_sem)
    sem = wl.make_sem_features(N, d_sem, seed + 4) if d_sem else None
    return kg, qb, negs, params, sem


# ---------------------------------------------------------------- operators
def test_1p_closed_form():
    """1p reduces to one projection: s = gamma - ||W2 relu(W1 (E[a]+R[r]) + b1) + b2 - E[t]||_1."""
    _, _, _, p, _ = tiny(d=6, h=5)
    a, r, t = 3, 2, 7
    qb = wl.batch_from_trees([("p", r, ("e", a))], [t])
    M = om.Model(p, 12.0)
    _, s = om.query_step(qb.query_nodes(0), t, [11, 12], M, 1)
    P = {k: v.astype(np.float64) for k, v in p.items()}
    d, h = 6, 5
    z = [P["E"][a][k] + P["R"][r][k] for k in range(d)]
    hid = [max(0.0, sum(P["W1"][j][k] * z[k] for k in range(d)) + P["b1"][j]) for j in range(h)]
    y = [sum(P["W2"][k][j] * hid[j] for j in range(h)) + P["b2"][k] for k in range(d)]
    for idx, e in enumerate((t, 11, 12)):
        want = 12.0 - sum(abs(y[k] - P["E"][e][k]) for k in range(d))
        assert s[idx] == pytest.approx(want, rel=1e-13, abs=1e-13)


def test_intersection_of_identical_inputs_is_the_input():
    _, _, _, p, _ = tiny()
    M = om.Model(p, 12.0)
    child = ("p", 1, ("e", 4))
    y_child, _ = om.forward(child, M)
    for k in (2, 3, 4):
        y, tape = om.forward(("i",) + (child,) * k, M)
        np.testing.assert_allclose(y, y_child, rtol=1e-14, atol=1e-15)
        np.testing.assert_allclose(tape[4].sum(axis=0), 1.0, rtol=1e-14)


def test_intersection_permutation_invariant_and_convex():
    _, _, _, p, _ = tiny()
    M = om.Model(p, 12.0)
    kids = [("p", 1, ("e", 4)), ("p", 0, ("e", 9)), ("n", ("p", 3, ("e", 2)))]
    y0, tape = om.forward(("i",) + tuple(kids), M)
    y1, _ = om.forward(("i", kids[2], kids[0], kids[1]), M)
    np.testing.assert_allclose(y0, y1, rtol=1e-13, atol=1e-15)
    X, W = tape[3], tape[4]
    np.testing.assert_allclose(W.sum(axis=0), 1.0, rtol=1e-14)
    assert np.all(y0 <= X.max(axis=0) + 1e-15) and np.all(y0 >= X.min(axis=0) - 1e-15)


def test_intersection_attention_against_torch_softmax():
    _, _, _, p, _ = tiny()
    M = om.Model(p, 12.0)
    kids = [("p", 1, ("e", 4)), ("p", 0, ("e", 9)), ("p", 5, ("e", 30))]
    y, _ = om.forward(("i",) + tuple(kids), M)
    P = {k: torch.tensor(v, dtype=torch.float64) for k, v in p.items()}
    xs = torch.stack([torch.tensor(om.forward(k, M)[0]) for k in kids])
    att = torch.relu(xs @ P["U1"].T + P["u1"]) @ P["U2"].T + P["u2"]
    want = (torch.softmax(att, dim=0) * xs).sum(0)
    np.testing.assert_allclose(y, want.numpy(), rtol=1e-12, atol=1e-14)


def test_union_dnf_shapes():
    up = ("p", 7, ("u", ("p", 1, ("e", 2)), ("p", 3, ("e", 4))))
    assert om.dnf(up) == [("p", 7, ("p", 1, ("e", 2))), ("p", 7, ("p", 3, ("e", 4)))]
    two_u = ("u", ("p", 1, ("e", 2)), ("p", 3, ("e", 4)))
    assert om.dnf(two_u) == [("p", 1, ("e", 2)), ("p", 3, ("e", 4))]
    with pytest.raises(om.Unsupported):
        om.dnf(("i", two_u, ("p", 1, ("e", 2))))
    with pytest.raises(om.Unsupported):
        om.dnf(("n", two_u))


def test_union_of_identical_branches_equals_1p_and_max_of_branch_scores():
    _, _, _, p, _ = tiny()
    M = om.Model(p, 12.0)
    one = wl.batch_from_trees([("p", 1, ("e", 4))], [5])
    two = wl.batch_from_trees([("u", ("p", 1, ("e", 4)), ("p", 1, ("e", 4)))], [5])
    negs = np.array([[1, 2, 3]])
    l1, g1, s1 = om.batch_loss_and_grads(one, negs, M)
    l2, g2, s2 = om.batch_loss_and_grads(two, negs, M)
    assert l1 == pytest.approx(l2, rel=1e-14)
    np.testing.assert_allclose(g1.dense["W1"], g2.dense["W1"], rtol=1e-13, atol=1e-18)
    # distinct branches: score is the max of the two 1p scores
    a = wl.batch_from_trees([("p", 1, ("e", 4))], [5])
    b = wl.batch_from_trees([("p", 2, ("e", 8))], [5])
    u = wl.batch_from_trees([("u", ("p", 1, ("e", 4)), ("p", 2, ("e", 8)))], [5])
    sa = om.batch_loss_and_grads(a, negs, M, False)[2][0]
    sb = om.batch_loss_and_grads(b, negs, M, False)[2][0]
    su = om.batch_loss_and_grads(u, negs, M, False)[2][0]
    np.testing.assert_allclose(su, np.maximum(sa, sb), rtol=1e-14)


def test_score_is_gamma_when_entity_equals_query_embedding():
    _, _, _, p, _ = tiny()
    M = om.Model(p, 12.0)
    y, _ = om.forward(("p", 1, ("e", 4)), M)
    M.P["E"][17] = y
    s, win = om.score(y[None], M.entity(np.array([17, 3])), 12.0)
    assert s[0] == 12.0 and s[1] < 12.0


# --------------------------------------------------------------------- loss
def test_loss_is_ln2_when_all_scores_are_zero():
    assert om.pair_loss_terms(0.0, np.zeros(7)) / 2.0 == pytest.approx(math.log(2.0), rel=1e-15)


def test_loss_against_torch_logsigmoid():
    rng = np.random.default_rng(0)
    sp, sn = rng.normal() * 5, rng.normal(size=9) * 5
    want = -torch.nn.functional.logsigmoid(torch.tensor(sp, dtype=torch.float64)) \
        - torch.nn.functional.logsigmoid(-torch.tensor(sn, dtype=torch.float64)).mean()
    assert om.pair_loss_terms(sp, sn) == pytest.approx(float(want), rel=1e-13)
    # stable far out in the tails
    assert om.pair_loss_terms(-800.0, np.array([800.0])) == pytest.approx(1600.0, rel=1e-15)
    assert om.pair_loss_terms(800.0, np.array([-800.0])) == pytest.approx(0.0, abs=1e-300)


def test_repeated_negatives_and_repeated_queries():
    _, qb, negs, p, _ = tiny(B=6)
    M = om.Model(p, 12.0)
    one = qb.select([2])
    l1, g1, _ = om.batch_loss_and_grads(one, negs[2:3, :1], M)
    lk, gk, _ = om.batch_loss_and_grads(one, np.repeat(negs[2:3, :1], 5, axis=1), M)
    assert l1 == pytest.approx(lk, rel=1e-13)
    np.testing.assert_allclose(g1.dense["W2"], gk.dense["W2"], rtol=1e-12, atol=1e-18)
    many = qb.select([2, 2, 2])
    lb, gb, _ = om.batch_loss_and_grads(many, np.repeat(negs[2:3, :1], 3, axis=0), M)
    assert l1 == pytest.approx(lb, rel=1e-13)
    np.testing.assert_allclose(g1.table_dense("E", p["E"].shape), gb.table_dense("E", p["E"].shape),
                               rtol=1e-12, atol=1e-18)


def test_split_and_permutation_invariance():
    _, qb, negs, p, _ = tiny(B=12)
    M = om.Model(p, 12.0)
    l, g, _ = om.batch_loss_and_grads(qb, negs, M)
    perm = np.random.default_rng(5).permutation(12)
    lp, gp, _ = om.batch_loss_and_grads(qb.select(perm), negs[perm], M)
    assert l == pytest.approx(lp, rel=1e-13)
    np.testing.assert_allclose(g.dense["U1"], gp.dense["U1"], rtol=1e-10, atol=1e-16)
    la, ga, _ = om.batch_loss_and_grads(qb.select(range(6)), negs[:6], M)
    lb, gb, _ = om.batch_loss_and_grads(qb.select(range(6, 12)), negs[6:], M)
    assert l == pytest.approx((la + lb) / 2, rel=1e-13)
    for k in g.dense:
        np.testing.assert_allclose(g.dense[k], (ga.dense[k] + gb.dense[k]) / 2, rtol=1e-10, atol=1e-16)
    sh = p["E"].shape
    np.testing.assert_allclose(g.table_dense("E", sh),
                               (ga.table_dense("E", sh) + gb.table_dense("E", sh)) / 2,
                               rtol=1e-10, atol=1e-16)


# ---------------------------------------------------------------- gradients
def _torch_loss(qb, negs, P, gamma, sem=None, cand_rows=None):
    """Independent re-statement with torch ops + autograd (per query, fp64)."""
    def ent(e):
        row = P["E"][e]
        if sem is not None:
            row = row + sem[e] @ P["Wp_used"].T
        return row

    def ev(t):
        if t[0] == "e":
            return ent(t[1])
        if t[0] == "p":
            z = ev(t[2]) + P["R"][t[1]]
            return P["W2"] @ torch.relu(P["W1"] @ z + P["b1"]) + P["b2"]
        if t[0] == "n":
            return P["V2"] @ torch.relu(P["V1"] @ ev(t[1]) + P["c1"]) + P["c2"]
        xs = torch.stack([ev(c) for c in t[1:]])
        att = torch.relu(xs @ P["U1"].T + P["u1"]) @ P["U2"].T + P["u2"]
        return (torch.softmax(att, 0) * xs).sum(0)

    total = 0.0
    for i in range(qb.B):
        Y = torch.stack([ev(b) for b in om.dnf(qb.tree(i))])
        cand = torch.tensor(np.concatenate([[qb.pos[i]], negs[i]]), dtype=torch.long)
        rows = cand_rows[cand] if cand_rows is not None else ent(cand)
        dist = (Y[:, None, :] - rows[None]).abs().sum(-1).min(0).values
        s = gamma - dist
        total = total + (-torch.nn.functional.logsigmoid(s[0])
                         - torch.nn.functional.logsigmoid(-s[1:]).mean()) / (2 * qb.B)
    return total


@pytest.mark.parametrize("seed", [0, 1])
def test_loss_and_all_gradients_against_torch_autograd(seed):
    _, qb, negs, p, _ = tiny(seed=seed, B=28, K=5)
    # one entity that is anchor, positive and negative in the same batch
    a = int(qb.arg[0])
    qb.pos[3] = a
    negs[5, 2] = a
    negs[5, 3] = a
    M = om.Model(p, 12.0)
    loss, G, _ = om.batch_loss_and_grads(qb, negs, M)
    P = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in p.items()}
    tl = _torch_loss(qb, negs, P, 12.0)
    tl.backward()
    assert loss == pytest.approx(float(tl), rel=1e-12)
    for k in om.Grads(M.P).dense:
        np.testing.assert_allclose(G.dense[k], P[k].grad.numpy(), rtol=1e-9, atol=1e-14, err_msg=k)
    for tname in ("E", "R"):
        np.testing.assert_allclose(G.table_dense(tname, p[tname].shape), P[tname].grad.numpy(),
                                   rtol=1e-9, atol=1e-14, err_msg=tname)
    # touched rows are exactly the rows that occur as anchor / positive / negative / relation
    ents = set(int(x) for x in negs.reshape(-1)) | set(int(x) for x in qb.pos) \
        | set(int(qb.arg[n]) for n in range(len(qb.op)) if qb.op[n] == 0)
    assert set(G.rows["E"]) == ents


def test_semantic_fuse_gradients_against_torch_autograd():
    _, qb, negs, p, sem = tiny(seed=3, B=10, K=4, d_sem=12)
    M = om.Model(p, 12.0, sem)
    loss, G, _ = om.batch_loss_and_grads(qb, negs, M)
    P = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in p.items()}
    wp_used = torch.tensor(p["Wp"]).bfloat16().double()
    # straight-through: the bf16 copy is what is used, its gradient is the master's
    P["Wp_used"] = (wp_used - P["Wp"]).detach() + P["Wp"]
    semt = torch.tensor((sem.astype(np.uint32) << 16).view(np.float32).astype(np.float64))
    tl = _torch_loss(qb, negs, P, 12.0, semt)
    tl.backward()
    assert loss == pytest.approx(float(tl), rel=1e-12)
    np.testing.assert_allclose(G.dense["Wp"], P["Wp"].grad.numpy(), rtol=1e-9, atol=1e-14)
    np.testing.assert_allclose(G.table_dense("E", p["E"].shape), P["E"].grad.numpy(), rtol=1e-9, atol=1e-14)


def test_bf16_candidate_rows_against_torch():
    """Scoring from a bf16 copy of E: the rounding is torch's; positives and negatives use the
    rounded rows, anchors the exact ones, and the gradient of a rounded row goes to E unchanged."""
    _, qb, negs, p, _ = tiny(seed=6, B=20, K=5)
    a = int(qb.arg[0])                 # an entity that is anchor and negative
    negs[2, 1] = a
    M = om.Model(p, 12.0, score_bf16=True)
    E32 = torch.tensor(p["E"])
    assert np.array_equal(M.candidate(np.arange(p["E"].shape[0])), E32.bfloat16().double().numpy())
    assert not np.array_equal(M.candidate(3), M.entity(3))
    loss, G, _ = om.batch_loss_and_grads(qb, negs, M)
    P = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in p.items()}
    rounded = (E32.bfloat16().double() - P["E"]).detach() + P["E"]          # straight-through
    tl = _torch_loss(qb, negs, P, 12.0, cand_rows=rounded)
    tl.backward()
    assert loss == pytest.approx(float(tl.detach()), rel=1e-12)
    exact_loss = om.batch_loss_and_grads(qb, negs, om.Model(p, 12.0), want_grads=False)[0]
    assert abs(loss - exact_loss) > 1e-7 * abs(exact_loss)                   # the rounding is visible
    for k in G.dense:
        np.testing.assert_allclose(G.dense[k], P[k].grad.numpy(), rtol=1e-9, atol=1e-14, err_msg=k)
    for tname in ("E", "R"):
        np.testing.assert_allclose(G.table_dense(tname, p[tname].shape), P[tname].grad.numpy(),
                                   rtol=1e-9, atol=1e-14, err_msg=tname)
    # ranking reads the same rows
    full = orank.distances_all(qb, 0, M)
    s = orank.score_candidates(qb, negs, M)
    np.testing.assert_allclose(12.0 - full[negs[0]], s[0], rtol=1e-13)


def test_finite_differences_every_tensor():
    _, qb, negs, p, _ = tiny(seed=4, N=50, d=8, h=16, B=10, K=4)
    M = om.Model(p, 12.0)
    _, G, _ = om.batch_loss_and_grads(qb, negs, M)
    dense = dict(G.dense)
    dense["E"] = G.table_dense("E", p["E"].shape)
    dense["R"] = G.table_dense("R", p["R"].shape)
    rng = np.random.default_rng(0)
    eps = 1e-6
    checked = 0
    for name, g in dense.items():
        flat = M.P[name].reshape(-1)
        nz = np.flatnonzero(g.reshape(-1))
        pick = rng.choice(nz, size=min(6, len(nz)), replace=False) if len(nz) else []
        for j in pick:
            old = flat[j]
            flat[j] = old + eps
            lp = om.batch_loss_and_grads(qb, negs, M, False)[0]
            flat[j] = old - eps
            lm = om.batch_loss_and_grads(qb, negs, M, False)[0]
            flat[j] = old
            fd = (lp - lm) / (2 * eps)
            # a kink (relu / abs / min) inside the +-eps interval shows as a large
            # mismatch; those coordinates are skipped, the others must agree
            if abs(fd - g.reshape(-1)[j]) <= 1e-6 * max(1e-3, abs(fd)):
                checked += 1
    assert checked >= 0.8 * 6 * len(dense)


# --------------------------------------------------------------------- Adam
def test_adam_first_step_closed_form_and_untouched_rows():
    _, qb, negs, p, _ = tiny(seed=6, N=200, B=6, K=3)
    P = om.to_f64(p)
    before = {k: v.copy() for k, v in P.items()}
    st = om.new_state(P)
    _, G = om.train_step(qb, negs, P, st, 1, HP)
    g = G.dense["W1"]
    np.testing.assert_allclose(P["W1"] - before["W1"], -1e-4 * g / (np.abs(g) + 1e-8), rtol=1e-9, atol=1e-18)
    touched = sorted(G.rows["E"])
    mask = np.ones(200, bool)
    mask[touched] = False
    assert mask.sum() > 0
    assert np.array_equal(P["E"][mask], before["E"][mask])
    assert np.all(st["E"][0][mask] == 0) and np.all(st["E"][1][mask] == 0)
    gE = G.table_dense("E", p["E"].shape)[touched]
    np.testing.assert_allclose(P["E"][touched] - before["E"][touched],
                               -1e-4 * gE / (np.abs(gE) + 1e-8), rtol=1e-9, atol=1e-18)


def test_adam_three_steps_against_torch_optimisers():
    """Dense tensors against torch.optim.Adam, tables against torch.optim.SparseAdam
    (the lazy, row-wise variant with the global step in the bias correction), fed
    with the oracle's own gradients.  SparseAdam adds eps before the bias
    correction of v, so gradients are scaled up until eps is immaterial."""
    _, qb, _, p, _ = tiny(seed=7, N=120, B=8, K=3)
    P = om.to_f64(p)
    st = om.new_state(P)
    tW = torch.tensor(p["W2"], dtype=torch.float64, requires_grad=True)
    tE = torch.tensor(p["E"], dtype=torch.float64, requires_grad=True)
    optW = torch.optim.Adam([tW], lr=1e-2, betas=(0.9, 0.999), eps=1e-8)
    optE = torch.optim.SparseAdam([tE], lr=1e-2, betas=(0.9, 0.999), eps=1e-8)
    hp = dict(HP, lr=1e-2)
    touched_sets = []
    for t in (1, 2, 3):
        negs = wl.make_negatives(120, 8, 3, 100 + t)
        M = om.Model(P, 12.0)
        M.P = P
        _, G, _ = om.batch_loss_and_grads(qb, negs, M)
        for k in G.dense:
            G.dense[k] *= 1e8
        for tab in ("E", "R"):
            for r in G.rows[tab]:
                G.rows[tab][r] *= 1e8
        om.adam_step(P, st, G, t, hp)
        tW.grad = torch.tensor(G.dense["W2"])
        optW.step()
        rows = sorted(G.rows["E"])
        touched_sets.append(set(rows))
        vals = np.stack([G.rows["E"][r] for r in rows])
        tE.grad = torch.sparse_coo_tensor(torch.tensor([rows]), torch.tensor(vals), tE.shape)
        optE.step()
        np.testing.assert_allclose(P["W2"], tW.detach().numpy(), rtol=1e-10, atol=1e-14)
        np.testing.assert_allclose(P["E"] - p["E"], tE.detach().numpy() - p["E"], rtol=1e-5, atol=1e-12)
    # the check is only meaningful if some row was skipped in a later step
    assert touched_sets[0] - touched_sets[1] and touched_sets[1] - touched_sets[0]


def test_adam_second_step_by_hand():
    p0, g1, g2 = 0.3, 0.5, -0.2
    p, m, v = om.adam_update(np.array(p0), np.array(0.0), np.array(0.0), np.array(g1), 1)
    p, m, v = om.adam_update(p, m, v, np.array(g2), 2)
    m2 = 0.9 * (0.1 * g1) + 0.1 * g2
    v2 = 0.999 * (0.001 * g1 * g1) + 0.001 * g2 * g2
    step1 = 1e-4 * g1 / (abs(g1) + 1e-8)
    want = p0 - step1 - 1e-4 * (m2 / (1 - 0.81)) / (math.sqrt(v2 / (1 - 0.999 ** 2)) + 1e-8)
    assert float(p) == pytest.approx(want, rel=1e-14)


# ------------------------------------------------------------------ ranking
def test_topk_against_python_sort_and_candidate_scores():
    _, qb, _, p, _ = tiny(seed=8, N=300, B=4)
    M = om.Model(p, 12.0)
    for i in range(4):
        ids, dist = orank.topk_all(qb, i, M, 10)
        full = orank.distances_all(qb, i, M, chunk=64)
        want = sorted(range(300), key=lambda e: (full[e], e))[:10]
        assert list(ids) == want
        assert np.all(np.diff(dist) >= 0)
        sc = orank.score_candidates(qb.select([i]), ids[None], M)
        np.testing.assert_allclose(sc[0], 12.0 - dist, rtol=1e-14)
        # same numbers as the training-time score of the same pairs
        _, s = om.query_step(qb.query_nodes(i), int(ids[0]), ids[1:], M, 1)
        np.testing.assert_allclose(s, sc[0], rtol=1e-14)


# ---------------------------------------------------------------- filtered ranks, MRR, Hit@k
def test_filtered_ranks_against_python_loops_and_special_cases():
    from oracle import rank as orank
    _, qb, _, p, _ = tiny(seed=9, N=60, B=12, K=1, mix={"2u": 1.0, "2i": 1.0, "1p": 1.0})
    M = om.Model(p, 12.0)
    rng = np.random.default_rng(3)
    for q in range(qb.B):
        dist = orank.distances_all(qb, q, M)
        answers = [int(a) for a in rng.choice(60, 1 + q % 5, replace=False)]
        ranks, d_ans = orank.filtered_ranks(qb, q, answers, M)
        for a, r, da in zip(answers, ranks, d_ans):
            want = 1
            for e in range(60):                       # the definition, entity by entity
                if e not in answers and dist[e] < dist[a]:
                    want += 1
            assert r == want and da == dist[a]
        # the nearest entity alone has rank 1; so has anything once every entity is filtered
        order = np.argsort(dist, kind="stable")
        assert orank.filtered_ranks(qb, q, [int(order[0])], M)[0][0] == 1
        assert np.all(orank.filtered_ranks(qb, q, list(range(60)), M)[0] == 1)
        # unfiltered (single answer): rank = position in the full sort
        for pos in (0, 7, 59):
            assert orank.filtered_ranks(qb, q, [int(order[pos])], M)[0][0] == pos + 1
        # filtering the k nearest entities lifts the (k+1)-th to rank 1
        assert orank.filtered_ranks(qb, q, [int(e) for e in order[:6]], M)[0][5] == 1


def test_ranking_metrics_closed_forms():
    from oracle import rank as orank
    m = orank.ranking_metrics([[1, 2, 4]])
    assert m[0] == pytest.approx((1 + 0.5 + 0.25) / 3) and list(m[1:]) == [pytest.approx(1 / 3), pytest.approx(2 / 3), 1.0]
    # per query first, then over queries: not the pooled mean
    m = orank.ranking_metrics([[1], [10, 100, 1000], []])
    assert m[0] == pytest.approx((1.0 + (0.1 + 0.01 + 0.001) / 3) / 2)
    assert m[3] == pytest.approx((1.0 + 1 / 3) / 2) and m[1] == pytest.approx(0.5)
    assert np.all(orank.ranking_metrics([[], []]) == 0)
