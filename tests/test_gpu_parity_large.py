"""Parity at the full sizes of the larger workloads (needs an MI355X).

NELL shape: everything is compared, as for the benchmark workload.  wikikg2 shape
(2.5 M entities, 4096 queries x 1024 negatives): plan and index bit-exact in
full; values on sampled outputs the oracle computes one by one (queries: root
embeddings, all 1025 scores, loss term; entity rows: the gradient summed over
every query that touches the row); dense gradients and the loss through the
batch-split property; the optimiser on sampled rows."""
import numpy as np
import pytest

import workloads as wl
from oracle import model as om
from oracle import plan as oplan
from tests import parity as par

pytestmark = pytest.mark.gpu


def _say(msg):
    print("[case] " + msg, flush=True)


def test_nell_shape_full_size_multi_stream():
    _say("config 2 (N=63000, B=1024, K=128, d=400, 4 streams), forward_backward + 1 train step")
    case = par.Case.from_config(2)
    par.check_forward_backward(case, eng=case.engine(num_streams=4))
    par.check_train_steps(case, steps=1, num_streams=4)


def _anchor_owner(qb):
    """Query of every anchor, in the planner's anchor order (query, branch, post-order)."""
    owner = []
    for q in range(qb.B):
        def count(t):
            return 1 if t[0] == "e" else sum(count(c) for c in t[1:] if isinstance(c, tuple))
        owner.extend([q] * sum(count(b) for b in om.dnf(qb.tree(q))))
    return np.asarray(owner)


def test_wikikg2_shape_full_size_sampled():
    import torch
    cfg = wl.get_config(3)
    _say("config 3 (N=2.5M, B=4096, K=1024): building inputs")
    kg = wl.make_kg(cfg.N, cfg.R, cfg.T, cfg.alpha, cfg.seed)
    n_sample = 48
    rng = np.random.default_rng(5)
    params = wl.make_params(cfg.N, cfg.R, cfg.d, cfg.h, cfg.seed + 3)
    qb = wl.make_batch(kg, cfg.B, cfg.mix, cfg.seed + 1)
    negs = wl.make_negatives(cfg.N, cfg.B, cfg.K, cfg.seed + 2)
    M = om.Model(params, cfg.gamma)
    B, K, d = cfg.B, cfg.K, cfg.d

    from paper_2602_21597_amd import Engine
    eng = Engine(cfg.N, cfg.R, cfg.d, cfg.h, cfg.gamma)
    eng.bind_numpy(params)
    plan = eng.plan(qb)
    _say("plan + index, bit-exact")
    ref_plan = oplan.build_plan(qb)
    got_plan = plan.export()
    for k in ref_plan:
        assert np.array_equal(np.asarray(got_plan[k]), np.asarray(ref_plan[k])), "plan." + k
    neg_dev = torch.from_numpy(negs).cuda()
    loss = eng.forward_backward(plan, neg_dev)
    torch.cuda.synchronize()
    gv = eng.grad_view()
    u, off, src = oplan.entity_index(ref_plan, qb.pos, negs)
    U = gv.n_e_uniq
    assert U == len(u)
    from paper_2602_21597_amd.binding import copy_to_host
    assert np.array_equal(copy_to_host(gv.e_uniq, (U,), np.int32), u)
    assert np.array_equal(copy_to_host(gv.e_seg_off, (U + 1,), np.int32), off)
    assert np.array_equal(copy_to_host(gv.e_src, (gv.n_e_contrib,), np.int32), src)

    _say("sampled queries: embeddings, scores, loss terms")
    scores = copy_to_host(gv.pair_score, (B, K + 1), np.float32)
    terms = copy_to_host(gv.loss_terms, (B,), np.float32)
    for q in rng.choice(B, n_sample, replace=False):
        br = om.dnf(qb.tree(q))
        slots = ref_plan["root_slot"][ref_plan["root_off"][q]:ref_plan["root_off"][q + 1]]
        Y = np.stack([om.forward(b, M)[0] for b in br])
        got = eng.read_rows(gv.act, slots, d)
        par.assert_close(got, Y, "root embedding q%d" % q)
        cand = np.concatenate([[qb.pos[q]], negs[q]])
        s, _ = om.score(Y, M.entity(cand), M.gamma)
        par.assert_close(scores[q], s, "scores q%d" % q)
        want = om.pair_loss_terms(s[0], s[1:])
        assert abs(terms[q] - want) <= 1e-4 * abs(want)

    _say("sampled entity rows: gradient summed over every contributing query")
    owner = _anchor_owner(qb)
    nA = ref_plan["n_anchor"]
    assert len(owner) == nA

    def query_of(c):
        return owner[c] if c < nA else (c - nA if c < nA + B else (c - nA - B) // K)

    # rows with a positive or an anchor among their contributions carry the large gradients
    heavy = [i for i in range(U) if src[off[i]] < nA + B]
    pick = list(rng.choice(heavy, 12, replace=False)) + list(rng.choice(U, 12, replace=False))
    need = sorted(set(int(query_of(int(c))) for i in pick for c in src[off[i]:off[i + 1]]))
    G = om.Grads(M.P)
    for q in need:
        om.query_step(qb.query_nodes(q), int(qb.pos[q]), negs[q], M, B, G)
    got = eng.read_rows(gv.gE, pick, d)
    ref = np.stack([G.rows["E"][int(u[i])] for i in pick])
    par.assert_rows_close(got, ref, "sampled E gradient rows", tol=1e-3)
    par.assert_close(got[:12], ref[:12], "sampled heavy E gradient rows")

    _say("dense gradients and loss: the full batch equals the weighted sum of its quarters")
    full_loss = float(loss.cpu()[0])
    full = {n: copy_to_host(gv.g_mlp[i], shp, np.float32).astype(np.float64)
            for i, (n, shp) in enumerate(zip(par_names(), par_shapes(cfg)))}
    acc = {n: np.zeros_like(v) for n, v in full.items()}
    acc_loss = 0.0
    for c in range(4):
        idx = np.arange(c * B // 4, (c + 1) * B // 4)
        sub = qb.select(idx)
        sp = eng.plan(sub)
        sl = eng.forward_backward(sp, torch.from_numpy(np.ascontiguousarray(negs[idx])).cuda())
        torch.cuda.synchronize()
        sg = eng.grad_view()
        for i, (n, shp) in enumerate(zip(par_names(), par_shapes(cfg))):
            acc[n] += copy_to_host(sg.g_mlp[i], shp, np.float32) / 4.0
        acc_loss += float(sl.cpu()[0]) / 4.0
        sp.free()
    assert abs(full_loss - acc_loss) <= 1e-4 * abs(acc_loss)
    for n in full:
        if n != "u2":
            par.assert_close(full[n], acc[n], "split-sum " + n)

    _say("train step: sampled rows follow Adam on the step's own gradients, others untouched")
    touched = rng.choice(U, 64, replace=False)
    rows_t = u[touched]
    all_rows = np.zeros(cfg.N, bool)
    all_rows[u] = True
    untouched = rng.choice(np.flatnonzero(~all_rows), 64, replace=False)
    loss = eng.forward_backward(plan, neg_dev)
    torch.cuda.synchronize()
    gv = eng.grad_view()
    g_rows = eng.read_rows(gv.gE, touched, d).astype(np.float64)
    E, mE, vE = eng.tensors["E"]
    before = E[torch.from_numpy(rows_t).long().cuda()].cpu().numpy()
    before_u = E[torch.from_numpy(untouched).long().cuda()].cpu().numpy()
    eng.train_step(plan, neg_dev)
    torch.cuda.synchronize()
    after = E[torch.from_numpy(rows_t).long().cuda()].cpu().numpy()
    after_u = E[torch.from_numpy(untouched).long().cuda()].cpu().numpy()
    assert np.array_equal(before_u, after_u)
    wp, wm, wv = om.adam_update(before.astype(np.float64), 0.0, 0.0, g_rows, 1)
    ulp = np.spacing(np.abs(before)).astype(np.float64)
    assert np.all(np.abs(after - wp) <= 1e-4 * np.abs(wp - before).max() + ulp)
    m_after = mE[torch.from_numpy(rows_t).long().cuda()].cpu().numpy()
    par.assert_close(m_after, wm, "m rows")
    plan.free()


def par_names():
    from paper_2602_21597_amd import MLP_NAMES
    return MLP_NAMES


def par_shapes(cfg):
    return [(cfg.h, cfg.d), (cfg.h,), (cfg.d, cfg.h), (cfg.d,)] * 3
