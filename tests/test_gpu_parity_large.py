"""Parity at the full sizes of the larger workloads (needs an MI355X).

NELL shape: everything is compared, as for the benchmark workload.  wikikg2 shape
(2.5 M entities, 4096 queries x 1024 negatives) and text-feature shape (5 M
entities with 1024 bf16 features each): plan and index bit-exact in full;
values on sampled outputs the oracle computes one by one (queries: root
embeddings, all 1025 scores, loss term; entity rows: the gradient summed over
every query that touches the row); dense gradients and the loss through the
batch-split property (an extra, not the evidence); the optimiser on sampled rows.
Then the first 256 (wikikg2 shape) / 64 (text features) queries of the batch as a
batch of their own on the full tables: loss, every gradient (12 MLP tensors, E
rows, R rows, the text projection) and one optimiser step on every tensor with
its moments against the oracle.  With text features also the all-entity ranking
of 1024 queries, checked on 16 of them."""
import numpy as np
import pytest

import workloads as wl
from oracle import model as om
from oracle import plan as oplan
from tests import parity as par

pytestmark = pytest.mark.gpu


_say = par.say


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
    _full_size_sampled(wl.get_config(3), n_sample=48, n_sub=256)


def test_text_feature_shape_full_size_sampled():
    _full_size_sampled(wl.get_config(4), n_sample=16, n_sub=64)


def _compact(sub, sub_negs, params, sem_bits):
    """The sub-batch with its entities renumbered 0..n-1 in id order, and the rows of E (and of the
    text features) it reads.  A relabelling of inputs only: the oracle's result for compact row i is
    its result for entity used[i], and its fp64 copies then hold the rows in use instead of the
    whole table (8 bytes per element of millions of rows, three times over with the moments)."""
    import dataclasses
    anchors = sub.arg[sub.op == 0]
    used = np.unique(np.concatenate([anchors, sub.pos, sub_negs.ravel()])).astype(np.int64)
    remap = lambda x: np.searchsorted(used, x).astype(np.int32)
    arg = sub.arg.copy()
    arg[sub.op == 0] = remap(anchors)
    qc = dataclasses.replace(sub, arg=arg, pos=remap(sub.pos))
    pc = dict(params)
    pc["E"] = params["E"][used]
    return qc, remap(sub_negs), pc, (sem_bits[used] if sem_bits is not None else None), used


def _sub_batch_on_full_tables(cfg, eng, qb, negs, params, sem_bits, n_sub):
    """The first n_sub queries of the workload's batch as a batch of their own, on the full tables:
    loss, every gradient (MLP tensors, E rows, R rows, the text projection) and one optimiser step
    (both checks of parity.check_train_steps on every tensor, moments included) against the oracle."""
    import torch
    d = cfg.d
    hp = dict(lr=cfg.lr, beta1=cfg.beta1, beta2=cfg.beta2, eps=cfg.eps, gamma=cfg.gamma)
    _say("%d-query batch on the full tables: every gradient against the oracle" % n_sub)
    sub = qb.select(np.arange(n_sub))
    sub_negs = np.ascontiguousarray(negs[:n_sub])
    qc, negs_c, pc, sem_c, used = _compact(sub, sub_negs, params, sem_bits)
    eng.bind_numpy(params, sem_bits=sem_bits)          # fresh parameters and moments: earlier steps moved them
    sp = eng.plan(sub)
    nd = torch.from_numpy(sub_negs).cuda()
    sl = eng.forward_backward(sp, nd)
    torch.cuda.synchronize()
    g = eng.grads()
    pexp = sp.export()
    Mc = om.Model(pc, cfg.gamma, sem_c)
    ref_loss, G, _ = om.batch_loss_and_grads(qc, negs_c, Mc, track_sq=True)
    assert abs(float(sl.cpu()[0]) - ref_loss) <= 1e-4 * abs(ref_loss)
    floor = par.dense_gradient_floor(G.dense)
    for name in G.dense:
        if name == "u2":
            par.assert_zero_gradient(g[name], G.dense)
        else:
            par.assert_close(g[name], G.dense[name], "grad " + name, par.tol_of(name, par.TOL), floor)
    e_uniq = g["e_uniq"].astype(np.int64)
    assert np.array_equal(used[sorted(G.rows["E"])], e_uniq)
    comp = np.searchsorted(used, e_uniq)               # compact number of every touched row
    ref_rows = np.stack([G.rows["E"][int(c)] for c in comp])
    par.assert_close(g["gE"], ref_rows, "grad E")
    r_uniq = pexp["r_uniq"]
    assert sorted(G.rows["R"]) == list(r_uniq)
    ref_R = np.stack([G.rows["R"][int(r)] for r in r_uniq])
    par.assert_close(g["gR"], ref_R, "grad R")
    par.assert_rows_close(g["gR"], ref_R, "grad rows R")
    # row by row, except rows of candidates that sit on an |.| kink of a query (some coordinate of
    # the winning branch within fp32 rounding of the candidate's: either sign is a correct answer;
    # this batch is not redrawn clear of kinks as the small cases are)
    on_kink = set()
    for q in range(n_sub):
        Y = np.stack([om.forward(b, Mc)[0] for b in om.dnf(qc.tree(q))])
        cand = np.concatenate([[qc.pos[q]], negs_c[q]])
        rows = Mc.entity(cand)
        win = np.abs(Y[:, None, :] - rows[None]).sum(axis=2).argmin(axis=0)
        margin = np.abs(Y[win] - rows).min(axis=1)
        on_kink.update(int(e) for e in cand[margin < par.TAU_ABS])
    clear = np.array([int(c) not in on_kink for c in comp])
    _say("  %d of %d touched rows hold a candidate on an |.| kink (left out of the row-wise checks)" % (
        int((~clear).sum()), len(clear)))
    assert clear.sum() >= 0.99 * len(clear)
    par.assert_rows_close(g["gE"][clear], ref_rows[clear], "grad rows E")

    _say("  one optimiser step of that batch: every tensor, moments included")
    idx_dev = torch.from_numpy(e_uniq).cuda()
    read = lambda name, k, rows=None: (eng.tensors[name][k] if rows is None else eng.tensors[name][k][rows]).cpu().numpy()
    names = list(G.dense) + ["E", "R"]
    rows_of = {"E": idx_dev, "R": torch.from_numpy(r_uniq.astype(np.int64)).cuda()}
    before = {n: tuple(read(n, k, rows_of.get(n)) for k in range(3)) for n in names}
    E_before = eng.tensors["E"][0].clone()
    R_before = eng.tensors["R"][0].clone()
    loss = eng.train_step(sp, nd)
    torch.cuda.synchronize()
    assert abs(float(loss.cpu()[0]) - ref_loss) <= 1e-4 * abs(ref_loss)
    after = {n: tuple(read(n, k, rows_of.get(n)) for k in range(3)) for n in names}
    for tab, bef, ids in (("E", E_before, idx_dev), ("R", R_before, rows_of["R"])):
        same = torch.ones(bef.shape[0], dtype=torch.bool, device=bef.device)
        same[ids] = False
        assert torch.equal(eng.tensors[tab][0][same], bef[same]), tab + ": untouched rows moved"
        assert not bool(eng.tensors[tab][1][same].any()) and not bool(eng.tensors[tab][2][same].any())
    del E_before, R_before
    P = om.to_f64(pc)
    state = om.new_state(P)
    P0 = {k: v.copy() for k, v in P.items()}
    om.adam_step(P, state, G, 1, hp)
    kept = {}
    for name in names:
        table = name in ("E", "R")
        if table:
            sel = comp if name == "E" else r_uniq
            own = g["g" + name].astype(np.float64)
            gref = ref_rows if name == "E" else ref_R
            mass = np.array([G.mass[name][int(c)] for c in sel])[:, None]
            delta = par.gradient_noise(name) * mass
            cancels, exclude = False, (~clear[:, None] if name == "E" else None)
        else:
            sel = slice(None)
            own = g[name].astype(np.float64)
            gref = G.dense[name]
            rms = np.sqrt(G.dense_sq[name])
            delta = par.gradient_noise(name) * np.maximum(rms, np.abs(gref).max() * 1e-3)
            cancels, exclude = np.abs(gref).max() < 0.05 * rms.max(), None
        zeros = np.zeros_like(P0[name][sel])
        res = par.check_update(name, 1, hp, before[name], after[name], own, (P0[name][sel], zeros, zeros),
                               (P[name][sel], state[name][0][sel], state[name][1][sel]), gref, delta,
                               cancels=cancels, dense_floor=None if table else floor, exclude=exclude)
        if res is not None:
            kept[name] = res
    par.report_kept(kept, "config %d, %d queries" % (cfg.index, n_sub))
    sp.free()


def _full_size_sampled(cfg, n_sample, n_sub):
    import torch
    _say("config %d (N=%d, B=%d, K=%d, d_sem=%d): building inputs" % (cfg.index, cfg.N, cfg.B, cfg.K, cfg.d_sem))
    kg = wl.make_kg(cfg.N, cfg.R, cfg.T, cfg.alpha, cfg.seed)
    rng = np.random.default_rng(5)
    params = wl.make_params(cfg.N, cfg.R, cfg.d, cfg.h, cfg.seed + 3, d_sem=cfg.d_sem)
    sem_bits = wl.make_sem_features(cfg.N, cfg.d_sem, cfg.seed + 5) if cfg.d_sem else None
    qb = wl.make_batch(kg, cfg.B, cfg.mix, cfg.seed + 1)
    negs = wl.make_negatives(cfg.N, cfg.B, cfg.K, cfg.seed + 2)
    M = om.Model(params, cfg.gamma, sem_bits)
    B, K, d = cfg.B, cfg.K, cfg.d

    from paper_2602_21597_amd import Engine
    eng = Engine(cfg.N, cfg.R, cfg.d, cfg.h, cfg.gamma, d_sem=cfg.d_sem, num_streams=cfg.streams)
    eng.bind_numpy(params, sem_bits=sem_bits)
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
    # (rows of at most 16 contributions keep the number of queries the oracle has to run small);
    # then hub rows: the shortest four of the segments with more than 64 contributions (more than one
    # round of the table kernel's record loop; every contributing query is run by the oracle)
    seg_len = np.diff(off)
    small = np.flatnonzero(seg_len <= 16)
    heavy = [int(i) for i in small if src[off[i]] < nA + B]
    pick = list(rng.choice(heavy, 12, replace=False)) + list(rng.choice(small, 12, replace=False))
    hubs = np.flatnonzero(seg_len > 64)
    hubs = [int(i) for i in hubs[np.argsort(seg_len[hubs], kind="stable")[:4]]]
    _say("  segment lengths: max %d, %d above 64; hub rows checked: %s" % (
        seg_len.max(), int((seg_len > 64).sum()), [int(seg_len[i]) for i in hubs]))
    pick += hubs
    need = sorted(set(int(query_of(int(c))) for i in pick for c in src[off[i]:off[i + 1]]))
    G = om.Grads(M.P)
    for q in need:
        om.query_step(qb.query_nodes(q), int(qb.pos[q]), negs[q], M, B, G)
    got = eng.read_rows(gv.gE, pick, d)
    ref = np.stack([G.rows["E"][int(u[i])] for i in pick])
    par.assert_rows_close(got, ref, "sampled E gradient rows", tol=1e-3)
    par.assert_close(got[:12], ref[:12], "sampled heavy E gradient rows")
    if hubs:
        par.assert_close(got[24:], ref[24:], "sampled hub E gradient rows")

    _say("dense gradients and loss: the full batch equals the weighted sum of its quarters")
    full_loss = float(loss.cpu()[0])
    full = {n: copy_to_host(gv.g_mlp[i], shp, np.float32).astype(np.float64)
            for i, (n, shp) in enumerate(zip(par_names(), par_shapes(cfg)))}
    if cfg.d_sem:
        full["Wp"] = copy_to_host(gv.g_Wp, (d, cfg.d_sem), np.float32).astype(np.float64)
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
        if cfg.d_sem:
            acc["Wp"] += copy_to_host(sg.g_Wp, (d, cfg.d_sem), np.float32) / 4.0
        acc_loss += float(sl.cpu()[0]) / 4.0
        sp.free()
    assert abs(full_loss - acc_loss) <= 1e-4 * abs(acc_loss)
    for n in full:
        if n != "u2":
            par.assert_close(full[n], acc[n], "split-sum " + n, par.tol_of(n, par.TOL))

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

    _sub_batch_on_full_tables(cfg, eng, qb, negs, params, sem_bits, n_sub)
    if not cfg.d_sem:
        return

    _say("ranking: 1024 queries against all entities, top-10; 16 queries checked")
    eng.bind_numpy(params, sem_bits=sem_bits)          # the parameters the oracle holds: the step above moved them
    from oracle import rank as orank
    rq = wl.make_batch(kg, 1024, cfg.mix, cfg.seed + 7)
    rp = eng.plan(rq)
    ids, dist = eng.rank_all(rp, 10)
    torch.cuda.synchronize()
    ids, dist = ids.cpu().numpy(), dist.cpu().numpy()
    assert np.all(np.diff(dist, axis=1) >= 0)
    check = rng.choice(1024, 16, replace=False)
    Y = [orank.query_embeddings(rq, int(q), M) for q in check]
    full_d = np.empty((16, cfg.N), np.float64)
    chunk = 1 << 15
    for lo in range(0, cfg.N, chunk):
        e = np.arange(lo, min(cfg.N, lo + chunk))
        rows = M.entity(e)                               # fused rows of the chunk, once for all 16 queries
        for j in range(16):
            full_d[j, lo:lo + len(e)] = np.abs(Y[j][:, None, :] - rows[None]).sum(axis=2).min(axis=0)
        if (lo // chunk) % 32 == 0:
            _say("  oracle distances: %d of %d entities" % (lo, cfg.N))
    for j, q in enumerate(check):
        order = np.lexsort((np.arange(cfg.N), full_d[j]))[:10]
        ref_d = full_d[j][order]
        par.assert_close(dist[q], ref_d, "top-10 distances q%d" % q)
        assert len(set(ids[q])) == 10 and ids[q].min() >= 0 and ids[q].max() < cfg.N
        assert np.all(full_d[j][ids[q]] <= ref_d[-1] * (1 + 1e-4)), "q%d" % q
        par.assert_close(dist[q], full_d[j][ids[q]], "returned distances belong to returned ids q%d" % q)
    rp.free()


def par_names():
    from paper_2602_21597_amd import MLP_NAMES
    return MLP_NAMES


def par_shapes(cfg):
    return [(cfg.h, cfg.d), (cfg.h,), (cfg.d, cfg.h), (cfg.d,)] * 3
