"""Helpers of the GPU parity tests of the box family: the same plan, the same tolerances and
the same comparisons as tests/parity.py, against oracle.box.

Kinks the seeded inputs keep clear of (fp32 rounding decides the side there and the model
does not say which one is right): hidden units of either MLP at 0, a candidate coordinate
with |e - c| at 0 or at the offset (inside/outside), near-equal smallest offsets of an
intersection's inputs, near-equal distances of two union branches.
"""
import numpy as np

import workloads as wl
from oracle import box as ob
from oracle import model as om
from oracle import plan as oplan

from .parity import (TAU_ABS, TAU_PRE, TAU_TIE, TOL, _adam_f64, assert_close, assert_rows_close, check_filtered_ranks,  # noqa: F401
                     check_topk, dense_gradient_floor, say)

TABLES = ob.TABLES


class BoxCase:
    def __init__(self, N, R, d, h, B, K, gamma, alpha=0.02, mix=None, seed=0, T=None, kg_alpha=2.1, trees=None,
                 pos=None, schedule="level", b_max=0):
        self.N, self.R, self.d, self.h, self.K, self.gamma, self.alpha = N, R, d, h, K, gamma, alpha
        self.schedule, self.b_max = schedule, b_max
        self.hp = dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, gamma=gamma, alpha=alpha)
        self.params = wl.make_box_params(N, R, d, h, seed + 3)
        if trees is not None:
            qb = wl.batch_from_trees(trees, pos)
            want = B or qb.B                             # B > 0: the first B of the trees that are clear of kinks
        else:
            kg = wl.make_kg(N, R, T or 10 * N, kg_alpha, seed)
            want = B
            qb = wl.make_batch(kg, B + B // 4 + 8, mix or {n: 1.0 for n in wl.EPFO9}, seed + 1)
        negs = wl.make_negatives(N, qb.B, K, seed + 2)
        self.qb, self.negs, self.n_redrawn = keep_clear_of_kinks(qb, negs, self.model(), N, want, seed + 4,
                                                                 strict=trees is None or B > 0)
        self.B = self.qb.B

    @classmethod
    def from_config(cls, idx, B=None, K=None, seed_offset=0):
        c = wl.get_config(idx)
        return cls(c.N, c.R, c.d, c.h, B or c.B, K or c.K, c.gamma, seed=c.seed + seed_offset, T=c.T, kg_alpha=c.alpha)

    distances_all = staticmethod(ob.distances_all)
    sem_bits = None

    def model(self):
        return ob.BoxModel(self.params, self.gamma, self.alpha)

    def fresh_negs(self, seed):
        negs = wl.make_negatives(self.N, self.B, self.K, seed)
        _, negs, _ = keep_clear_of_kinks(self.qb, negs, self.model(), self.N, self.B, seed + 1, strict=False,
                                         queries_are_clean=True)
        return negs

    def engine(self, num_streams=1):
        from paper_2602_21597_amd import Engine
        from paper_2602_21597_amd.binding import FAMILY_BOX
        eng = Engine(self.N, self.R, self.d, self.h, self.gamma, num_streams=num_streams, family=FAMILY_BOX,
                     box_alpha=self.alpha, schedule={"level": 0, "max_fill": 1}[self.schedule], b_max=self.b_max)
        eng.bind_numpy(self.params)
        return eng

    def neg_dev(self, negs=None):
        import torch
        return torch.from_numpy(np.ascontiguousarray(self.negs if negs is None else negs, np.int32)).cuda()


def keep_clear_of_kinks(qb, negs, M, N, want, seed, strict=True, queries_are_clean=False):
    rng = np.random.default_rng(seed)
    negs = negs.copy()
    keep, redrawn = [], 0
    for i in range(qb.B):
        if len(keep) == want:
            break
        fw = [ob.forward(b, M) for b in om.dnf(qb.tree(i))]
        C = np.stack([c for c, _, _ in fw])
        O = np.stack([o for _, o, _ in fw])
        margins = [ob.kink_margins(t) for _, _, t in fw]
        ok = min(m[0] for m in margins) >= TAU_PRE and min(m[1] for m in margins) >= TAU_ABS

        def clear(e):
            row = M.P["E"][e][None]
            dist = ob.box_distance(C, O, row, M.alpha)[:, 0]
            w = int(np.argmin(dist))
            tie = len(dist) > 1 and np.sort(dist)[1] - dist[w] < TAU_TIE
            a = np.abs(row[0] - C[w])
            return (not tie) and a.min() >= TAU_ABS and np.abs(a - O[w]).min() >= TAU_ABS

        ok = queries_are_clean or (ok and clear(int(qb.pos[i])))
        if ok:
            for j in range(negs.shape[1]):
                tries = 0
                while not clear(int(negs[i, j])):
                    negs[i, j] = rng.integers(0, N)
                    redrawn += 1
                    tries += 1
                    assert tries < 100
            keep.append(i)
        elif not strict:
            raise AssertionError("hand-built query %d sits on a kink; change the test's constants" % i)
    assert len(keep) == want, "not enough kink-free queries: %d of %d" % (len(keep), want)
    return qb.select(keep), negs[keep], redrawn


def check_forward_backward(case, eng=None, tol=TOL):
    """Plan, index, boxes at the roots, scores, loss and every gradient against the oracle."""
    import torch
    eng = eng or case.engine()
    plan = eng.plan(case.qb)
    ref_plan = oplan.build_plan(case.qb, case.schedule, case.b_max)
    got_plan = plan.export()
    for k in ref_plan:
        assert np.array_equal(np.asarray(got_plan[k]), np.asarray(ref_plan[k])), "plan." + k
    loss = eng.forward_backward(plan, case.neg_dev())
    torch.cuda.synchronize()
    g = eng.grads()
    M = case.model()
    ref_loss, G, ref_scores = ob.batch_loss_and_grads(case.qb, case.negs, M)

    u, off, src = oplan.entity_index(ref_plan, case.qb.pos, case.negs)
    assert np.array_equal(g["e_uniq"], u) and np.array_equal(g["e_seg_off"], off) and np.array_equal(g["e_src"], src)
    for q in range(case.B):
        br = om.dnf(case.qb.tree(q))
        slots = ref_plan["root_slot"][ref_plan["root_off"][q]:ref_plan["root_off"][q + 1]]
        for b, s in zip(br, slots):
            c, o, _ = ob.forward(b, M)
            assert_close(g["act"][s], c, "root centre q%d" % q, tol)
            assert_close(g["off"][s], o, "root offset q%d" % q, tol)
    if case.B:
        assert_close(g["pair_score"].reshape(case.B, case.K + 1), np.stack(ref_scores), "scores", tol)
        got_loss = float(loss.cpu()[0])
        assert abs(got_loss - ref_loss) <= tol * abs(ref_loss), "loss %r vs %r" % (got_loss, ref_loss)
    assert "W1" not in g
    floor = dense_gradient_floor(G.dense) if case.B else 0.0
    for name in G.dense:
        if name == "u2":      # softmax ignores a common shift of the logits: zero up to rounding
            assert np.abs(g[name]).max() <= tol * max(np.abs(G.dense["c2"]).max(), 1e-30), "grad u2 not ~0"
        elif np.abs(G.dense[name]).max() > 0:
            assert_close(g[name], G.dense[name], "grad " + name, tol, floor)
        else:
            assert np.abs(g[name]).max() == 0, name
    for tab, uniq, rows in (("E", g["e_uniq"], g["gE"]), ("R", got_plan["r_uniq"], g["gR"]),
                            ("Ro", got_plan["r_uniq"], g["gRo"])):
        assert sorted(G.rows[tab]) == list(uniq), tab + " touched rows"
        if len(uniq):
            ref_rows = np.stack([G.rows[tab][int(r)] for r in uniq])
            assert_close(rows, ref_rows, "grad " + tab, tol)
            # row by row, against the size of the row's contributions (an anchor that is also a
            # candidate of its query receives two that cancel: translations, oracle.box.Grads)
            assert_rows_close(rows, ref_rows, "grad rows " + tab, scale=[G.mass[tab][int(r)] for r in uniq])
    plan.free()
    return eng


def check_train_steps(case, steps=3, num_streams=1, tol=TOL):
    """As tests/parity.py: (A) the optimiser alone on the library's own gradients, every element;
    (B) end to end against the oracle's step on the well-conditioned elements."""
    import torch
    eng = case.engine(num_streams)
    plan = eng.plan(case.qb)
    pexp = plan.export()
    P = om.to_f64(case.params)
    state = {k: [np.zeros_like(v), np.zeros_like(v)] for k, v in P.items()}
    shapes = {k: v.shape for k, v in P.items()}
    for t in range(1, steps + 1):
        negs = case.fresh_negs(7000 + t)
        nd = case.neg_dev(negs)
        eng.forward_backward(plan, nd)
        gg = eng.grads()
        g_gpu = {n: gg[n].astype(np.float64) for n in shapes if n not in TABLES}
        touched_gpu = {"E": gg["e_uniq"], "R": pexp["r_uniq"], "Ro": pexp["r_uniq"]}
        for tab, key in (("E", "gE"), ("R", "gR"), ("Ro", "gRo")):
            full = np.zeros(shapes[tab], np.float64)
            full[touched_gpu[tab]] = gg[key]
            g_gpu[tab] = full
        before_ref = {k: v.copy() for k, v in P.items()}
        state_before = {k: [x.copy() for x in v] for k, v in state.items()}
        b_p, b_m, b_v = eng.params_numpy("p"), eng.params_numpy("m"), eng.params_numpy("v")
        loss = eng.train_step(plan, nd)
        torch.cuda.synchronize()
        ref_loss, G = ob.train_step(case.qb, negs, P, state, t, case.hp, track_sq=True)
        a_p, a_m, a_v = eng.params_numpy("p"), eng.params_numpy("m"), eng.params_numpy("v")
        if case.B:
            assert abs(float(loss.cpu()[0]) - ref_loss) <= tol * abs(ref_loss)
        assert eng.step_count() == t
        for name in P:
            ulp = np.spacing(np.abs(b_p[name]).astype(np.float32)).astype(np.float64)
            rows = slice(None)
            if name in TABLES:
                touched = np.zeros(shapes[name][0], bool)
                touched[touched_gpu[name]] = True
                assert sorted(G.rows[name]) == list(np.flatnonzero(touched)), name + " touched rows"
                for bb, aa in ((b_p, a_p), (b_m, a_m), (b_v, a_v)):
                    assert np.array_equal(aa[name][~touched], bb[name][~touched]), name + " untouched rows moved"
                rows = touched
            wp, wm, wv = _adam_f64(b_p[name][rows], b_m[name][rows], b_v[name][rows], g_gpu[name][rows], t, case.hp)
            upd = wp - b_p[name][rows]
            err = np.abs(a_p[name][rows] - wp)
            assert np.all(err <= tol * max(np.abs(upd).max(), 1e-300) + ulp[rows]), \
                "%s: Adam on own gradients, worst %.3g" % (name, err.max())
            assert_close(a_m[name][rows], wm, "m(own g) " + name, tol)
            assert_close(a_v[name][rows], wv, "v(own g) " + name, tol)
            if name == "u2":
                continue
            gref = G.table_dense(name, shapes[name]) if name in TABLES else G.dense[name]
            if np.abs(gref).max() == 0 or (name not in TABLES and np.abs(gref).max() < dense_gradient_floor(G.dense)):
                continue         # a tensor at the noise floor: the direction of its update is rounding noise
            m0, v0 = state_before[name]
            if name in TABLES:      # fp32 rounding level of a row sum: set by its contributions (oracle.box.Grads.mass)
                mass = np.zeros((shapes[name][0], 1))
                for i, v in G.mass[name].items():
                    mass[i, 0] = v
                delta = 1e-5 * mass
            else:                   # of a dense sum: independent errors of the terms add in quadrature
                rms = np.sqrt(G.dense_sq[name])
                delta = 1e-5 * np.maximum(rms, np.abs(gref).max() * 1e-3)
            hi = _adam_f64(before_ref[name], m0, v0, gref + delta, t, case.hp)[0]
            lo = _adam_f64(before_ref[name], m0, v0, gref - delta, t, case.hp)[0]
            upd_ref = P[name] - before_ref[name]
            scale = np.abs(upd_ref).max()
            keep = (np.abs(hi - lo) / 2 <= tol * scale)
            keep |= (gref == 0.0) & (g_gpu[name] == 0.0) & (m0 == 0.0) & (v0 == 0.0)   # dead units, now and before
            if name in TABLES:
                keep &= touched[:, None]
                n_all = int(touched.sum()) * shapes[name][1]
            else:
                n_all = keep.size
            upd_gpu = a_p[name].astype(np.float64) - b_p[name].astype(np.float64)
            err = np.abs(upd_gpu - upd_ref)
            bound = tol * scale + ulp
            assert np.all(err[keep] <= bound[keep]), \
                "%s update: worst %.3g x bound" % (name, (err[keep] / bound[keep]).max())
            cancels = name not in TABLES and np.abs(gref).max() < 0.05 * np.sqrt(G.dense_sq[name]).max()
            assert cancels or keep.sum() >= 0.3 * n_all, "%s: only %d of %d elements are well conditioned" % (
                name, keep.sum(), n_all)
            assert_close(a_m[name], state[name][0], "m " + name, tol)
            assert_close(a_v[name], state[name][1], "v " + name, 2 * tol)
    plan.free()
    return eng
