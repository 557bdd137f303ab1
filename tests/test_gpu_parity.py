"""HIP library against the CPU oracle on identical seeded inputs (needs an MI355X).

Plan and index arrays bit-exact; fp32 loss, activations, gradients and updates
within 1e-4 relative (definitions in tests/parity.py)."""
import numpy as np
import pytest

import workloads as wl
from oracle import model as om
from oracle import plan as oplan
from oracle import rank as orank
from tests import parity as par

pytestmark = pytest.mark.gpu


_say = par.say


def test_tiny_config_forward_backward():
    _say("config 0 (tiny), forward_backward")
    par.check_forward_backward(par.Case.from_config(0))


def test_tiny_config_unsaturated_margin():
    # margin near the typical distance so that negatives carry real gradient
    _say("config 0 shapes, gamma 3")
    c = wl.get_config(0)
    par.check_forward_backward(par.Case(c.N, c.R, c.d, c.h, c.B, c.K, 3.0, mix=c.mix, seed=5, T=c.T))


def test_tiny_config_train_steps():
    _say("config 0, 3 train steps")
    par.check_train_steps(par.Case.from_config(0), steps=3)


def test_all_templates_ragged_sizes():
    # d=400/h=800 rows that are no multiple of any tile, several tiles per GEMM
    _say("N=3000 d=400 h=800 B=150 K=19")
    par.check_forward_backward(par.Case(3000, 30, 400, 800, 150, 19, 55.0, seed=11))


def test_ragged_train_steps_multi_stream_matches_single_stream():
    _say("N=2000 d=100 h=72 B=90 K=7, streams 1 vs 4")
    case = par.Case(2000, 20, 100, 72, 90, 7, 12.0, seed=12)
    e1 = par.check_train_steps(case, steps=2, num_streams=1)
    e4 = par.check_train_steps(case, steps=2, num_streams=4)
    p1, p4 = e1.params_numpy(), e4.params_numpy()
    for k in p1:
        assert np.array_equal(p1[k], p4[k]), k


def test_general_shapes_wide_intersections_and_unions():
    _say("hand-built queries: 4..8-way intersections, 3-way unions, negated anchors")
    rng = np.random.default_rng(3)
    N, R = 300, 9

    def proj(depth=1):
        t = ("e", int(rng.integers(N)))
        for _ in range(depth):
            t = ("p", int(rng.integers(R)), t)
        return t

    trees = []
    for k in range(2, 9):
        trees.append(("i",) + tuple(proj(1 + (j % 2)) for j in range(k)))
    trees.append(("u", proj(), proj(2), proj(3)))
    trees.append(("p", 1, ("p", 2, ("u", proj(), proj()))))
    trees.append(("u", ("i", proj(), proj()), ("n", proj())))
    trees.append(("n", ("e", 5)))
    trees.append(("i", ("e", 6), proj()))
    trees.append(("i", ("n", ("e", 6)), ("e", 7), proj(), ("n", proj(2))))
    pos = [int(rng.integers(N)) for _ in trees]
    par.check_forward_backward(par.Case(N, R, 64, 128, 0, 6, 8.0, seed=13, trees=trees, pos=pos))
    par.check_train_steps(par.Case(N, R, 64, 128, 0, 6, 8.0, seed=13, trees=trees, pos=pos), steps=2)


@pytest.mark.parametrize("B", [1100, 2100])
def test_scoring_workgroup_shapes_with_unions(B):
    """Batches of 1024..2047 and of 2048 and more queries take the scoring kernel with 8 and with 4
    wavefronts per workgroup (other sums of the gradients over the wavefronts than the small
    batches of the other tests); unions of 2 and 3 branches at every position of the batch."""
    _say("B=%d: 1p / 2i / 2u / 3-way union / up / 2in, d=36 h=24 K=3; both families, text features" % B)
    from tests import parity_box as pb
    rng = np.random.default_rng(B)
    N, R = 900, 11

    def proj(depth=1):
        t = ("e", int(rng.integers(N)))
        for _ in range(depth):
            t = ("p", int(rng.integers(R)), t)
        return t

    def tree(kind, box):
        if kind == 0:
            return proj(1 + int(rng.integers(2)))
        if kind == 1:
            return ("i", proj(), proj())
        if kind == 2:
            return ("u", proj(), proj())
        if kind == 3:
            return ("u", proj(), proj(2), proj())
        if kind == 4:
            return ("p", int(rng.integers(R)), ("u", proj(), proj()))
        return ("i", proj(), proj()) if box else ("i", proj(), ("n", proj()))

    for box in (False, True):
        trees = [tree(int(rng.integers(6)), box) for _ in range(B + B // 2)]      # spares for those on a kink
        pos = [int(rng.integers(N)) for _ in trees]
        if box:
            cases = [pb.BoxCase(N, R, 36, 24, B, 3, 6.0, alpha=0.2, seed=B + 1, trees=trees, pos=pos)]
        else:
            cases = [par.Case(N, R, 36, 24, B, 3, 6.0, seed=B + 2, trees=trees, pos=pos),
                     par.Case(N, R, 40, 24, B, 3, 6.0, seed=B + 3, trees=trees, pos=pos, d_sem=64)]
        for case in cases:
            assert case.B == B
            (pb if box else par).check_forward_backward(case)


def test_degenerate_batches():
    _say("single query; all negatives equal; anchor = positive = negative; empty batch")
    one = par.Case(100, 5, 32, 64, 0, 5, 6.0, seed=14, trees=[("p", 1, ("e", 2))], pos=[3])
    par.check_forward_backward(one)
    case = par.Case(400, 8, 32, 64, 40, 9, 6.0, seed=15)
    case.negs[:] = 17
    case.negs[3, :] = int(case.qb.arg[0])          # an anchor entity as negative
    case.qb.pos[3] = int(case.qb.arg[0])           # and as positive
    par.check_forward_backward(case)
    par.check_train_steps(case, steps=1)
    empty = par.Case(100, 5, 32, 64, 0, 5, 6.0, seed=16, trees=[], pos=[])
    eng = empty.engine()
    plan = eng.plan(empty.qb)
    before = eng.params_numpy()
    loss = eng.train_step(plan, empty.neg_dev(np.zeros((0, 5), np.int32)))
    after = eng.params_numpy()
    assert float(loss.cpu()[0]) == 0.0
    for k in before:
        assert np.array_equal(before[k], after[k]), k   # zero gradient from zero state moves nothing


def test_candidate_scores_against_oracle():
    _say("ngdb_score candidate mode")
    import torch
    case = par.Case(500, 10, 48, 96, 60, 4, 10.0, seed=17)
    eng = case.engine()
    plan = eng.plan(case.qb)
    cand = wl.make_negatives(500, case.B, 33, 99)
    got = eng.score(plan, torch.from_numpy(cand).cuda()).cpu().numpy()
    want = orank.score_candidates(case.qb, cand, om.Model(case.params, 10.0))
    par.assert_close(got, want, "candidate scores")
    # a candidate list too long for the kernel's stash of per-pair results (its other store path)
    _say("ngdb_score candidate mode, 4500 candidates per query")
    few = case.qb.select(list(range(12)))
    plan = eng.plan(few)
    cand = wl.make_negatives(500, 12, 4500, 5)
    got = eng.score(plan, torch.from_numpy(cand).cuda()).cpu().numpy()
    want = orank.score_candidates(few, cand, om.Model(case.params, 10.0))
    par.assert_close(got, want, "candidate scores, long lists")


@pytest.mark.parametrize("schedule,b_max,d_sem", [("level", 0, 0), ("max_fill", 0, 0), ("max_fill", 7, 0), ("level", 0, 64)])
def test_forward_only_passes_reclaim_outputs(schedule, b_max, d_sem):
    """ngdb_score keeps an operator output only until its consumer has run (eager reference
    counting): fewer storage rows than outputs, the rows of the oracle's assignment, and scores
    bit-identical to those of the training pass, which keeps every output."""
    _say("forward-only pass with reclaimed outputs: %s schedule, B_max %d, d_sem %d" % (schedule, b_max, d_sem))
    import torch
    case = par.Case(2000, 20, 104, 72, 90, 7, 12.0, seed=61, schedule=schedule, b_max=b_max, d_sem=d_sem)
    eng = case.engine()
    plan = eng.plan(case.qb)
    pe = plan.export()
    f_row, n_rows, step_rows = oplan.forward_rows(oplan.build_plan(case.qb, schedule, b_max))
    assert np.array_equal(pe["f_row"], f_row) and pe["n_f_rows"] == n_rows == pe["peak_live"] < pe["n_slots"]
    assert np.array_equal(pe["f_step_rows"], step_rows)
    nd = case.neg_dev()
    eng.forward_backward(plan, nd)
    torch.cuda.synchronize()
    kept_all = eng.grads()["pair_score"].reshape(case.B, case.K + 1)[:, 1:]
    got = eng.score(plan, nd).cpu().numpy()
    assert np.array_equal(got, kept_all)
    par.assert_close(got, orank.score_candidates(case.qb, case.negs, case.model()), "candidate scores")
    plan.free()


def test_all_entity_topk_small_and_ragged():
    _say("ngdb_score all-entity mode: N=1000 (one ragged chunk), k=10 and k=16; N=300 d=64, k=1")
    par.check_topk(par.Case.from_config(0), 10, 64)
    par.check_topk(par.Case.from_config(0), 16, 16)
    par.check_topk(par.Case(300, 9, 64, 128, 20, 2, 8.0, seed=31), 1, 20)


def test_all_entity_topk_many_chunks():
    _say("ngdb_score all-entity mode: N=150000 (3 chunks), d=400, 200 queries incl. unions, k=10")
    case = par.Case(150000, 40, 400, 800, 200, 2, 24.0, seed=32, T=400000)
    par.check_topk(case, 10, 12)


# ---------------------------------------------------------------- filtered ranks, MRR, Hit@k
def test_filtered_ranks_and_metrics():
    _say("ngdb_rank_answers: N=1000 (one chunk); N=150000 d=64 (3 chunks); with text features")
    par.check_filtered_ranks(par.Case.from_config(0), 1)
    par.check_filtered_ranks(par.Case(150000, 20, 64, 128, 24, 2, 8.0, seed=51, T=300000), 2)
    par.check_filtered_ranks(par.Case(1500, 10, 48, 96, 30, 4, 6.0, seed=45, d_sem=128), 3)


# ---------------------------------------------------------------- Max-Fillness schedule
def test_max_fillness_schedule_same_values():
    _say("Max-Fillness steps, B_max = unbounded / 64 / 5: N=3000 d=400 h=800 B=150 K=19; tiny config train steps")
    for b_max in (0, 64, 5):
        par.check_forward_backward(par.Case(3000, 30, 400, 800, 150, 19, 55.0, seed=11, schedule="max_fill",
                                            b_max=b_max))
    c = wl.get_config(0)
    par.check_train_steps(par.Case(c.N, c.R, c.d, c.h, c.B, c.K, c.gamma, mix=c.mix, seed=c.seed, T=c.T,
                                   schedule="max_fill", b_max=16), steps=2)


def test_max_fillness_schedule_with_text_features_and_streams():
    _say("Max-Fillness steps with text features (d_sem=128) and 3 streams")
    case = par.Case(1200, 12, 64, 128, 70, 9, 8.0, seed=41, d_sem=128, schedule="max_fill", b_max=32)
    par.check_forward_backward(case, eng=case.engine(num_streams=3))


# ---------------------------------------------------------------- text-feature fusion
def test_text_features_forward_backward():
    _say("d_sem=128: N=1200 d=64 h=128 B=70 K=9")
    par.check_forward_backward(par.Case(1200, 12, 64, 128, 70, 9, 8.0, seed=41, d_sem=128))


def test_text_features_ragged_tiles():
    # d=104: coordinate tiles of 80 + 24; d_sem=320: feature tiles of 256 + 64; ~700 touched rows: 3 row tiles
    _say("d_sem=320: N=700 d=104 h=72 B=120 K=11")
    par.check_forward_backward(par.Case(700, 9, 104, 72, 120, 11, 12.0, seed=42, d_sem=320))


def test_text_features_train_steps():
    _say("d_sem=64: N=900 d=32 h=64 B=60 K=8, 3 train steps; streams 1 vs 3 bit-identical")
    case = par.Case(900, 10, 32, 64, 60, 8, 5.0, seed=43, d_sem=64)
    e1 = par.check_train_steps(case, steps=3)
    e3 = par.check_train_steps(case, steps=3, num_streams=3)
    p1, p3 = e1.params_numpy(), e3.params_numpy()
    for k in p1:
        assert np.array_equal(p1[k], p3[k]), k


def test_text_features_workload_widths():
    # the widths of the text-feature workload (d=400, h=800, d_sem=1024) on a small graph
    _say("d_sem=1024: N=6000 d=400 h=800 B=96 K=24, forward_backward + 1 train step")
    case = par.Case(6000, 30, 400, 800, 96, 24, 30.0, seed=44, d_sem=1024)
    par.check_forward_backward(case)
    par.check_train_steps(case, steps=1)


def test_text_features_scores_and_ranking():
    import torch
    _say("d_sem=128: candidate scores and all-entity top-k")
    case = par.Case(1500, 10, 48, 96, 50, 4, 6.0, seed=45, d_sem=128)
    eng = case.engine()
    plan = eng.plan(case.qb)
    cand = wl.make_negatives(case.N, case.B, 21, 98)
    got = eng.score(plan, torch.from_numpy(cand).cuda()).cpu().numpy()
    want = orank.score_candidates(case.qb, cand, om.Model(case.params, case.gamma, case.sem_bits))
    par.assert_close(got, want, "candidate scores with text features")
    plan.free()
    par.check_topk(case, 10, 16)
    par.check_topk(par.Case(70000, 10, 64, 128, 30, 2, 8.0, seed=46, T=200000, d_sem=64), 5, 6)   # 2 entity chunks


def test_text_features_bad_widths_are_rejected():
    from paper_2602_21597_amd import Engine, NgdbError, binding
    for d, d_sem in ((64, 100), (36, 64)):
        with pytest.raises(NgdbError) as e:
            Engine(100, 5, d, 64, 6.0, d_sem=d_sem)
        assert e.value.code == binding.ERR_ARG


def _bf16_bits(x):
    b = np.ascontiguousarray(x, np.float32).view(np.uint32)
    return ((b + 0x7FFF + ((b >> 16) & 1)) >> 16).astype(np.uint16)


def test_candidate_rows_from_a_bf16_copy_of_the_table():
    _say("score_bf16: N=2000 d=104 h=72 B=90 K=7 and N=3000 d=400 h=800 B=150 K=19; copy stays the rounding of E")
    import torch
    small = par.Case(2000, 20, 104, 72, 90, 7, 12.0, seed=61, score_bf16=True)
    par.check_forward_backward(small)
    par.check_train_steps(small, steps=1, num_streams=2)
    case = par.Case(3000, 30, 400, 800, 150, 19, 55.0, seed=62, score_bf16=True)
    eng = par.check_forward_backward(case)
    # the values are those of the rounded rows, not of the fp32 rows
    g = eng.grads()
    s_fp32 = np.stack(om.batch_loss_and_grads(case.qb, case.negs, om.Model(case.params, case.gamma), want_grads=False)[2])
    assert np.abs(g["pair_score"].reshape(case.B, case.K + 1) - s_fp32).max() > 1e-3
    np.testing.assert_array_equal(g["e_shadow"], _bf16_bits(case.params["E"]))
    # three steps: the copy follows the table bit for bit; untouched rows keep theirs
    plan = eng.plan(case.qb)
    for t in range(3):
        eng.train_step(plan, case.neg_dev(case.fresh_negs(7100 + t)))
    torch.cuda.synchronize()
    eng.forward_backward(plan, case.neg_dev())
    np.testing.assert_array_equal(eng.grads()["e_shadow"], _bf16_bits(eng.params_numpy()["E"]))
    # candidate scores and the all-entity ranking read the same rows
    cand = wl.make_negatives(case.N, case.B, 9, 5)
    M = case.model()
    fresh = case.engine()
    p2 = fresh.plan(case.qb)
    got = fresh.score(p2, torch.from_numpy(cand).cuda()).cpu().numpy()
    par.assert_close(got, orank.score_candidates(case.qb, cand, M), "candidate scores from the bf16 copy")
    par.check_topk(case, 10, 8)
    par.check_filtered_ranks(par.Case(1000, 20, 32, 64, 40, 8, 12.0, seed=63, score_bf16=True), 4)


def test_fb15k237_shape_full_size():
    # the benchmark workload itself, in the launch configuration bench.py times
    _say("config 1 (B=512, K=128, d=400), forward_backward + 1 train step")
    case = par.Case.from_config(1)
    streams = wl.get_config(1).streams                    # the launch configuration bench.py times
    par.check_forward_backward(case, eng=case.engine(num_streams=streams))
    par.check_train_steps(case, steps=1, num_streams=streams)


def test_planning_on_a_second_thread_gives_the_same_parameters():
    _say("config 0: 12 steps, batch t+1 planned on a second host thread while step t is enqueued")
    from concurrent.futures import ThreadPoolExecutor
    import torch
    case = par.Case.from_config(0)
    kg = wl.make_kg(case.N, case.R, 10 * case.N, 2.1, 77)
    c = wl.get_config(0)
    batches = [wl.make_batch(kg, c.B, c.mix, 80 + i) for i in range(4)]
    negs = [torch.from_numpy(wl.make_negatives(case.N, c.B, c.K, 90 + i)).cuda() for i in range(4)]
    serial, threaded = case.engine(), case.engine()
    for i in range(12):
        p = serial.plan(batches[i % 4])
        serial.train_step(p, negs[i % 4])
        p.free()
    with ThreadPoolExecutor(1) as ex:
        nxt = ex.submit(threaded.plan, batches[0])
        for i in range(12):
            p = nxt.result()
            if i + 1 < 12:
                nxt = ex.submit(threaded.plan, batches[(i + 1) % 4])
            threaded.train_step(p, negs[i % 4])
            p.free()
    a, b = serial.params_numpy(), threaded.params_numpy()
    for k in a:
        assert np.array_equal(a[k], b[k]), k
    assert threaded.step_count() == 12


def test_sampled_batches_train_like_any_other():
    _say("online sampler -> plan -> forward_backward: plan, scores and loss against the oracle on 3 sampled batches")
    import torch
    from paper_2602_21597_amd import Sampler
    c = wl.get_config(0)
    kg = wl.make_kg(c.N, c.R, c.T, c.alpha, c.seed)
    params = wl.make_params(c.N, c.R, c.d, c.h, 3)
    from paper_2602_21597_amd import Engine
    eng = Engine(c.N, c.R, c.d, c.h, c.gamma)
    eng.bind_numpy(params)
    M = om.Model(params, c.gamma)
    smp = Sampler(c.N, c.R, kg.head, kg.rel, kg.tail, list(wl.configs.ALL14), None, 7, 4)
    for _ in range(3):
        b = smp.next(96, 6)
        plan = eng.plan(b)
        ref_plan = oplan.build_plan(b)
        got_plan = plan.export()
        for k in ref_plan:
            assert np.array_equal(np.asarray(got_plan[k]), np.asarray(ref_plan[k])), "plan." + k
        loss = eng.forward_backward(plan, torch.from_numpy(b.negs).cuda())
        torch.cuda.synchronize()
        ref_loss, _, ref_scores = om.batch_loss_and_grads(b, b.negs, M, want_grads=False)
        par.assert_close(eng.grads()["pair_score"].reshape(b.B, 7), np.stack(ref_scores), "scores")
        assert abs(float(loss.cpu()[0]) - ref_loss) <= 1e-4 * abs(ref_loss)
        plan.free()


def test_declared_maxima_steps_allocate_nothing():
    """With b_max_queries / k_max declared, ngdb_create allocates everything: 50 steps of sampled batches
    of varying sizes (planning, training, candidate scoring) make no device allocation, the
    parameters end up bit-identical to those of a context that grows on demand, and a batch beyond
    the maxima is refused."""
    _say("declared maxima: 50 steps of varying batch sizes allocate nothing; same results as growing on demand")
    import torch
    from paper_2602_21597_amd import Engine, Sampler
    from paper_2602_21597_amd.binding import NgdbError, ERR_ARG
    c = wl.get_config(0)
    kg = wl.make_kg(c.N, c.R, c.T, c.alpha, c.seed)
    params = wl.make_params(c.N, c.R, c.d, c.h, 3)
    fixed = Engine(c.N, c.R, c.d, c.h, c.gamma, num_streams=2, b_max_queries=96, k_max=16)
    grows = Engine(c.N, c.R, c.d, c.h, c.gamma, num_streams=2)
    fixed.bind_numpy(params)
    grows.bind_numpy(params)
    n0 = fixed.alloc_count()
    assert n0 > 0
    smp = Sampler(c.N, c.R, kg.head, kg.rel, kg.tail, list(wl.configs.ALL14), None, 21, 2)
    rng = np.random.default_rng(4)
    for t in range(50):
        b = smp.next(int(rng.integers(1, 97)), int(rng.integers(1, 17)))
        negs = torch.from_numpy(b.negs).cuda()
        for eng in (fixed, grows):
            plan = eng.plan(b)
            eng.train_step(plan, negs)
            if t % 10 == 0:
                eng.score(plan, negs)
            plan.free()
    torch.cuda.synchronize()
    assert fixed.alloc_count() == n0, "a step allocated device memory although maxima were declared"
    assert grows.alloc_count() > 0
    pf, pg = fixed.params_numpy(), grows.params_numpy()
    for k in pf:
        assert np.array_equal(pf[k], pg[k]), k
    too_many = smp.next(97, 4)
    with pytest.raises(NgdbError) as ei:
        fixed.plan(too_many)
    assert ei.value.code == ERR_ARG
    ok = smp.next(20, 16)
    plan = fixed.plan(ok)
    with pytest.raises(NgdbError) as ei:
        fixed.train_step(plan, torch.zeros((20, 17), dtype=torch.int32, device="cuda"))
    assert ei.value.code == ERR_ARG
    plan.free()
    assert fixed.alloc_count() == n0


@pytest.mark.parametrize("family", ["vec", "box"])
def test_long_run_of_the_whole_pipeline_learns(family):
    """600 steps of sampler -> planner thread -> train step with the library stream on: the steady
    state of the plan-buffer pool, the events and the two streams; the loss of a fixed probe batch,
    measured by the oracle on the parameters before and after, must fall."""
    _say("600 steps, online sampler, planning on a second thread, library stream; %s family" % family)
    import torch
    from concurrent.futures import ThreadPoolExecutor
    from oracle import box as ob
    from paper_2602_21597_amd import Engine, Sampler, binding
    c = wl.get_config(0)
    box = family == "box"
    kg = wl.make_kg(c.N, c.R, c.T, c.alpha, c.seed)
    params = wl.make_box_params(c.N, c.R, c.d, c.h, 3) if box else wl.make_params(c.N, c.R, c.d, c.h, 3)
    eng = Engine(c.N, c.R, c.d, c.h, 3.0, lr=3e-3, num_streams=2, family=binding.FAMILY_BOX if box else 0,
                 box_alpha=0.25)
    eng.bind_numpy(params)
    names = list(wl.EPFO9 if box else wl.configs.ALL14)
    smp = Sampler(c.N, c.R, kg.head, kg.rel, kg.tail, names, None, 11, 4)
    probe = Sampler(c.N, c.R, kg.head, kg.rel, kg.tail, names, None, 12, 1).next(128, 16)

    def probe_loss(p):
        if box:
            return ob.batch_loss_and_grads(probe, probe.negs, ob.BoxModel(p, 3.0, 0.25), want_grads=False)[0]
        return om.batch_loss_and_grads(probe, probe.negs, om.Model(p, 3.0), want_grads=False)[0]

    before = probe_loss(eng.params_numpy())
    B, K = 64, 16
    pool = ThreadPoolExecutor(1)

    def produce():
        b = smp.next(B, K)
        return eng.plan(b), torch.from_numpy(b.negs).pin_memory()

    nxt = pool.submit(produce)
    losses = []
    for t in range(600):
        plan, negs = nxt.result()
        nxt = pool.submit(produce)
        loss = eng.train_step(plan, negs.cuda(non_blocking=True))
        plan.free()
        if t % 100 == 99:
            losses.append(float(loss.cpu()[0]))
    nxt.result()[0].free()
    pool.shutdown()
    torch.cuda.synchronize()
    assert eng.step_count() == 600 and np.all(np.isfinite(losses))
    after = probe_loss(eng.params_numpy())
    assert after < 0.9 * before, (before, after, losses)


def test_errors_are_reported_not_raised_as_faults():
    from paper_2602_21597_amd import NgdbError, binding
    case = par.Case.from_config(0)
    eng = case.engine()
    with pytest.raises(NgdbError) as e:
        eng.plan(wl.batch_from_trees([("p", 99, ("e", 1))], [0]))
    assert e.value.code == binding.ERR_RANGE
    host_plan = binding.plan_host(case.N, case.R, case.qb)
    with pytest.raises(NgdbError) as e:
        eng.train_step(host_plan, case.neg_dev())
    assert e.value.code == binding.ERR_ARG
    # ranking calls: a plan without a device, top-k out of range, answer lists without output
    import torch
    L = binding.lib()
    plan = eng.plan(case.qb)
    ids = torch.empty((case.B, 4), dtype=torch.int32, device="cuda")
    dist = torch.empty((case.B, 4), dtype=torch.float32, device="cuda")
    assert L.ngdb_score(eng.ctx, plan.handle, None, 0, 0, None, ids.data_ptr(), dist.data_ptr(), None) == binding.ERR_ARG
    assert L.ngdb_score(eng.ctx, plan.handle, None, 0, 17, None, ids.data_ptr(), dist.data_ptr(), None) == binding.ERR_ARG
    assert L.ngdb_score(eng.ctx, host_plan.handle, None, 0, 4, None, ids.data_ptr(), dist.data_ptr(), None) == binding.ERR_ARG
    off = torch.zeros(case.B + 1, dtype=torch.int32, device="cuda")
    assert L.ngdb_rank_answers(eng.ctx, plan.handle, off.data_ptr(), None, 3, None, None, None) == binding.ERR_ARG
    assert L.ngdb_rank_answers(eng.ctx, plan.handle, None, None, 0, None, None, None) == binding.ERR_ARG
    assert L.ngdb_rank_answers(eng.ctx, plan.handle, off.data_ptr(), None, 0, None, None, None) == binding.NGDB_OK
    assert L.ngdb_rank_metrics(None, None, None, 0, None, None) == binding.ERR_ARG
    fresh = binding.Engine(case.N, case.R, case.d, case.h, case.gamma)        # nothing bound yet
    p2 = fresh.plan(case.qb)
    with pytest.raises(NgdbError) as e:
        fresh.train_step(p2, case.neg_dev())
    assert e.value.code == binding.ERR_STATE
    loss = torch.zeros(1, device="cuda")
    assert L.ngdb_train_step(eng.ctx, plan.handle, case.neg_dev().data_ptr(), 0, None, loss.data_ptr()) == binding.ERR_ARG
    assert L.ngdb_train_step(eng.ctx, plan.handle, None, case.K, None, loss.data_ptr()) == binding.ERR_ARG
    assert L.ngdb_train_step(eng.ctx, plan.handle, case.neg_dev().data_ptr(), case.K, None, None) == binding.ERR_ARG
    with pytest.raises(NgdbError) as e:
        binding.Engine(case.N, case.R, case.d, case.h, case.gamma, schedule=7)
    assert e.value.code == binding.ERR_ARG
    # a plan that outlives its context: still readable and freeable, no longer executable
    short_lived = case.engine()
    orphan = short_lived.plan(case.qb)
    short_lived.close()
    assert orphan.export()["n_queries"] == case.B
    with pytest.raises(NgdbError) as e:
        eng.train_step(orphan, case.neg_dev())
    assert e.value.code == binding.ERR_ARG
    orphan.free()
    # the bf16 copy: plain vector family only, width a multiple of 8
    for kw in (dict(d=32, d_sem=64), dict(d=32, family=binding.FAMILY_BOX), dict(d=36)):
        with pytest.raises(NgdbError) as e:
            binding.Engine(case.N, case.R, kw.pop("d"), 64, case.gamma, score_bf16=True, **kw)
        assert e.value.code == binding.ERR_ARG
