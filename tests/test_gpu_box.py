"""Box family of the HIP library against oracle.box on identical seeded inputs (needs an MI355X).
Plan and index arrays bit-exact; fp32 values within 1e-4 relative (tests/parity_box.py)."""
import numpy as np
import pytest

import workloads as wl
from oracle import box as ob
from tests import parity_box as pb

pytestmark = pytest.mark.gpu
_say = pb.say


def test_box_tiny_forward_backward_and_steps():
    _say("box family, N=1000 d=32 h=64 B=64 K=8")
    case = pb.BoxCase(1000, 20, 32, 64, 64, 8, 3.0, alpha=0.25, seed=1)
    pb.check_forward_backward(case)
    pb.check_train_steps(case, steps=3)


def test_box_paper_alpha_saturated_margin():
    _say("box family, alpha 0.02, gamma 12")
    pb.check_forward_backward(pb.BoxCase(1000, 20, 32, 64, 64, 8, 12.0, alpha=0.02, seed=2))


def test_box_workload_widths_ragged_sizes():
    # d=400/h=800 rows that are no multiple of any tile, several tiles per contraction
    _say("box family, N=3000 d=400 h=800 B=150 K=19")
    case = pb.BoxCase(3000, 30, 400, 800, 150, 19, 24.0, alpha=0.02, seed=3)
    pb.check_forward_backward(case)
    pb.check_train_steps(case, steps=2)


def test_box_odd_width_and_streams():
    _say("box family, d=100 h=72, streams 1 vs 4")
    case = pb.BoxCase(2000, 20, 100, 72, 90, 7, 6.0, alpha=0.1, seed=4)
    e1 = pb.check_train_steps(case, steps=2, num_streams=1)
    e4 = pb.check_train_steps(case, steps=2, num_streams=4)
    p1, p4 = e1.params_numpy(), e4.params_numpy()
    for k in p1:
        assert np.array_equal(p1[k], p4[k]), k


def test_box_wide_intersections_unions_and_max_fillness():
    _say("box family, hand-built queries: 2..8-way intersections, unions; both schedules")
    rng = np.random.default_rng(5)
    N, R = 300, 9

    def proj(depth=1):
        t = ("e", int(rng.integers(N)))
        for _ in range(depth):
            t = ("p", int(rng.integers(R)), t)
        return t

    trees = [("i",) + tuple(proj(1 + (j % 2)) for j in range(k)) for k in range(2, 9)]
    trees.append(("u", proj(), proj(2), proj(3)))
    trees.append(("p", 1, ("p", 2, ("u", proj(), proj()))))
    trees.append(("u", ("i", proj(), proj()), proj(2)))
    trees.append(("p", 3, ("i", proj(), ("i", proj(), proj(2)))))
    same = proj()
    trees.append(("i", same, same))                       # equal offsets: the first input takes the gradient
    pos = [int(rng.integers(N)) for _ in trees]
    for schedule, b_max in (("level", 0), ("max_fill", 0), ("max_fill", 3)):
        case = pb.BoxCase(N, R, 64, 128, 0, 6, 4.0, alpha=0.25, seed=6, trees=trees, pos=pos, schedule=schedule,
                          b_max=b_max)
        pb.check_forward_backward(case)
    pb.check_train_steps(case, steps=2)


def test_box_degenerate_batches():
    # (an anchor that is also its query's positive and every negative has an exactly zero gradient
    # here: the projection is a translation, so the two sides of every pair cancel)
    _say("box family: single query; anchor = every negative; empty batch")
    one = pb.BoxCase(100, 5, 32, 64, 0, 5, 2.0, alpha=0.25, seed=7, trees=[("p", 1, ("e", 2))], pos=[3])
    pb.check_forward_backward(one)
    same = pb.BoxCase(100, 5, 32, 64, 0, 3, 2.0, alpha=0.25, seed=8, trees=[("p", 1, ("e", 2)), ("p", 2, ("e", 2))],
                      pos=[3, 4])
    same.negs[:] = 2
    pb.check_forward_backward(same)
    pb.check_train_steps(same, steps=2)
    empty = pb.BoxCase(100, 5, 32, 64, 0, 3, 2.0, seed=9, trees=[], pos=[])
    eng = empty.engine()
    plan = eng.plan(empty.qb)
    before = eng.params_numpy()
    loss = eng.train_step(plan, empty.neg_dev())
    assert float(loss.cpu()[0]) == 0.0
    after = eng.params_numpy()
    for k in ("E", "R", "Ro"):
        assert np.array_equal(before[k], after[k]), k


def test_box_candidate_scores():
    _say("box family: ngdb_score candidate mode")
    import torch
    case = pb.BoxCase(500, 10, 48, 96, 60, 4, 10.0, alpha=0.25, seed=10)
    eng = case.engine()
    plan = eng.plan(case.qb)
    cand = wl.make_negatives(500, case.B, 33, 99)
    got = eng.score(plan, torch.from_numpy(cand).cuda()).cpu().numpy()
    M = case.model()
    want = np.stack([ob.query_step(case.qb.query_nodes(i), int(cand[i, 0]), cand[i, 1:], M, 1)[1]
                     for i in range(case.B)])
    pb.assert_close(got, want, "candidate scores")


def test_box_all_entity_topk_and_filtered_ranks():
    _say("box family: all-entity top-k (1 ragged chunk; 3 chunks of 65 536) and filtered ranks")
    pb.check_topk(pb.BoxCase(1000, 20, 32, 64, 64, 8, 3.0, alpha=0.25, seed=12), 10, 32)
    pb.check_topk(pb.BoxCase(150000, 40, 400, 800, 100, 2, 24.0, alpha=0.02, seed=13, T=400000), 10, 8)
    pb.check_filtered_ranks(pb.BoxCase(1000, 20, 32, 64, 64, 8, 3.0, alpha=0.25, seed=14), 1)
    pb.check_filtered_ranks(pb.BoxCase(150000, 20, 64, 128, 24, 2, 8.0, alpha=0.1, seed=15, T=300000), 2)


def test_box_fb15k237_shape_full_size():
    _say("box family at the FB15k-237 shape: N=15000 d=400 h=800 B=512 K=128")
    case = pb.BoxCase.from_config(1)
    pb.check_forward_backward(case, eng=case.engine(num_streams=wl.get_config(1).streams))


def test_box_errors():
    from paper_2602_21597_amd import NgdbError, binding
    case = pb.BoxCase(100, 5, 32, 64, 4, 3, 2.0, seed=11)
    eng = case.engine()
    for tree in (("n", ("p", 1, ("e", 2))), ("i", ("e", 3), ("p", 1, ("e", 2)))):
        with pytest.raises(NgdbError) as e:
            eng.plan(wl.batch_from_trees([tree], [0]))
        assert e.value.code == binding.ERR_UNSUPPORTED
    L = binding.lib()
    for kw in (dict(d_sem=64), dict(box_alpha=-1.0), dict(box_alpha=1.5), dict(box_alpha=float("nan"))):
        with pytest.raises(NgdbError) as e:
            binding.Engine(100, 5, 32, 64, 2.0, family=binding.FAMILY_BOX, **kw)
        assert e.value.code == binding.ERR_ARG
    with pytest.raises(NgdbError) as e:
        binding.Engine(100, 5, 32, 64, 2.0, family=2)
    assert e.value.code == binding.ERR_ARG
    fresh = binding.Engine(100, 5, 32, 64, 2.0, family=binding.FAMILY_BOX)
    P = binding.Params()                                  # relation offsets missing
    for name, (p, m, v) in eng.tensors.items():
        if name != "Ro":
            setattr(P, name, binding.Tensor(p.data_ptr(), m.data_ptr(), v.data_ptr()))
    import ctypes as C
    assert L.ngdb_bind_params(fresh.ctx, C.byref(P)) == binding.ERR_ARG
