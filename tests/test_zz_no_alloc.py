"""ngdb_score_noalloc (candidate scoring whose forward workspace is a static device array)
against ngdb_score, through the C boundary (needs an MI355X).  Collected last on purpose."""
import numpy as np
import pytest

import workloads as wl
from oracle import model as om
from oracle import rank as orank
from tests import parity as par

pytestmark = pytest.mark.gpu


def test_score_noalloc_matches_score_on_two_calls_in_a_row():
    par.say("ngdb_score_noalloc against ngdb_score and the oracle: 200 queries x 33 candidates, then 23 x 5")
    import torch
    from paper_2602_21597_amd.binding import NgdbError, ERR_ARG
    case = par.Case(3000, 30, 400, 800, 200, 4, 24.0, seed=61)
    eng = case.engine()
    M = om.Model(case.params, 24.0)
    # first a large input, then a smaller one: the scratch keeps the first call's rows
    for n_q, C, seed in ((200, 33, 7), (23, 5, 8)):
        qb = case.qb.select(np.arange(n_q))
        plan = eng.plan(qb)
        cand_np = wl.make_negatives(case.N, n_q, C, seed)
        cand = torch.from_numpy(cand_np).cuda()
        out = torch.full((n_q, C), float("nan"), dtype=torch.float32, device="cuda")
        assert 0 < eng.score_noalloc_bytes(plan) <= 32 << 20
        got = eng.score_noalloc(plan, cand, out).cpu().numpy()
        want = eng.score(plan, cand).cpu().numpy()
        assert np.array_equal(got, want)                       # same kernels, same arithmetic: bit for bit
        par.assert_close(got, orank.score_candidates(qb, cand_np, M), "candidate scores (no-alloc entry)")
        plan.free()
    # a batch beyond the static array is refused, with the sizes in the message
    big = par.Case(3000, 30, 400, 800, 3000, 1, 24.0, seed=62)
    eng2 = big.engine()
    plan = eng2.plan(big.qb)
    assert eng2.score_noalloc_bytes(plan) > 32 << 20
    cand = torch.zeros((big.B, 2), dtype=torch.int32, device="cuda")
    out = torch.zeros((big.B, 2), dtype=torch.float32, device="cuda")
    with pytest.raises(NgdbError) as ei:
        eng2.score_noalloc(plan, cand, out)
    assert ei.value.code == ERR_ARG and "static scratch" in str(ei.value)
    assert np.isfinite(eng2.score(plan, cand).cpu().numpy()).all()      # the allocating entry point still takes it
    plan.free()
