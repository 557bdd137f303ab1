"""The relabelling helper of the full-size GPU tests (no GPU needed): renumbering the entities
a batch reads, and handing the oracle only their rows, must not change any result."""
import numpy as np

import workloads as wl
from oracle import model as om
from tests.test_gpu_parity_large import _compact


def test_compact_relabelling_leaves_the_oracle_results_unchanged():
    N, R, d, h, B, K = 900, 8, 16, 24, 30, 5
    kg = wl.make_kg(N, R, 9000, 2.1, 3)
    qb = wl.make_batch(kg, B, {n: 1.0 for n in wl.configs.ALL14}, 4)
    negs = wl.make_negatives(N, B, K, 5)
    params = wl.make_params(N, R, d, h, 6, d_sem=64)
    sem = wl.make_sem_features(N, 64, 7)
    full_loss, G, scores = om.batch_loss_and_grads(qb, negs, om.Model(params, 6.0, sem))
    qc, nc, pc, sc, used = _compact(qb, negs, params, sem)
    assert pc["E"].shape[0] == len(used) < N and sc.shape[0] == len(used)
    loss_c, Gc, scores_c = om.batch_loss_and_grads(qc, nc, om.Model(pc, 6.0, sc))
    assert loss_c == full_loss
    for a, b in zip(scores, scores_c):
        assert np.array_equal(a, b)
    for n in G.dense:
        assert np.array_equal(G.dense[n], Gc.dense[n]), n
    assert [int(used[i]) for i in sorted(Gc.rows["E"])] == sorted(G.rows["E"])
    for i, row in Gc.rows["E"].items():
        assert np.array_equal(row, G.rows["E"][int(used[i])])
    assert sorted(Gc.rows["R"]) == sorted(G.rows["R"])
