"""The synthetic input generators: determinism, shapes, structure."""
import os

import numpy as np

import workloads as wl
from oracle import plan as oplan
from workloads.queries import OP_ANCHOR, OP_PROJ


def test_kg_is_distinct_loop_free_and_heavy_tailed():
    kg = wl.make_kg(2000, 15, 30000, 2.1, 5)
    assert kg.T == 30000
    assert np.unique(kg.keys).shape[0] == 30000
    assert np.all(kg.head != kg.tail)
    assert kg.head.min() >= 0 and kg.head.max() < 2000 and kg.rel.max() < 15
    assert np.all(np.diff(kg.tail) >= 0)
    indeg = np.diff(kg.in_off)
    assert indeg.sum() == 30000
    assert indeg.max() > 20 * max(1.0, np.median(indeg))       # hubs exist
    for j in (0, 17, 29999):
        assert kg.has_triple(kg.head[j], kg.rel[j], kg.tail[j])
    kg2 = wl.make_kg(2000, 15, 30000, 2.1, 5)
    assert np.array_equal(kg.keys, kg2.keys)


def test_batches_are_seeded_and_walks_follow_edges():
    kg = wl.make_kg(500, 8, 6000, 2.1, 6)
    cfg = wl.get_config(1)
    a = wl.make_batch(kg, 64, cfg.mix, 1)
    b = wl.make_batch(kg, 64, cfg.mix, 1)
    c = wl.make_batch(kg, 64, cfg.mix, 2)
    assert np.array_equal(a.arg, b.arg) and np.array_equal(a.pos, b.pos)
    assert not np.array_equal(a.pos, c.pos)
    assert set(a.names) <= set(cfg.mix)
    # a 1p query's (anchor, relation, positive) is an edge of the graph
    for i, name in enumerate(a.names):
        if name == "1p":
            (o0, ent, _), (o1, rel, ins) = a.query_nodes(i)
            assert o0 == OP_ANCHOR and o1 == OP_PROJ and ins == [0]
            assert kg.has_triple(ent, rel, int(a.pos[i]))
    # round trip through the nested form
    rt = wl.batch_from_trees([a.tree(i) for i in range(a.B)], a.pos)
    for f in ("node_off", "op", "arg", "in_off", "in_idx"):
        assert np.array_equal(getattr(a, f), getattr(rt, f))


def test_negatives_and_params():
    n = wl.make_negatives(1000, 16, 8, 3)
    assert n.shape == (16, 8) and n.dtype == np.int32 and n.min() >= 0 and n.max() < 1000
    p = wl.make_params(100, 5, 8, 16, 1, d_sem=4)
    assert p["W1"].shape == (16, 8) and p["W2"].shape == (8, 16) and p["Wp"].shape == (8, 4)
    assert all(v.dtype == np.float32 and np.abs(v).max() <= 0.1 for v in p.values())
    s = wl.make_sem_features(10, 64, 2)
    f = (s.astype(np.uint32) << 16).view(np.float32)
    assert np.allclose(np.linalg.norm(f, axis=1), 1.0, atol=2e-2)


def test_config_table():
    c = wl.get_config(1)
    assert (c.N, c.R, c.d, c.h, c.K, c.B, c.gamma) == (15000, 474, 400, 800, 128, 512, 24.0)
    assert abs(sum(wl.get_config(3).mix.values()) - 1.0) < 1e-12
    assert wl.get_config("tiny").B == 64 and wl.get_config(4).d_sem == 1024


def _golden(name):
    path = os.path.join(os.path.dirname(__file__), "golden", name)
    with open(path) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


def test_pattern_names_are_the_papers_fourteen():
    """The pattern list of the preliminaries: the workload mix, the hand-written operator
    census of the planner tests and the structure of every template (one projection per
    'p' counted with its multiplier, and so on) all refer to exactly these names."""
    from tests.test_plan_oracle import CENSUS
    names = [row[0] for row in _golden("query_patterns.txt")]
    assert len(names) == 14 and len(set(names)) == 14
    assert set(names) == set(wl.configs.ALL14) == set(CENSUS) == set(wl.configs.TEMPLATES)
    for c in (1, 2, 3, 4):
        assert set(wl.get_config(c).mix) == set(names)
    # what the name itself says about the operators of the pattern
    for name in names:
        _, _, groups = CENSUS[name]
        has = {t for (_, t, _) in groups}
        assert (oplan.OP_NEG in has) == ("n" in name), name
        assert (oplan.OP_INTER in has) == ("i" in name), name
        assert oplan.OP_PROJ in has, name
        roots = CENSUS[name][1]
        assert (roots > 1) == ("u" in name), name


def test_workload_sizes_follow_the_papers_graph_table():
    """Entity, relation and edge counts of the synthetic graphs stay within 4 % of the
    appendix table (relations doubled: one inverse each)."""
    rows = {r[0]: tuple(int(x) for x in r[1:]) for r in _golden("kg_statistics.txt")}
    for cfg, key in ((1, "FB15k-237"), (2, "NELL995"), (3, "ogbl-wikikg2")):
        c = wl.get_config(cfg)
        n, r, t = rows[key]
        assert abs(c.N - n) <= 0.04 * n, (key, c.N, n)
        assert c.R == 2 * r, (key, c.R, r)
        assert abs(c.T - t) <= 0.04 * t, (key, c.T, t)
