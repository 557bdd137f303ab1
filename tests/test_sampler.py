"""The library's online query sampler (host only): validity of every sampled query against a
symbolic evaluation of the query on the graph, shapes, mixture, determinism, errors."""
import numpy as np
import pytest

import workloads as wl
from oracle import plan as oplan
from paper_2602_21597_amd import NgdbError, Sampler, binding

ALL14 = list(wl.configs.ALL14)


@pytest.fixture(scope="module")
def kg():
    return wl.make_kg(400, 12, 6000, 2.1, 5)


def make(kg, templates=ALL14, weights=None, seed=1, n_threads=4):
    return Sampler(kg.N, kg.R, kg.head, kg.rel, kg.tail, templates, weights, seed, n_threads)


def tree_of(b, i):
    nodes = wl.QueryBatch.query_nodes(b, i)

    def build(j):
        op, arg, ins = nodes[j]
        if op == 0:
            return ("e", arg)
        if op == 1:
            return ("p", arg, build(ins[0]))
        if op == 3:
            return ("n", build(ins[0]))
        return ("i" if op == 2 else "u",) + tuple(build(k) for k in ins)

    return build(len(nodes) - 1)


def answers(tree, out_edges, N):
    """Set semantics of a query on the graph: projection = image under a relation,
    intersection / union of sets, negation = complement."""
    kind = tree[0]
    if kind == "e":
        return {tree[1]}
    if kind == "p":
        src = answers(tree[2], out_edges, N)
        return {t for s in src for t in out_edges.get((s, tree[1]), ())}
    if kind == "n":
        return set(range(N)) - answers(tree[1], out_edges, N)
    sets = [answers(c, out_edges, N) for c in tree[1:]]
    return set.intersection(*sets) if kind == "i" else set.union(*sets)


def shape(tree):
    """The template a query instantiates: the tree with ids removed."""
    if tree[0] == "e":
        return ("e",)
    if tree[0] == "p":
        return ("p", shape(tree[2]))
    return (tree[0],) + tuple(shape(c) for c in tree[1:])


def test_every_sampled_positive_is_an_answer_and_shapes_match(kg):
    out_edges = {}
    for h, r, t in zip(kg.head, kg.rel, kg.tail):
        out_edges.setdefault((int(h), int(r)), set()).add(int(t))
    b = make(kg).next(700, 3)
    assert b.B == 700 and b.negs.shape == (700, 3)
    assert b.negs.min() >= 0 and b.negs.max() < kg.N
    seen = set()
    for i in range(b.B):
        tree = tree_of(b, i)
        assert shape(tree) == wl.configs.TEMPLATES[b.names[i]], b.names[i]
        assert int(b.pos[i]) in answers(tree, out_edges, kg.N), (b.names[i], tree)
        if tree[0] == "i":                     # no two identical children
            assert len(set(tree[1:])) == len(tree) - 1
        seen.add(b.names[i])
    assert seen == set(ALL14)
    # the batch plans like any other
    qb = wl.batch_from_trees([tree_of(b, i) for i in range(b.B)], list(b.pos))
    got = binding.plan_host(kg.N, kg.R, b).export()
    ref = oplan.build_plan(qb)
    for k in ref:
        assert np.array_equal(np.asarray(got[k]), np.asarray(ref[k])), k


def test_batches_do_not_depend_on_thread_count_and_differ_from_each_other(kg):
    s1, s4 = make(kg, n_threads=1), make(kg, n_threads=4)
    first = None
    for step in range(3):
        a, b = s1.next(300, 5), s4.next(300, 5)
        for f in ("node_off", "op", "arg", "in_off", "in_idx", "pos", "negs"):
            assert np.array_equal(getattr(a, f), getattr(b, f)), f
        assert a.names == b.names
        if first is None:
            first = a
        else:
            assert not np.array_equal(first.pos, a.pos)
    again = make(kg, n_threads=2).next(300, 5)
    assert np.array_equal(again.arg, first.arg) and np.array_equal(again.negs, first.negs)
    other = make(kg, seed=2).next(300, 5)
    assert not np.array_equal(other.pos, first.pos)


def test_read_ahead_does_not_change_the_batches_and_keeps_one_valid_over_the_next_call(kg):
    """Batch t is a function of (seed, t, sizes): a sampler that is asked for other sizes in
    between (its read-ahead is dropped each time) gives the same batches as one asked for equal
    sizes throughout (read-ahead used); a raw batch stays unchanged over the following call."""
    steady, mixed = make(kg, seed=5), make(kg, seed=5, n_threads=3)
    for t in range(6):
        a = steady.next(200, 6)
        b = mixed.next(200, 6) if t % 2 else mixed.next(17 + t, 2)
        if t % 2:
            for f in ("node_off", "op", "arg", "in_off", "in_idx", "pos", "negs"):
                assert np.array_equal(getattr(a, f), getattr(b, f)), (t, f)
    s = make(kg, seed=6)
    c0, n0 = s.next_raw(128, 9)
    keep = n0.copy()
    s.next_raw(128, 9)
    assert np.array_equal(n0, keep)
    s.close()                                            # with a batch being read ahead


def test_template_mixture_follows_the_weights(kg):
    s = make(kg, ["1p", "2i", "pni"], [0.6, 0.3, 0.1], seed=3)
    names = []
    for _ in range(4):
        names += s.next(1000, 0).names
    frac = {n: names.count(n) / len(names) for n in ("1p", "2i", "pni")}
    assert abs(frac["1p"] - 0.6) < 0.03 and abs(frac["2i"] - 0.3) < 0.03 and abs(frac["pni"] - 0.1) < 0.02
    assert make(kg, ["2u"]).next(5, 0).names == ["2u"] * 5
    assert make(kg).next(0, 4).B == 0


def test_sampler_errors():
    with pytest.raises(NgdbError) as e:
        Sampler(10, 2, [0, 1], [0, 1], [1, 2], ["1p", "4p"])
    assert e.value.code == binding.ERR_ARG
    with pytest.raises(NgdbError) as e:
        Sampler(10, 2, [0, 11], [0, 1], [1, 2], ["1p"])
    assert e.value.code == binding.ERR_RANGE
    with pytest.raises(NgdbError) as e:
        Sampler(10, 2, [0], [0], [1], ["1p"], weights=[0.0])
    assert e.value.code == binding.ERR_ARG
    # a graph whose only edge cannot carry a two-hop walk: sampling reports, does not spin
    s = Sampler(10, 2, [0], [0], [1], ["2p"])
    with pytest.raises(NgdbError) as e:
        s.next(4, 1)
    assert e.value.code == binding.ERR_UNSUPPORTED and "2p" in str(e.value)
