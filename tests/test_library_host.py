"""CPU-only checks of libngdb.so: it loads, exports what include/ngdb.h declares,
and its host planner reproduces the reference planner bit for bit."""
import ctypes
import os
import re

import numpy as np
import pytest

import workloads as wl
from oracle import plan as oplan
from paper_2602_21597_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "ngdb.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ngdb_[a-z_0-9]+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    names = declared_functions()
    assert {"ngdb_plan", "ngdb_train_step", "ngdb_score", "ngdb_create"} <= set(names)
    lib = ctypes.CDLL(binding.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    assert binding.lib().ngdb_strerror(-3).decode() == "entity or relation id out of range"


def same_plan(a, b):
    """a: the library's export, b: the reference plan (a carries a few derived counts more)."""
    assert set(b) <= set(a)
    for k in b:
        assert np.array_equal(np.asarray(a[k]), np.asarray(b[k])), k
    assert a["n_refs"] == len(b["in_ref"]) and a["n_r_uniq"] == len(b["r_uniq"])
    # rows of a forward-only pass with outputs reclaimed once their consumer has run
    f_row, n_rows, step_rows = oplan.forward_rows(b)
    assert np.array_equal(a["f_row"], f_row) and a["n_f_rows"] == n_rows == a["peak_live"]
    assert np.array_equal(a["f_step_rows"], step_rows)
    assert a["n_queries"] == len(a["pos"]) == len(b["root_off"]) - 1


@pytest.fixture(scope="module")
def kg():
    return wl.make_kg(3000, 40, 40000, 2.1, 21)


@pytest.mark.parametrize("seed,B", [(0, 1), (1, 64), (2, 700)])
def test_host_planner_is_bit_exact_with_reference(kg, seed, B):
    qb = wl.make_batch(kg, B, wl.get_config(1).mix, seed)
    same_plan(binding.plan_host(3000, 40, qb).export(), oplan.build_plan(qb))


def test_host_planner_weighted_mix_and_single_templates(kg):
    qb = wl.make_batch(kg, 256, wl.get_config(3).mix, 7)
    same_plan(binding.plan_host(3000, 40, qb).export(), oplan.build_plan(qb))
    for name in wl.configs.ALL14:
        qb = wl.make_batch(kg, 9, {name: 1.0}, 8)
        same_plan(binding.plan_host(3000, 40, qb).export(), oplan.build_plan(qb))


@pytest.mark.parametrize("b_max", [0, 1, 7, 64])
def test_host_planner_max_fillness_is_bit_exact_with_reference(kg, b_max):
    qb = wl.make_batch(kg, 300, wl.get_config(1).mix, 12)
    same_plan(binding.plan_host(3000, 40, qb, binding.SCHED_MAX_FILL, b_max).export(),
              oplan.build_plan(qb, "max_fill", b_max))
    qb = wl.make_batch(kg, 64, wl.get_config(3).mix, 13)
    same_plan(binding.plan_host(3000, 40, qb, binding.SCHED_MAX_FILL, b_max).export(),
              oplan.build_plan(qb, "max_fill", b_max))


def test_host_planner_general_shapes():
    trees = [
        ("p", 5, ("p", 4, ("u", ("p", 0, ("e", 1)), ("p", 1, ("e", 2)), ("p", 2, ("e", 3))))),
        ("i", ("p", 1, ("e", 2)), ("p", 2, ("e", 3)), ("p", 3, ("e", 4)), ("n", ("p", 4, ("e", 5)))),
        ("u", ("i", ("p", 1, ("e", 2)), ("p", 2, ("e", 3))), ("p", 3, ("n", ("p", 0, ("e", 9))))),
        ("n", ("e", 7)),
        ("i", ("e", 7), ("p", 2, ("e", 8))),
    ]
    qb = wl.batch_from_trees(trees, [0, 1, 2, 3, 4])
    same_plan(binding.plan_host(50, 6, qb).export(), oplan.build_plan(qb))
    same_plan(binding.plan_host(50, 6, wl.batch_from_trees([], [])).export(),
              oplan.build_plan(wl.batch_from_trees([], [])))


def test_host_planner_error_codes():
    def code(trees, pos, N=50, R=6):
        with pytest.raises(binding.NgdbError) as e:
            binding.plan_host(N, R, wl.batch_from_trees(trees, pos))
        return e.value.code

    one_p = ("p", 1, ("e", 2))
    assert code([("i", ("u", one_p, one_p), one_p)], [0]) == binding.ERR_UNSUPPORTED
    assert code([("n", ("u", one_p, one_p))], [0]) == binding.ERR_UNSUPPORTED
    assert code([("e", 3)], [0]) == binding.ERR_UNSUPPORTED
    assert code([("i",) + (one_p,) * 9], [0]) == binding.ERR_UNSUPPORTED
    assert code([("p", 6, ("e", 2))], [0]) == binding.ERR_RANGE
    assert code([("p", 1, ("e", 50))], [0]) == binding.ERR_RANGE
    assert code([one_p], [50]) == binding.ERR_RANGE
    assert code([("i", one_p)], [0]) == binding.ERR_ARG
    deep = ("e", 1)
    for _ in range(70):
        deep = ("p", 0, deep)
    assert code([deep], [0]) == binding.ERR_UNSUPPORTED
    # a forward reference is malformed input
    qb = wl.batch_from_trees([one_p], [0])
    qb.in_idx[0] = 1
    with pytest.raises(binding.NgdbError) as e:
        binding.plan_host(50, 6, qb)
    assert e.value.code == binding.ERR_ARG
