"""Draft-tree topology for a node budget: the library's choice against the brute-force oracle
(host only, no GPU)."""
import numpy as np
import pytest

from oracle import tree_search_oracle as tso
from paper_2410_20488_amd import binding


def _table(seed, k, b):
    g = np.random.default_rng(seed)
    a = g.random((k, b))
    a = np.sort(a, axis=1)[:, ::-1] * g.uniform(0.3, 0.95, size=(k, 1)) / a.sum(axis=1, keepdims=True)
    return a.astype(np.float32)      # per level: decreasing in rank, sum below 1


def _valid(parent, rank, k, b):
    level = [0] * len(parent)
    assert parent[0] == -1
    for v in range(1, len(parent)):
        assert 0 <= parent[v] < v and 0 <= rank[v] < b
        level[v] = level[parent[v]] + 1
        assert level[v] <= k
    kids = {}
    for v in range(1, len(parent)):
        assert (parent[v], rank[v]) not in kids, "two children of a node with the same rank"
        kids[(parent[v], rank[v])] = v


def test_oracle_expectation_closed_forms():
    """The outcome enumeration against hand-computed cases: a chain accepts level by level
    (1 + p + p^2), siblings add up, a node below a rejected parent adds its path product."""
    a = [[0.5, 0.25], [0.4, 0.1]]
    assert tso.expected_tokens([-1], [0], a) == 1.0
    assert abs(tso.expected_tokens([-1, 0, 1], [0, 0, 0], a) - (1 + 0.5 + 0.5 * 0.4)) < 1e-12
    assert abs(tso.expected_tokens([-1, 0, 0], [0, 0, 1], a) - (1 + 0.5 + 0.25)) < 1e-12
    assert abs(tso.expected_tokens([-1, 0, 0, 2], [0, 0, 1, 1], a) - (1 + 0.5 + 0.25 + 0.25 * 0.1)) < 1e-12


@pytest.mark.parametrize("seed,k,b,n", [(1, 2, 3, 5), (2, 2, 3, 7), (3, 3, 2, 6), (4, 3, 2, 9), (5, 1, 4, 3),
                                        (6, 2, 2, 7)])
def test_library_tree_is_optimal_and_its_value_exact(seed, k, b, n):
    a = _table(seed, k, b)
    parent, rank, value = binding.build_tree(a, n)
    _valid(parent, rank, k, b)
    assert len(parent) <= n
    exact = tso.expected_tokens(parent, rank, a.astype(np.float64).tolist())
    assert abs(value - exact) < 1e-9
    best = tso.best_tree_value(a.astype(np.float64).tolist(), n)
    assert abs(value - best) < 1e-9, (value, best)


def test_degenerate_tables_and_budgets():
    # only the first candidate is ever right: the best tree is the chain, cut at k levels
    a = np.array([[0.8, 0.0], [0.5, 0.0], [0.25, 0.0]], dtype=np.float32)
    parent, rank, value = binding.build_tree(a, 10)
    assert parent == [-1, 0, 1, 2] and rank == [0, 0, 0, 0]
    assert abs(value - (1 + 0.8 + 0.4 + 0.1)) < 1e-6      # the rates are fp32
    # ties: shallower node first, then the smaller rank path
    a = np.full((2, 2), 0.5, dtype=np.float32)
    parent, rank, _ = binding.build_tree(a, 4)
    assert parent == [-1, 0, 0, 1] and rank == [0, 0, 1, 0]
    # budget of one node: the root alone
    assert binding.build_tree(a, 1) == ([-1], [0], 1.0)
    # k = 0: nothing to draft
    assert binding.build_tree(np.zeros((0, 1), dtype=np.float32), 5) == ([-1], [0], 1.0)


def test_argument_errors():
    lib = binding.load_library()
    import ctypes as C
    a = (C.c_float * 2)(0.5, 1.5)
    buf = (C.c_int32 * 4)()
    n = C.c_int32(0)
    assert lib.firp_build_tree(a, 1, 2, 4, buf, buf, C.byref(n), None) == -1      # rate above 1
    a = (C.c_float * 2)(0.5, 0.25)
    assert lib.firp_build_tree(a, 1, 2, 0, buf, buf, C.byref(n), None) == -1      # no root
    assert lib.firp_build_tree(None, 1, 2, 4, buf, buf, C.byref(n), None) == -1
    assert lib.firp_build_tree(a, 1, 2, 4, buf, buf, C.byref(n), None) == 0 and n.value == 3
