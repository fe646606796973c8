"""CPU oracle of the draft-tree topology choice.  TEST INFRASTRUCTURE ONLY.

Imported by tests/ only; the product (`firp_build_tree` in the library) shares no code with it.

What is defined here (paper: Experiment / Setup, "search for the best tree structures" under a
budget of tree nodes; Inference stage for what a step accepts):

* `expected_tokens(parent, rank, accept)`: the exact expectation of the number of tokens one
  step emits with a given draft tree, written out from the verification rule itself.  The
  target's token at draft level i is the rank-r candidate of prediction step i with probability
  accept[i][r] (the events exclude each other; with the remaining probability it is none of
  them), independently per level.  Every joint outcome is enumerated; for each one the walk of
  greedy verification is run on the tree (descend to the child that carries the target's
  token, stop when there is none) and the tokens it emits are counted (accepted nodes + 1).
* `best_tree_value(accept, n_nodes)`: the maximum of that expectation over every tree of at most
  `n_nodes` nodes whose nodes are rank paths of depth <= k, by brute force over all
  ancestor-closed subsets of the complete b-ary tree.  Only for tiny k, b, n.
"""
from __future__ import annotations

import itertools
from typing import List, Sequence, Tuple


def expected_tokens(parent: Sequence[int], rank: Sequence[int], accept: Sequence[Sequence[float]]) -> float:
    k = len(accept)
    b = len(accept[0]) if k else 0
    n = len(parent)
    children: List[List[int]] = [[] for _ in range(n)]
    for v in range(1, n):
        children[parent[v]].append(v)
    total = 0.0
    # outcome[i] in 0..b-1: the target's token at level i+1 is that rank; b: none of the candidates
    for outcome in itertools.product(range(b + 1), repeat=k):
        p = 1.0
        for i, r in enumerate(outcome):
            p *= accept[i][r] if r < b else 1.0 - sum(accept[i])
        if p == 0.0:
            continue
        cur, emitted, level = 0, 1, 0
        while level < k:
            nxt = next((c for c in children[cur] if rank[c] == outcome[level]), None)
            if nxt is None:
                break
            cur = nxt
            emitted += 1
            level += 1
        total += p * emitted
    return total


def _complete_tree(k: int, b: int) -> List[Tuple[int, ...]]:
    nodes: List[Tuple[int, ...]] = [()]
    for level in range(1, k + 1):
        nodes += list(itertools.product(range(b), repeat=level))
    return nodes


def best_tree_value(accept: Sequence[Sequence[float]], n_nodes: int) -> float:
    k = len(accept)
    b = len(accept[0]) if k else 0
    nodes = _complete_tree(k, b)[1:]
    best = 1.0
    for m in range(0, min(n_nodes - 1, len(nodes)) + 1):
        for subset in itertools.combinations(nodes, m):
            chosen = set(subset)
            if any(len(v) > 1 and v[:-1] not in chosen for v in chosen):
                continue                         # not ancestor-closed
            order = [()] + sorted(chosen, key=lambda v: (len(v), v))
            index = {v: i for i, v in enumerate(order)}
            parent = [-1] + [index[v[:-1]] for v in order[1:]]
            rank = [0] + [v[-1] for v in order[1:]]
            best = max(best, expected_tokens(parent, rank, accept))
    return best
