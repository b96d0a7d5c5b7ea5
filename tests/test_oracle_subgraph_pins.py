"""Pins for the oracle's optimal-subgraph search of the offline calibration (Alg. 2 part 3, App. D.1), checked
without a GPU: a hand-worked example, the breadth-first growth from the root levels as a second formulation,
and closed forms on structured graphs."""
import itertools
import json
import math
import os

import numpy as np
import pytest

from oracle import spiffy_oracle as O
from paper_2509_18085_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def grow_connected_sets(level, edges, N, D):
    """Second formulation, the breadth-first brute force App. D.2 mentions: start from the single root-level
    nodes and add, one at a time, a node that is root-level or has a parent in the set.  On an acyclic graph
    this reaches every connected set."""
    parents = [set() for _ in range(N)]
    for p, q in edges:
        parents[q].add(p)
    frontier = {frozenset([r]) for r in range(N) if level[r] in (1, 2)}
    for _ in range(D - 1):
        nxt = set()
        for g in frontier:
            for q in range(N):
                if q not in g and (level[q] in (1, 2) or parents[q] & g):
                    nxt.add(g | {q})
        frontier = nxt
    return frontier if D >= 1 else {frozenset()}


def all_connected_sets(count, level, edges, D):
    N = len(count)
    parents = [set() for _ in range(N)]
    for p, q in edges:
        parents[q].add(int(p))
    return {frozenset(c) for c in itertools.combinations(range(N), D) if O.subgraph_is_connected(c, level, parents)}


def test_hand_worked_example():
    g = json.load(open(os.path.join(GOLDEN, "subgraph_case.json")))
    for c in g["cases"]:
        r = O.subgraph_search(g["count"], g["level"], np.array(g["edges"]), c["D"])
        assert r["n_connected"] == len(c["sets"]), c
        assert r["best_nodes"] == c["best_nodes"] and r["best_sum"] == c["best_sum"] and r["best_mask"] == c["best_mask"], c
        assert all_connected_sets(g["count"], g["level"], g["edges"], c["D"]) == {frozenset(s) for s in c["sets"]}


@pytest.mark.parametrize("seed", range(6))
def test_growth_from_the_roots_finds_the_same_sets_and_optimum(seed):
    count, level, edges, _ = synth.candidate_graph(4 + seed % 3, seed=seed)
    N = len(count)
    for D in (1, 2, 3, 5, min(7, N)):
        grown = grow_connected_sets(level, [tuple(e) for e in edges.tolist()], N, D)
        assert grown == all_connected_sets(count, level, edges, D)
        r = O.subgraph_search(count, level, edges, D)
        assert r["n_connected"] == len(grown)
        best = max(grown, key=lambda g: (sum(int(count[q]) for q in g), -sum(1 << q for q in g)))
        assert sorted(best) == r["best_nodes"]
        assert r["best_sum"] == sum(int(count[q]) for q in best) and r["best_mask"] == sum(1 << q for q in best)


def test_all_root_level_nodes_take_the_largest_counts():
    count = [7, 3, 9, 9, 1, 4, 9, 2]
    level = [1, 2, 1, 2, 2, 1, 1, 2]
    for D in range(1, 9):
        r = O.subgraph_search(count, level, np.zeros((0, 2), int), D)
        assert r["n_connected"] == math.comb(8, D)
        order = sorted(range(8), key=lambda q: (-count[q], q))[:D]          # equal counts: lower node first
        assert r["best_nodes"] == sorted(order) and r["best_sum"] == sum(count[q] for q in order)


def test_chain_and_star():
    # chain 0 -> 1 -> 2 -> 3 -> 4, only node 0 root-level: the one connected set of size D is the first D nodes
    level = [1, 3, 4, 5, 6]
    count = [1, 50, 2, 90, 3]
    edges = np.array([[0, 1], [1, 2], [2, 3], [3, 4]])
    for D in range(1, 6):
        r = O.subgraph_search(count, level, edges, D)
        assert r["n_connected"] == 1 and r["best_nodes"] == list(range(D)) and r["best_sum"] == sum(count[:D])
    # star: root 0, leaves 1..6 at level 3: the root plus any D-1 leaves
    level = [2] + [3] * 6
    count = [1, 8, 3, 9, 4, 7, 2]
    edges = np.array([[0, q] for q in range(1, 7)])
    for D in range(1, 8):
        r = O.subgraph_search(count, level, edges, D)
        assert r["n_connected"] == math.comb(6, D - 1)
        leaves = sorted(range(1, 7), key=lambda q: -count[q])[:D - 1]
        assert r["best_nodes"] == sorted([0] + leaves)


def test_one_parent_in_the_set_is_enough_and_direction_matters():
    # node 3 (level 3) has parents 1 and 2 (level 2) and a child 4 (level 4)
    level = [1, 2, 2, 3, 4]
    count = [1, 1, 1, 100, 1000]
    edges = np.array([[1, 3], [2, 3], [3, 4]])
    r = O.subgraph_search(count, level, edges, 2)
    assert r["best_nodes"] == [1, 3] and r["best_sum"] == 101            # {1,3} and {2,3} tie: smaller mask
    assert r["n_connected"] == 3 + 2                                         # pairs of roots, {1,3}, {2,3}
    # {3,4}: node 4 has its parent, node 3 has none in the set -> not connected, however large the counts
    assert not O.subgraph_is_connected([3, 4], level, [set(), set(), set(), {1, 2}, {3}])
    r3 = O.subgraph_search(count, level, edges, 3)
    assert r3["best_nodes"] == [1, 3, 4] and r3["best_sum"] == 1101
    # rows with an end outside the graph are ignored
    r_bad = O.subgraph_search(count, level, np.array([[1, 3], [2, 3], [3, 4], [9, 4], [-1, 3], [0, 7]]), 3)
    assert r_bad == r3


def test_equal_sums_go_to_the_smallest_mask_and_level_three_is_not_a_root():
    level = [1, 1, 1, 1]
    r = O.subgraph_search([5, 5, 5, 5], level, np.zeros((0, 2), int), 2)
    assert r["best_nodes"] == [0, 1] and r["best_mask"] == 3 and r["n_connected"] == 6
    r = O.subgraph_search([5, 5, 5, 5], [1, 2, 3, 3], np.zeros((0, 2), int), 2)
    assert r["n_connected"] == 1 and r["best_nodes"] == [0, 1]
    # the condition is the local one of App. D.1: two non-root nodes that are each other's parent count as connected
    r = O.subgraph_search([1, 1, 9, 9], [1, 2, 3, 3], np.array([[2, 3], [3, 2]]), 2)
    assert r["best_nodes"] == [2, 3] and r["n_connected"] == 2
