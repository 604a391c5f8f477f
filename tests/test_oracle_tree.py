"""Pins for the oracle's tree topology against the counts the paper prints."""
import itertools

import numpy as np
import pytest

from oracle import tree


@pytest.mark.parametrize("splits,nfe", [((0, 3, 6, 9), "13.68"), ((0, 4, 8, 12), "11.56"), ((0, 5, 10, 15), "9.44")])
def test_nfe_per_sample_matches_table_1_and_3(splits, nfe):
    # Sec. 4.2: depth 20, K = 2, 16 leaves; Table 1 / Table 3: average per-sample NFE
    t = tree.tree_build(20, splits, 2)
    assert t["n_leaves"] == 16
    val = tree.nfe_per_sample_all_nodes(t)
    assert abs(val - float(nfe)) < 0.01          # the paper prints two decimals
    assert {(0, 3, 6, 9): 219, (0, 4, 8, 12): 185, (0, 5, 10, 15): 151}[splits] == t["n_nodes"]


def test_leaf_counts_of_the_scaling_study():
    # Sec. 4.5: K = 2, 3, 4 with four splits -> 16, 81, 256; 3, 4, 5 splits (K = 2) -> 8, 16, 32
    for K, w in ((2, 16), (3, 81), (4, 256)):
        assert tree.tree_build(20, (0, 3, 6, 9), K)["n_leaves"] == w
    for splits, w in (((0, 3, 6), 8), ((0, 3, 6, 9), 16), ((0, 3, 6, 9, 12), 32)):
        assert tree.tree_build(20, splits, 2)["n_leaves"] == w


def test_widths_follow_the_noisy_end_reading():
    t = tree.tree_build(20, (0, 3, 6, 9), 2)
    assert list(t["width"]) == [1, 2, 2, 2, 4, 4, 4, 8, 8, 8] + [16] * 11
    assert tree.n_parent_evaluations(t) == 203   # non-leaf nodes


def test_k1_is_a_chain_and_ignores_splits():
    t = tree.tree_build(5, (1, 3), 1)
    assert t["n_nodes"] == 6 and t["n_leaves"] == 1
    assert list(t["parent"]) == [-1, 0, 1, 2, 3, 4]


@pytest.mark.parametrize("T,splits,K", [(3, (0, 2), 2), (4, (1, 2), 3), (5, (0, 1, 4), 2), (2, (), 2)])
def test_structure_by_brute_force(T, splits, K):
    t = tree.tree_build(T, splits, K)
    n = t["n_nodes"]
    # every non-root has a parent one level up; child counts are K at splits else 1
    for v in range(1, n):
        p = t["parent"][v]
        assert t["depth"][p] == t["depth"][v] - 1
    for v in range(n):
        kids = tree.children(t, v)
        d = t["depth"][v]
        if d == T:
            assert kids == []
        else:
            assert len(kids) == (K if d in splits else 1)
            assert [t["branch"][k] for k in kids] == list(range(len(kids)))
            j = v - t["off"][d]
            exp = [t["off"][d + 1] + j * K + b for b in range(K)] if d in splits else [t["off"][d + 1] + j]
            assert kids == exp
    # leaf intervals = set of leaves reachable by descending
    def reach(v):
        kids = tree.children(t, v)
        return {v - t["off"][T]} if not kids else set().union(*(reach(k) for k in kids))
    for v in range(n):
        assert reach(v) == set(range(t["leaf_lo"][v], t["leaf_hi"][v]))
    assert t["off"][T + 1] == n and t["n_edges"] == n - 1
