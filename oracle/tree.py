"""Rollout-tree topology for the oracle (test infrastructure).

Sec. 3.2 "Preliminaries": depth T = number of denoising steps, width w = number
of leaves, branching steps B = split timesteps, branching factor K.  Alg. 1
(tree-building loop): at every step a node either takes a single denoising step
or, if the step is in B, branches into K children.

Reading used (the paper's loop counts down while Eq. 2 / App. B.1 and the
ablation "early splits such as (0,3,6,9)" index from the noisy end): step i is
the transition from depth i to depth i+1, i = 0 the first (noisiest) step, and
i in B means every depth-i node gets K children at depth i+1.

Nodes are numbered in level order: node (d, j), j in [0, width_d), has local id
off[d] + j; the children of (i, j) are (i+1, j*K + b), b in [0, K), at a split
step and (i+1, j) otherwise.

Pins (tests/test_oracle_tree.py): the paper's leaf counts (Sec. 4.2: 16 leaves;
Sec. 4.5: 16/81/256 and 8/16/32) and per-sample NFE figures (Table 1: 13.68;
Table 3: 13.68/11.56/9.44), brute-force descendant sets on small trees.
"""
import numpy as np


def tree_build(T, split_steps, K):
    """Topology of one tree as a dict of int32 arrays.

    width[d], d = 0..T; off[d], d = 0..T+1 (off[T+1] = n_nodes); for each node
    parent (root: -1), depth, branch (index among its siblings; 0 if only
    child), and [leaf_lo, leaf_hi): the interval of leaf indices below it."""
    T = int(T)
    K = int(K)
    splits = sorted(int(s) for s in split_steps) if K > 1 else []
    assert T >= 1 and K >= 1
    assert all(0 <= s < T for s in splits) and len(set(splits)) == len(splits)
    width = [1]
    for i in range(T):
        width.append(width[-1] * (K if i in splits else 1))
    off = [0]
    for d in range(T + 1):
        off.append(off[-1] + width[d])
    n_nodes = off[-1]
    w = width[T]
    parent = np.full(n_nodes, -1, dtype=np.int32)
    depth = np.zeros(n_nodes, dtype=np.int32)
    branch = np.zeros(n_nodes, dtype=np.int32)
    leaf_lo = np.zeros(n_nodes, dtype=np.int32)
    leaf_hi = np.zeros(n_nodes, dtype=np.int32)
    for d in range(T + 1):
        for j in range(width[d]):
            n = off[d] + j
            depth[n] = d
            if d > 0:
                if (d - 1) in splits:
                    parent[n] = off[d - 1] + j // K
                    branch[n] = j % K
                else:
                    parent[n] = off[d - 1] + j
    # leaves below a node: walk every leaf up to the root (plain definition)
    below = [[] for _ in range(n_nodes)]
    for leaf in range(w):
        n = off[T] + leaf
        while n >= 0:
            below[n].append(leaf)
            n = parent[n]
    for n in range(n_nodes):
        ls = sorted(below[n])
        assert ls == list(range(ls[0], ls[-1] + 1))  # contiguous by construction
        leaf_lo[n], leaf_hi[n] = ls[0], ls[-1] + 1
    return dict(T=T, K=K, splits=list(splits), width=np.array(width, np.int32),
                off=np.array(off, np.int32), n_nodes=n_nodes, n_edges=n_nodes - 1,
                n_leaves=w, parent=parent, depth=depth, branch=branch,
                leaf_lo=leaf_lo, leaf_hi=leaf_hi)


def children(tree, n):
    """Local ids of the children of node n (empty for a leaf)."""
    return [int(c) for c in np.nonzero(tree["parent"] == n)[0]]


def nfe_per_sample_all_nodes(tree):
    """Table 1 caption: total function evaluations in the tree / final samples,
    with the paper's count of one evaluation per tree node."""
    return tree["n_nodes"] / tree["n_leaves"]


def n_parent_evaluations(tree):
    """Network evaluations when each parent is evaluated once: the drift of
    Eq. 2 depends only on the parent, so this is the number of non-leaf nodes."""
    return tree["n_nodes"] - tree["n_leaves"]
