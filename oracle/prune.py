"""Width and depth pruning (Sec. 3.4) for the oracle (test infrastructure).

Pruning runs after fusion and normalisation and only selects which edges take
part in the policy update; rollouts, rewards, fused rewards and advantages are
untouched (Sec. 3.4, second paragraph).

Width pruning chooses a subset of leaves:
  Parent-Top1   of the children of each parent at the last branching step, keep
                the one with the higher reward (tie: lower branch index);
  Extreme-b     keep the b globally best and the b worst leaves of a tree by
                reward, ordered by (reward, leaf index); 2b >= w keeps all.
Depth pruning: a set of pruned step indices; edges of those steps are dropped.
The sliding-window schedule starts at the last split step, has a fixed size and
moves one step deeper at fixed iteration intervals until it reaches a stop
depth (Sec. 3.4 "Depth pruning"; Sec. 4.4: size 4, every 30 iterations).

Reading for which edges a kept leaf keeps (paper silent): edge (p -> c) is kept
iff c has at least one kept descendant leaf and step depth(c)-1 is not pruned.
Output: ascending global child ids.

Pins (tests/test_oracle_prune.py): Parent-Top1 keeps w/K leaves and every
last-split parent keeps exactly one child; Extreme-b on hand values; the kept
edge set equals a brute-force union of root-to-leaf paths; window positions at
given iterations.
"""
import numpy as np

from . import philox


def width_keep_leaves(tree, rewards_tree, mode, b=0):
    """Boolean [w] for one tree.  mode: 0 none (keep all), 1 Parent-Top1,
    2 Extreme-b.  rewards are compared as float32, the precision they are given in."""
    w, K, T = tree["n_leaves"], tree["K"], tree["T"]
    r = np.asarray(rewards_tree, np.float32)
    keep = np.zeros(w, dtype=bool)
    if mode == 0 or (mode == 1 and (K == 1 or not tree["splits"])):
        keep[:] = True
    elif mode == 1:
        # no split follows the last one, so each child of a last-split parent
        # has exactly one leaf below it: child j of that depth <-> leaf j
        last = max(tree["splits"])
        assert int(tree["width"][last + 1]) == w
        for parent_j in range(w // K):
            sibs = [parent_j * K + br for br in range(K)]
            best = sibs[0]
            for j in sibs[1:]:
                if r[j] > r[best]:
                    best = j
            keep[best] = True
    elif mode == 2:
        if 2 * b >= w:
            keep[:] = True
        else:
            order = sorted(range(w), key=lambda l: (float(r[l]), l))
            for l in order[:b] + order[w - b:]:
                keep[l] = True
    else:
        raise ValueError(mode)
    return keep


def kept_edges(tree, leaf_rewards, n_cond, mode, b, depth_pruned):
    """Ascending int32 array of kept global child ids over all trees."""
    nn, w, T = tree["n_nodes"], tree["n_leaves"], tree["T"]
    r = np.asarray(leaf_rewards, np.float32).reshape(n_cond, w)
    out = []
    for c in range(n_cond):
        keep = width_keep_leaves(tree, r[c], mode, b)
        for n in range(1, nn):
            lo, hi = int(tree["leaf_lo"][n]), int(tree["leaf_hi"][n])
            if keep[lo:hi].any() and not depth_pruned[int(tree["depth"][n]) - 1]:
                out.append(c * nn + n)
    return np.array(out, dtype=np.int32)


def depth_mask_window(T, last_split, window, iteration, every, stop):
    """Sliding-window set of pruned steps as a uint8 mask [T]."""
    start = min(last_split + iteration // every, stop - window)
    start = max(start, 0)
    mask = np.zeros(T, dtype=np.uint8)
    mask[start:min(start + window, T)] = 1
    return mask


def depth_mask_seeded(T, n_drop, seed):
    """A seeded subset of n_drop steps: rank steps by (Philox word, step) with
    the word drawn from counter (0, 0, step, depth tag); drop the smallest."""
    x = [int(philox.words(seed, 0, i, philox.TAG_DEPTH, 1)[0, 0]) for i in range(T)]
    order = sorted(range(T), key=lambda i: (x[i], i))
    mask = np.zeros(T, dtype=np.uint8)
    mask[order[:n_drop]] = 1
    return mask


def mix_schedule(T, split_steps, window_mask, eta):
    """Hybrid ODE-SDE schedule (ablation "Hybrid ODE-SDE"): split steps and the steps inside the
    sliding window are SDE steps with diffusion coefficient eta, every other step is an ODE step.
    -> (sigma float64 [T], ode_mask bool [T])."""
    sde = np.zeros(T, dtype=bool)
    for i in split_steps:
        sde[i] = True
    sde |= np.asarray(window_mask).astype(bool)
    return np.where(sde, float(eta), 0.0), ~sde
