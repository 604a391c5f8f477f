"""Pins for the oracle's pruning (Sec. 3.4)."""
import numpy as np

from oracle import prune, tree


def test_parent_top1_keeps_one_child_per_last_split_parent():
    t = tree.tree_build(6, (0, 2, 4), 2)                     # 8 leaves
    r = np.array([0.1, 0.9, 0.5, 0.4, -1.0, -1.0, 2.0, 3.0], np.float32)
    keep = prune.width_keep_leaves(t, r, 1)
    assert list(np.nonzero(keep)[0]) == [1, 2, 4, 7]         # tie (-1, -1) -> lower branch index
    assert keep.sum() == t["n_leaves"] // t["K"]             # "roughly halves" for K = 2
    t3 = tree.tree_build(4, (1, 2), 3)
    r3 = np.random.default_rng(0).standard_normal(9).astype(np.float32)
    k3 = prune.width_keep_leaves(t3, r3, 1)
    assert k3.sum() == 3 and all(k3[3 * p + np.argmax(r3[3 * p:3 * p + 3])] for p in range(3))


def test_extreme_b_hand_values():
    t = tree.tree_build(6, (0, 2, 4), 2)
    r = np.array([0.5, -2.0, 0.5, 3.0, 0.0, 0.5, -1.0, 2.5], np.float32)
    assert list(np.nonzero(prune.width_keep_leaves(t, r, 2, 2))[0]) == [1, 3, 6, 7]
    # ties among (0.5, 0.5, 0.5) are ordered by leaf index: b = 3 -> worst {1, 6, 4}, best {5, 7, 3}
    assert list(np.nonzero(prune.width_keep_leaves(t, r, 2, 3))[0]) == [1, 3, 4, 5, 6, 7]
    assert prune.width_keep_leaves(t, r, 2, 4).all() and prune.width_keep_leaves(t, r, 0).all()


def _paths_union(t, leaves):
    e = set()
    for l in leaves:
        n = t["off"][t["T"]] + l
        while t["parent"][n] >= 0:
            e.add(int(n))
            n = t["parent"][n]
    return e


def test_kept_edges_are_the_union_of_root_to_leaf_paths():
    t = tree.tree_build(7, (1, 3, 4), 2)
    rng = np.random.default_rng(1)
    C = 3
    r = rng.standard_normal(C * t["n_leaves"]).astype(np.float32)
    none = np.zeros(t["T"], np.uint8)
    for mode, b in ((0, 0), (1, 0), (2, 1), (2, 3)):
        got = prune.kept_edges(t, r, C, mode, b, none)
        exp = []
        for c in range(C):
            keep = prune.width_keep_leaves(t, r.reshape(C, -1)[c], mode, b)
            exp += sorted(c * t["n_nodes"] + n for n in _paths_union(t, np.nonzero(keep)[0]))
        assert list(got) == exp and got.dtype == np.int32
    # no pruning at all keeps every edge
    assert len(prune.kept_edges(t, r, C, 0, 0, none)) == C * t["n_edges"]
    # depth mask removes exactly the edges of the masked steps
    mask = np.zeros(t["T"], np.uint8)
    mask[[0, 5]] = 1
    got = prune.kept_edges(t, r, C, 0, 0, mask)
    assert all(t["depth"][g % t["n_nodes"]] - 1 not in (0, 5) for g in got)
    assert len(got) == C * (t["n_edges"] - t["width"][1] - t["width"][6])


def test_sliding_window_schedule():
    # Sec. 4.4: starts at the last split, size 4, moves one step every 30 iterations
    m = prune.depth_mask_window(20, 9, 4, 0, 30, 20)
    assert list(np.nonzero(m)[0]) == [9, 10, 11, 12]
    assert list(np.nonzero(prune.depth_mask_window(20, 9, 4, 29, 30, 20))[0]) == [9, 10, 11, 12]
    assert list(np.nonzero(prune.depth_mask_window(20, 9, 4, 30, 30, 20))[0]) == [10, 11, 12, 13]
    assert list(np.nonzero(prune.depth_mask_window(20, 9, 4, 300, 30, 20))[0]) == [16, 17, 18, 19]   # stops
    assert list(np.nonzero(prune.depth_mask_window(20, 9, 4, 3000, 30, 18))[0]) == [14, 15, 16, 17]


def test_seeded_depth_subset():
    m = prune.depth_mask_seeded(20, 4, 42)
    assert m.sum() == 4 and m.dtype == np.uint8
    assert np.array_equal(m, prune.depth_mask_seeded(20, 4, 42))
    assert not np.array_equal(m, prune.depth_mask_seeded(20, 4, 43))
    assert prune.depth_mask_seeded(20, 0, 42).sum() == 0 and prune.depth_mask_seeded(5, 5, 1).all()


def test_seeded_depth_subset_drops_the_smallest_words():
    # direction of the selection: every dropped step has a smaller (word, step) than every kept one;
    # the stored cases list the words and the dropped steps (tests/golden/make_depth_mask_golden.py)
    import json
    import os
    gold = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "depth_mask_seeded.json")))["cases"]
    assert len(gold) >= 5
    for g in gold:
        m = prune.depth_mask_seeded(g["T"], g["n_drop"], g["seed"])
        assert sorted(np.nonzero(m)[0].tolist()) == g["dropped"], g
        key = [(g["words"][i], i) for i in range(g["T"])]
        dropped, keptk = [key[i] for i in range(g["T"]) if m[i]], [key[i] for i in range(g["T"]) if not m[i]]
        if dropped and keptk:
            assert max(dropped) < min(keptk)
    # the image workload's mask (T = 20, 4 drops, seed 42), read off the stored words by eye: the four
    # smallest are 138049223 (step 7), 830668340 (12), 834821491 (10), 853052770 (11); the next, 1012887007, is step 3
    assert (gold[0]["T"], gold[0]["n_drop"], gold[0]["seed"]) == (20, 4, 42)
    assert gold[0]["words"][7] == 138049223 and gold[0]["words"][3] == 1012887007
    assert list(np.nonzero(prune.depth_mask_seeded(20, 4, 42))[0]) == [7, 10, 11, 12]


def test_hybrid_ode_sde_schedule():
    # ablation "Hybrid ODE-SDE": split steps stay SDE, the window adds SDE steps, the rest are ODE steps
    win = prune.depth_mask_window(20, 16, 4, 0, 30, 20)          # steps 16..19
    sigma, ode = prune.mix_schedule(20, (4, 8, 12, 16), win, 0.3)
    sde_steps = sorted(set((4, 8, 12, 16)) | {16, 17, 18, 19})
    assert list(np.nonzero(sigma)[0]) == sde_steps and np.all(sigma[sde_steps] == 0.3)
    assert list(np.nonzero(ode)[0]) == [i for i in range(20) if i not in sde_steps]
    # an empty window leaves only the split steps stochastic; a full window gives the plain SDE sampler
    sigma, ode = prune.mix_schedule(6, (1, 3), np.zeros(6, np.uint8), 0.7)
    assert list(sigma) == [0.0, 0.7, 0.0, 0.7, 0.0, 0.0] and list(ode) == [True, False, True, False, True, True]
    sigma, ode = prune.mix_schedule(6, (), np.ones(6, np.uint8), 0.7)
    assert np.all(sigma == 0.7) and not ode.any()
    # edges of ODE steps leave the update when the ODE mask is used as depth mask
    t = tree.tree_build(6, (1, 3), 2)
    _, ode = prune.mix_schedule(6, (1, 3), np.zeros(6, np.uint8), 0.7)
    kept = prune.kept_edges(t, np.arange(t["n_leaves"], dtype=float), 1, 0, 0, ode.astype(np.uint8))
    assert sorted(set(t["depth"][k] - 1 for k in kept)) == [1, 3]
