"""Pins for the oracle's loss-guided growth (Sec. 2.3: the order in which nodes are opened can be
"closest to the root first" or "highest gain first") and for the judge that replays such a tree."""
import copy

import numpy as np
import pytest

import synth


def _prep(oracle, X, B):
    cuts, nb = oracle.cuts(X, B)
    sym, missing, mx = oracle.bin_matrix(X, cuts, nb)
    return cuts, nb, sym, missing


def _canon(leaf):
    """Leaf labels renamed to the smallest row id of each leaf: equal iff the partitions are equal."""
    first = {}
    for r, l in enumerate(leaf):
        first.setdefault(int(l), r)
    return np.array([first[int(l)] for l in leaf])


@pytest.mark.parametrize("seed,n,F,L", [(0, 400, 3, 7), (1, 900, 5, 16), (2, 250, 2, 31)])
def test_squared_error_best_first_equals_library_tree(oracle, seed, n, F, L):
    """With g = -y, h = 1, lambda = 0 the gain of a split is the drop of the children's summed squared
    error, and loss-guided growth is the textbook best-first regression tree.  On data whose every
    distinct value has its own bin (no quantisation loss) the leaves must be those of
    sklearn.tree.DecisionTreeRegressor(max_leaf_nodes=L), an independent implementation."""
    from sklearn.tree import DecisionTreeRegressor
    rng = np.random.default_rng(seed)
    X = rng.normal(size=(n, F)).astype(np.float32)
    y = (np.sin(2 * X[:, 0]) + 0.5 * X[:, 1 % F] * (X[:, 0] > 0) + 0.1 * rng.normal(size=n)).astype(np.float32)
    B = n + 1                                             # every distinct value its own bin
    cuts, nb, sym, missing = _prep(oracle, X, B)
    gp = np.stack([-y, np.ones(n, np.float32)], 1)
    t, rows, leaf = oracle.grow_tree_lossguide(sym, nb, cuts, missing, gp, max_leaves=L, max_depth=64,
                                               max_bins=B, lam=0.0, gamma=0.0, min_child_weight=1.0)
    ref = DecisionTreeRegressor(max_leaf_nodes=L, criterion="squared_error", splitter="best",
                                min_samples_leaf=1, random_state=0).fit(X.astype(np.float64), y.astype(np.float64))
    assert t["n_nodes"] == 2 * L - 1 == ref.tree_.node_count
    assert np.array_equal(_canon(leaf), _canon(ref.apply(X.astype(np.float32))))
    # leaf values: the library stores the mean of y, the oracle w = -G/H = mean of y
    nn = t["n_nodes"]
    mean_of = {int(l): float(y[leaf == l].astype(np.float64).mean()) for l in np.unique(leaf)}
    for l, m in mean_of.items():
        assert abs(t["weight"][l] - m) < 1e-9


def test_enough_leaves_gives_the_depth_wise_tree(oracle):
    """When neither the leaf budget nor anything else than max_depth stops the growth, both policies
    split exactly the same nodes; only the numbering differs."""
    d = synth.make(2, 6000)
    p = d["params"]
    cuts, nb, sym, missing = _prep(oracle, d["X"], 32)
    gp = oracle.gradients(p["objective"], np.zeros(6000, np.float32), d["y"])
    kw = dict(max_depth=4, max_bins=32, lam=1.0, gamma=0.0, min_child_weight=1.0)
    t_dw, rows_dw, leaf_dw = oracle.grow_tree(sym, nb, cuts, missing, gp, **kw)
    t_lg, rows_lg, leaf_lg = oracle.grow_tree_lossguide(sym, nb, cuts, missing, gp, max_leaves=16, **kw)
    assert t_lg["n_nodes"] == t_dw["n_nodes"]
    assert np.array_equal(_canon(leaf_lg), _canon(leaf_dw))
    assert np.array_equal(rows_lg, rows_dw)               # both keep every node's rows ascending, left run first
    # the multiset of (feature, bin, default, gain) over split nodes is the same
    key = lambda t: sorted((int(t["feature"][i]), int(t["bin"][i]), int(t["default_left"][i]), float(t["gain"][i]))
                           for i in range(t["n_nodes"]) if t["feature"][i] >= 0)
    assert key(t_lg) == key(t_dw)


def test_leaf_budget_and_order(oracle):
    d = synth.make(2, 5000)
    p = d["params"]
    cuts, nb, sym, missing = _prep(oracle, d["X"], 32)
    gp = oracle.gradients(p["objective"], np.zeros(5000, np.float32), d["y"])
    kw = dict(max_depth=6, max_bins=32, lam=1.0, gamma=0.0, min_child_weight=1.0)
    one, _, leaf1 = oracle.grow_tree_lossguide(sym, nb, cuts, missing, gp, max_leaves=1, **kw)
    assert one["n_nodes"] == 1 and not leaf1.any()
    two, _, _ = oracle.grow_tree_lossguide(sym, nb, cuts, missing, gp, max_leaves=2, **kw)
    h, cnt, G, H = oracle.hist(sym, 32, missing, None, gp)
    best = oracle.eval_split(h, cnt, nb, G, H, 5000, 1.0, 1.0)
    assert two["n_nodes"] == 3
    assert (two["feature"][0], two["bin"][0], two["default_left"][0]) == (best["feature"], best["bin"], best["default_left"])
    # growing further only appends: the first expansions of a bigger budget are those of a smaller one
    big, _, _ = oracle.grow_tree_lossguide(sym, nb, cuts, missing, gp, max_leaves=20, **kw)
    small, _, _ = oracle.grow_tree_lossguide(sym, nb, cuts, missing, gp, max_leaves=9, **kw)
    ns = small["n_nodes"]
    assert ns == 17 and big["n_nodes"] == 39
    split_s = small["feature"][:ns] >= 0
    for k in ("feature", "bin", "default_left", "left", "right"):
        assert np.array_equal(big[k][:ns][split_s], small[k][:ns][split_s]), k
    # at the moment of each expansion no open leaf had a larger gain: every expansion's gain is at
    # least the gain of every node expanded later that already existed (as a leaf) at that moment
    order = [int(np.flatnonzero(big["left"][:39] == 2 * k + 1)[0]) for k in range(19)]
    for k, node in enumerate(order):
        for later in order[k + 1:]:
            if later <= 2 * k:                             # `later` had been created before expansion k
                assert big["gain"][node] >= big["gain"][later]
    # a gamma above every gain: nothing splits; a gamma between two gains cuts the tree there
    none, _, _ = oracle.grow_tree_lossguide(sym, nb, cuts, missing, gp, max_leaves=20, **dict(kw, gamma=1e9))
    assert none["n_nodes"] == 1
    gains = np.sort(big["gain"][:39][big["feature"][:39] >= 0])
    cut, _, _ = oracle.grow_tree_lossguide(sym, nb, cuts, missing, gp, max_leaves=20, **dict(kw, gamma=float(gains[9])))
    assert all(cut["gain"][i] > gains[9] for i in range(cut["n_nodes"]) if cut["feature"][i] >= 0)


def test_equal_gains_expand_the_smaller_id_first(oracle):
    """Two mirror-image halves: after the root split both children have the same best gain."""
    x = np.array([0, 1, 2, 3, 10, 11, 12, 13], np.float32)[:, None]
    y = np.array([0, 0, 1, 1, 5, 5, 6, 6], np.float32)
    cuts, nb, sym, missing = _prep(oracle, x, 16)
    gp = np.stack([-y, np.ones(8, np.float32)], 1)
    t, rows, leaf = oracle.grow_tree_lossguide(sym, nb, cuts, missing, gp, max_leaves=3, max_depth=8, max_bins=16,
                                               lam=0.0, min_child_weight=1.0)
    assert t["n_nodes"] == 5
    assert t["gain"][0] == pytest.approx(2 * 8 * 2.5 ** 2 / 2 * 1.0, rel=1e-12)   # 4*0.5^2 + 4*5.5^2 - 8*3^2 = 50
    assert t["feature"][1] == 0 and t["feature"][2] == -1      # node 1 (left, smaller id) was expanded, node 2 not
    assert t["gain"][1] == pytest.approx(1.0, rel=1e-12)       # 2*0 + 2*1 - 4*0.25


def test_replay_judge_accepts_and_rejects(oracle):
    d = synth.make(2, 4000)
    p = d["params"]
    cuts, nb, sym, missing = _prep(oracle, d["X"], 32)
    gp = oracle.gradients(p["objective"], np.zeros(4000, np.float32), d["y"])
    kw = dict(max_leaves=10, max_depth=6, max_bins=32, lam=1.0, gamma=0.0, min_child_weight=1.0)
    t, rows, leaf = oracle.grow_tree_lossguide(sym, nb, cuts, missing, gp, **kw)
    rep = oracle.replay_tree_lossguide(t, sym, nb, missing, gp, **kw)
    assert rep["ok"] and rep["identical"] and not rep["errors"]
    assert np.array_equal(rep["row_idx"], rows) and np.array_equal(rep["leaf_of_row"], leaf)
    # a depth-wise tree with the same number of leaves expands low-gain nodes too early: rejected
    bad, _, _ = oracle.grow_tree(sym, nb, cuts, missing, gp, max_depth=3, max_bins=32, lam=1.0)
    assert bad["n_nodes"] == 15
    rep = oracle.replay_tree_lossguide(bad, sym, nb, missing, gp, **dict(kw, max_leaves=8))
    assert not rep["ok"] and any("expanded while" in e for e in rep["errors"])
    # stopping early with open leaves left: rejected
    short, _, _ = oracle.grow_tree_lossguide(sym, nb, cuts, missing, gp, **dict(kw, max_leaves=6))
    rep = oracle.replay_tree_lossguide(short, sym, nb, missing, gp, **kw)
    assert not rep["ok"] and any("stopped at" in e for e in rep["errors"])
    # a reported gain that is not the gain of the reported split
    t2 = copy.deepcopy(t)
    t2["gain"][1] *= 1.001
    rep = oracle.replay_tree_lossguide(t2, sym, nb, missing, gp, **kw)
    assert not rep["ok"] and all("reported gain" in e for e in rep["errors"])
    # a wrong bin, a wrong total, a wrong row count: each caught
    for field, delta, what in (("bin", 1, "gain"), ("sumG", 1.0, "sumG"), ("n_rows", 1, "n_rows")):
        t2 = copy.deepcopy(t)
        t2[field][0] += delta
        rep = oracle.replay_tree_lossguide(t2, sym, nb, missing, gp, **kw)
        assert not rep["ok"] and any(what in e for e in rep["errors"]), (field, rep["errors"][:2])
