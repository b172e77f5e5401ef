"""Pins for the oracle's tree growth, prediction, boosting loop and replay judge
(paper Alg. 1, Sec. 2.3, 2.4, Fig. 1)."""
import copy

import numpy as np
import pytest

import synth


def _prep(oracle, X, B):
    cuts, nb = oracle.cuts(X, B)
    sym, missing, mx = oracle.bin_matrix(X, cuts, nb)
    return cuts, nb, sym, missing


def _kw(p):
    return dict(max_depth=p["max_depth"], max_bins=p["max_bins"], lam=p["lam"], gamma=p["gamma"],
                min_child_weight=p["min_child_weight"])


@pytest.fixture(scope="module")
def c1(oracle):
    d = synth.make(1)
    cuts, nb, sym, missing = _prep(oracle, d["X"], 16)
    gp = np.stack([d["g"], d["h"]], 1)
    t, rows, leaf = oracle.grow_tree(sym, nb, cuts, missing, gp, **_kw(d["params"]))
    return d, cuts, nb, sym, missing, gp, t, rows, leaf


def test_tree_invariants(oracle, c1):
    d, cuts, nb, sym, missing, gp, t, rows, leaf = c1
    n = sym.shape[0]
    nn = t["n_nodes"]
    assert nn == 15                       # depth 3 on 10,000 informative-free rows: full tree
    assert np.array_equal(np.sort(rows), np.arange(n))        # every row exactly once
    is_leaf = t["feature"][:nn] < 0
    leaves = np.flatnonzero(is_leaf)
    assert np.array_equal(np.bincount(leaf, minlength=nn)[leaves], t["n_rows"][leaves])
    assert t["n_rows"][leaves].sum() == n
    # conservation: leaves' (G, H) add up to the root's; children add up to the parent
    assert np.isclose(t["sumG"][leaves].sum(), t["sumG"][0], rtol=1e-10, atol=1e-9)
    assert np.isclose(t["sumH"][leaves].sum(), t["sumH"][0], rtol=1e-12)
    for i in np.flatnonzero(~is_leaf):
        l, r = t["left"][i], t["right"][i]
        assert (l, r) == (t["left"][i], t["left"][i] + 1)
        assert t["n_rows"][l] + t["n_rows"][r] == t["n_rows"][i]
        assert np.isclose(t["sumG"][l] + t["sumG"][r], t["sumG"][i], rtol=1e-10, atol=1e-9)
        assert t["depth"][l] == t["depth"][i] + 1 <= 3
        assert t["gain"][i] > 1e-6
    # breadth-first numbering: depth never decreases with the node id
    assert np.all(np.diff(t["depth"][:nn]) >= 0)
    # leaf weight = -G/(H+lambda)
    assert np.allclose(t["weight"][:nn], -t["sumG"][:nn] / (t["sumH"][:nn] + 1.0), rtol=1e-15)
    # row order: each leaf's rows contiguous and ascending, leaves left to right
    pos = 0
    def walk(i):
        nonlocal pos
        if t["feature"][i] < 0:
            seg = rows[pos: pos + t["n_rows"][i]]
            assert np.all(leaf[seg] == i) and np.all(np.diff(seg.astype(np.int64)) > 0)
            pos += t["n_rows"][i]
        else:
            walk(t["left"][i]); walk(t["right"][i])
    walk(0)
    assert pos == n


def test_predict_agrees_with_partition_and_raw_floats(oracle, c1):
    d, cuts, nb, sym, missing, gp, t, rows, leaf = c1
    n = sym.shape[0]
    m0 = np.zeros(n, np.float32)
    m_sym, leaf_sym = oracle.predict_sym(t, sym, missing, 0.3, m0, want_leaf=True)
    m_raw, leaf_raw = oracle.predict_raw(t, d["X"], 0.3, m0, want_leaf=True)
    assert np.array_equal(leaf_sym, leaf) and np.array_equal(leaf_raw, leaf)
    assert np.array_equal(m_sym, m_raw)
    assert np.allclose(m_sym, (0.3 * t["weight"][leaf]).astype(np.float32), rtol=1e-7)
    # thresholds are the cuts to the right of the chosen bin
    for i in range(t["n_nodes"]):
        if t["feature"][i] >= 0:
            assert t["threshold"][i] == cuts[t["feature"][i], t["bin"][i]]


def test_depth1_generating_tree_is_recovered(oracle):
    rng = np.random.default_rng(3)
    n, F, B = 5000, 6, 32
    X = rng.random((n, F)).astype(np.float32)
    cuts, nb, sym, missing = _prep(oracle, X, B)
    f_true, b_true = 4, 13
    y = np.where(sym[:, f_true] <= b_true, -2.0, 3.0)
    gp = np.stack([0.0 - y, np.ones(n)], 1).astype(np.float32)      # squared error at margin 0
    t, rows, leaf = oracle.grow_tree(sym, nb, cuts, missing, gp, max_depth=1, max_bins=B, lam=0.0)
    assert (t["feature"][0], t["bin"][0]) == (f_true, b_true)
    assert np.isclose(t["weight"][1], -2.0) and np.isclose(t["weight"][2], 3.0)
    # a second level finds nothing: the children are pure
    t2, _, _ = oracle.grow_tree(sym, nb, cuts, missing, gp, max_depth=3, max_bins=B, lam=0.0)
    assert t2["n_nodes"] == 3


def test_gamma_and_depth_limits(oracle, c1):
    d, cuts, nb, sym, missing, gp, t, rows, leaf = c1
    kw = _kw(d["params"])
    kw["gamma"] = float(t["gain"][0]) * 1.01          # nothing beats gamma: a single leaf
    t1, rows1, leaf1 = oracle.grow_tree(sym, nb, cuts, missing, gp, **kw)
    assert t1["n_nodes"] == 1 and np.all(leaf1 == 0) and np.array_equal(rows1, np.arange(len(rows1)))
    kw = _kw(d["params"]); kw["max_depth"] = 0
    assert oracle.grow_tree(sym, nb, cuts, missing, gp, **kw)[0]["n_nodes"] == 1


def test_boosting_mse_never_increases(oracle):
    d = synth.make(5, 3000, F=40)
    p = d["params"]
    cuts, nb, sym, missing = _prep(oracle, d["X"], p["max_bins"])
    y = d["y"]
    prev = float(np.mean((0.0 - y.astype(np.float64)) ** 2))
    margin = np.zeros(len(y), np.float32)
    for _ in range(4):
        gp = oracle.gradients("squared", margin, y)
        t, _, _ = oracle.grow_tree(sym, nb, cuts, missing, gp, max_depth=3, max_bins=p["max_bins"])
        margin = oracle.predict_sym(t, sym, missing, 0.5, margin)
        mse = float(np.mean((margin.astype(np.float64) - y) ** 2))
        assert mse <= prev * (1 + 1e-6)
        prev = mse
    trees, m2 = oracle.boost(sym, nb, cuts, missing, y, objective="squared", rounds=4, eta=0.5,
                             max_depth=3, max_bins=p["max_bins"])
    assert len(trees) == 4 and np.array_equal(m2, margin)


def test_sparse_workload_learns_default_directions(oracle):
    d = synth.make(3, 20000)
    p = d["params"]
    cuts, nb, sym, missing = _prep(oracle, d["X"], p["max_bins"])
    assert missing == nb.max() and (sym == missing).mean() > 0.75
    indptr, indices, values = synth.dense_to_csr(d["X"])
    assert indptr[-1] == len(values) == (~np.isnan(d["X"])).sum()
    gp = oracle.gradients("squared", np.zeros(len(d["y"]), np.float32), d["y"])
    t, rows, leaf = oracle.grow_tree(sym, nb, cuts, missing, gp, max_depth=4, max_bins=p["max_bins"])
    nn = t["n_nodes"]
    assert nn > 7 and t["default_left"][:nn].max() == 1       # some split sends missing rows left
    m_sym, l1 = oracle.predict_sym(t, sym, missing, 1.0, np.zeros(len(leaf), np.float32), True)
    m_raw, l2 = oracle.predict_raw(t, d["X"], 1.0, np.zeros(len(leaf), np.float32), True)
    assert np.array_equal(l1, leaf) and np.array_equal(l2, leaf)


def test_judges_weight_tolerance_is_the_worst_corner(oracle):
    # G and H each off by at most a: the leaf weight -G/(H+lambda) moves furthest at one of the four corners
    # (the map is monotone in each argument while H+lambda stays positive), and the bound equals that corner
    rng = np.random.default_rng(11)
    for _ in range(200):
        G, H, lam = rng.standard_normal() * 10.0 ** rng.uniform(-2, 4), 10.0 ** rng.uniform(-3, 3), float(rng.choice([0.0, 1.0]))
        a = (H + lam) * 10.0 ** rng.uniform(-8, -0.1)
        w = -G / (H + lam)
        worst = max(abs(-(G + dg) / (H + lam + dh) - w) for dg in (-a, a) for dh in (-a, a))
        assert np.isclose(oracle._weight_atol(w, H + lam, a), worst, rtol=1e-9)
    assert oracle._weight_atol(-3.0, 2.0, 0.0) == 0.0 and oracle._weight_atol(-3.0, 2.0, 2.0) == np.inf
    assert oracle._weight_atol(0.0, 0.0, 0.0) == 0.0


def test_leaf_weight_minimises_the_quadratic_and_is_zero_without_curvature(oracle):
    # w = argmin G*w + (H + lambda)*w^2/2: no nearby w does better; and the defined value where no minimiser exists
    rng = np.random.default_rng(12)
    for _ in range(100):
        G, H, lam = float(rng.standard_normal() * 50), float(rng.uniform(0, 9)), float(rng.choice([0.0, 1.0, 4.0]))
        if H + lam == 0.0:
            continue
        w = oracle.leaf_weight(G, H, lam)
        loss = lambda x: G * x + (H + lam) * x * x / 2
        assert loss(w) <= min(loss(w * (1 + 1e-4) + 1e-6), loss(w * (1 - 1e-4) - 1e-6))
        assert np.isclose(loss(w), -G * G / (H + lam) / 2)          # the gain formula's term, halved
    assert oracle.leaf_weight(3.0, 0.0, 0.0) == 0.0 and oracle.leaf_weight(0.0, 0.0, 0.0) == 0.0
    # a node without any hessian mass under lambda = 0: one leaf, weight 0, and nothing divides by zero
    sym = np.array([[0], [1], [1], [2]], np.uint16)
    gp = np.array([[1, 0], [-2, 0], [0.5, 0], [3, 0]], np.float32)
    cuts = np.array([[1.0, 2.0]], np.float32)
    t, rows, leaf = oracle.grow_tree(sym, np.array([3], np.int32), cuts, 3, gp, max_depth=3, max_bins=3, lam=0.0,
                                     gamma=0.0, min_child_weight=0.0)
    assert t["n_nodes"] == 1 and t["weight"][0] == 0.0 and t["sumG"][0] == 2.5 and not leaf.any()


def test_replay_accepts_own_tree_and_rejects_planted_mistakes(oracle, c1):
    d, cuts, nb, sym, missing, gp, t, rows, leaf = c1
    kw = _kw(d["params"])
    rep = oracle.replay_tree(t, sym, nb, missing, gp, **kw)
    assert rep["ok"] and rep["identical"] and not rep["ties"]
    assert np.array_equal(rep["row_idx"], rows) and np.array_equal(rep["leaf_of_row"], leaf)
    # a worse split at the root
    bad = copy.deepcopy(t)
    bad["bin"][0] = (bad["bin"][0] + 3) % nb[bad["feature"][0]]
    assert not oracle.replay_tree(bad, sym, nb, missing, gp, **kw)["ok"]
    # a wrong total
    bad = copy.deepcopy(t); bad["sumH"][3] *= 1.0001
    assert not oracle.replay_tree(bad, sym, nb, missing, gp, **kw)["ok"]
    # a wrong leaf weight (sign dropped)
    bad = copy.deepcopy(t); bad["weight"][9] = -bad["weight"][9]
    assert not oracle.replay_tree(bad, sym, nb, missing, gp, **kw)["ok"]
    # a leaf where a split was due
    bad = copy.deepcopy(t); bad["feature"][1] = -1
    assert not oracle.replay_tree(bad, sym, nb, missing, gp, **kw)["ok"]
    # row counts
    bad = copy.deepcopy(t); bad["n_rows"][2] += 1
    assert not oracle.replay_tree(bad, sym, nb, missing, gp, **kw)["ok"]
    # a reported gain that is not the gain of the reported split (1e-4 off; the allowance is 3e-5 of the terms)
    bad = copy.deepcopy(t); bad["gain"][2] += 1e-4 * (t["sumG"][2] ** 2 / (t["sumH"][2] + kw["lam"]) + bad["gain"][2])
    rep = oracle.replay_tree(bad, sym, nb, missing, gp, **kw)
    assert not rep["ok"] and all("reported gain" in e for e in rep["errors"])
    # a tree that is consistent throughout (counts, totals, weights, partitions) but was grown blind to
    # the feature the root should split on: only the comparison of the gains can tell
    nb_blind = nb.copy(); nb_blind[int(t["feature"][0])] = 1
    blind, _, _ = oracle.grow_tree(sym, nb_blind, cuts, missing, gp, **kw)
    assert blind["feature"][0] != t["feature"][0]
    rep = oracle.replay_tree(blind, sym, nb, missing, gp, **kw)
    assert not rep["ok"] and any("vs best" in e for e in rep["errors"])
    # the same tree judged under stricter rules than it was grown with: every rule has to speak up
    split = np.flatnonzero(t["feature"][: t["n_nodes"]] >= 0)
    weakest = split[np.argmin(t["gain"][split])]
    rep = oracle.replay_tree(t, sym, nb, missing, gp, **dict(kw, gamma=float(t["gain"][weakest]) * 1.01))
    assert not rep["ok"] and any(e.startswith(f"node {weakest}: split although") for e in rep["errors"])
    rep = oracle.replay_tree(t, sym, nb, missing, gp, **dict(kw, max_depth=kw["max_depth"] - 1))
    assert not rep["ok"] and any("split at depth" in e for e in rep["errors"])
    lightest = min(float(min(t["sumH"][t["left"][k]], t["sumH"][t["right"][k]])) for k in split)
    rep = oracle.replay_tree(t, sym, nb, missing, gp, **dict(kw, min_child_weight=lightest * 1.01))
    assert not rep["ok"] and any("is not a valid candidate" in e for e in rep["errors"])
    # a consistent tree that stopped one level early: only "this leaf had a split due" can tell
    shallow, _, _ = oracle.grow_tree(sym, nb, cuts, missing, gp, **dict(kw, max_depth=kw["max_depth"] - 1))
    rep = oracle.replay_tree(shallow, sym, nb, missing, gp, **kw)
    assert not rep["ok"] and rep["errors"] and all("leaf although" in e for e in rep["errors"])
