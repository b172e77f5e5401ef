"""gbt_boost_round (one iteration of the loop of Fig. 1 in one call) against the three calls it stands for and
against the CPU oracle (-m gpu).  The call shares passes between the steps (the gradient kernel finds the bounds
of the pairs, the walk that updates the margins counts the last level's rows), so everything it returns is
compared: the pairs, every array of the tree, the margins."""
import numpy as np
import pytest
import torch

import synth
from gpu_util import dev, judge_on_grid, tree_kw
from test_gpu_tree import gpu_prep

pytestmark = pytest.mark.gpu

TREE_KEYS = ("feature", "bin", "default_left", "left", "right", "n_rows", "threshold", "weight", "gain", "sumG", "sumH")


@pytest.fixture(scope="module")
def ctx():
    import paper_1806_11248_amd as g
    c = g.Context(0)
    yield c
    c.close()


def _say(msg):
    print(msg, flush=True)


def _workload(cfg, n, F=None, B=None, miss=0.0, depth=None, seed=0):
    d = synth.make(cfg, n)
    X = d["X"]
    if F is not None:
        rng = np.random.default_rng(7000 + 13 * F + seed)
        X = X[:, rng.integers(0, X.shape[1], F)].copy()
        X += rng.normal(0, 0.01, X.shape).astype(np.float32)
        if miss > 0:
            X[rng.random(X.shape) < miss] = np.nan
    p = dict(d["params"])
    if B is not None:
        p["max_bins"] = B
    if depth is not None:
        p["max_depth"] = depth
    # (workload 1 brings pairs instead of labels: its g serves as the labels of a squared-error model)
    return dict(X=X, y=d["y"] if d.get("y") is not None else d["g"], params=p)


# (config, rows, features, bins, missing, depth, rounds): byte symbols of at most 16 features take the walk that
# counts (grow paths 2 and, with the fused pass switched off, 1); other shapes take the plain walks
CASES = [
    (4, 150_001, None, None, 0.0, 8, 3),      # the 115M-row workload's shape: 13 byte symbols
    (4, 70_001, 16, 256, 0.1, 6, 2),          # a missing symbol, 16 features
    (4, 20_000, 5, 200, 0.0, 9, 2),           # deeper than the rows support everywhere: empty and unsplit nodes
    (4, 60_000, 13, 256, 0.0, 10, 1),         # the deepest tree whose nodes the counting walk holds in LDS (2047)
    (4, 60_000, 8, 256, 0.05, 11, 1),         # one level more: the leaves are counted by a pass of their own again
    (4, 9_000, 13, 256, 0.0, 1, 2),           # the root's children are the last level
    (4, 9_000, 13, 256, 0.0, 0, 1),           # no split at all
    (2, 50_000, None, None, 0.0, 6, 3),       # 28 byte symbols: rows of 7 words (path 1, plain walk)
    (3, 40_000, None, None, 0.0, 5, 2),       # 9-bit symbols, 80% missing, squared error
    (1, 10_000, None, None, 0.0, 3, 1),       # 4-bit symbols
]


@pytest.mark.parametrize("cfg,n,F,B,miss,depth,rounds", CASES)
def test_boost_round_equals_the_three_calls(ctx, oracle, cfg, n, F, B, miss, depth, rounds):
    import paper_1806_11248_amd as g
    d = _workload(cfg, n, F, B, miss, depth)
    p = d["params"]
    n, F = d["X"].shape
    objective = "squared" if p["objective"] == "given" else p["objective"]
    y = d["y"]
    o, gdev = gpu_prep(ctx, oracle, d)
    params = g.make_params(max_depth=p["max_depth"], max_bins=p["max_bins"], lam=p["lam"], gamma=p["gamma"],
                           min_child_weight=p["min_child_weight"], eta=p["eta"], objective=objective)
    y_t = dev(np.asarray(y, np.float32))
    m_a = torch.zeros(n, dtype=torch.float32, device="cuda")       # the three calls
    m_b = torch.zeros(n, dtype=torch.float32, device="cuda")       # one call, in place
    m_c_in = torch.zeros(n, dtype=torch.float32, device="cuda")    # one call, into another array
    m_ref = np.zeros(n, np.float32)
    gp_b = torch.empty((n, 2), dtype=torch.float32, device="cuda")
    gp_c = torch.empty((n, 2), dtype=torch.float32, device="cuda")
    for r in range(rounds):
        _say(f"boost round C{cfg} n={n} F={F} bits={gdev['bits']} depth={p['max_depth']} round {r}")
        gp_a = ctx.gradients(objective, m_a, y_t)
        tree_a, _, _ = ctx.grow_tree(gdev["packed"], gdev["bits"], n, F, gdev["missing"], gdev["nb"], gdev["cuts"], gp_a,
                                     params, want_rows=False, want_leaf=False)
        ctx.predict([tree_a], m_a, p["eta"], packed=gdev["packed"], bits=gdev["bits"], missing_sym=gdev["missing"], n=n, F=F)
        tree_b = ctx.boost_round(gdev["packed"], gdev["bits"], n, F, gdev["missing"], gdev["nb"], gdev["cuts"], y_t,
                                 m_b, m_b, gp_b, params)
        m_c_out = torch.full((n,), 7.0, dtype=torch.float32, device="cuda")
        tree_c = ctx.boost_round(gdev["packed"], gdev["bits"], n, F, gdev["missing"], gdev["nb"], gdev["cuts"], y_t,
                                 m_c_in, m_c_out, gp_c, params)
        torch.cuda.synchronize()
        for name, t in (("in place", tree_b), ("other array", tree_c)):
            assert t["n_nodes"] == tree_a["n_nodes"], name
            nn = t["n_nodes"]
            for k in TREE_KEYS:
                assert np.array_equal(t[k][:nn], tree_a[k][:nn]), (name, k)
        assert torch.equal(gp_b, gp_a) and torch.equal(gp_c, gp_a)
        assert torch.equal(m_b, m_a) and torch.equal(m_c_out, m_a)
        m_c_in = m_c_out
        # ... and against the oracle: the pairs, the tree on those pairs (judged in the kernel's precision),
        # the row counts of every node, the margins
        gp_ref = oracle.gradients(objective, m_ref, np.asarray(y, np.float32))
        gp_host = gp_b.cpu().numpy()
        assert np.allclose(gp_host, gp_ref, rtol=1e-5, atol=1e-6)
        _, scale = ctx.gpair_fixed(gp_b)
        rep = judge_on_grid(oracle, oracle.replay_tree, tree_b, o, gp_host, scale, **tree_kw(p))
        nn = tree_b["n_nodes"]
        leaf = rep["leaf_of_row"]
        # rows per node from the judge's leaves, summed up the tree
        cnt = np.zeros(nn, np.int64)
        np.add.at(cnt, leaf, 1)
        for i in range(nn - 1, -1, -1):
            if tree_b["feature"][i] >= 0:
                cnt[i] = cnt[tree_b["left"][i]] + cnt[tree_b["right"][i]]
        assert np.array_equal(tree_b["n_rows"][:nn], cnt)
        m_ref = oracle.predict_sym(tree_b, o["sym"], o["missing"], p["eta"], m_ref)
        assert np.allclose(m_b.cpu().numpy(), m_ref, rtol=1e-5, atol=1e-6)


def test_boost_round_argument_errors(ctx):
    import paper_1806_11248_amd as g
    d = _workload(4, 5_000)
    n, F = d["X"].shape
    cuts, nb, sym, mv, ms = ctx.quantise(dev(d["X"]), max_bins=256)
    packed, bits = ctx.compress(sym, mv)
    y = dev(d["y"])
    m = torch.zeros(n, dtype=torch.float32, device="cuda")
    gp = torch.empty((n, 2), dtype=torch.float32, device="cuda")
    bad = g.make_params(max_depth=3, max_bins=256, objective="logistic")
    bad.objective = 9
    with pytest.raises(g.GbtError):
        ctx.boost_round(packed, bits, n, F, ms, nb, cuts, y, m, m, gp, bad)
    ok = g.make_params(max_depth=3, max_bins=256, objective="logistic")
    with pytest.raises(g.GbtError):   # NaN margins give non-finite pairs: refused like gbt_gpair_fixed refuses them
        ctx.boost_round(packed, bits, n, F, ms, nb, cuts, y, torch.full_like(m, float("nan")), m, gp, ok)
    t = ctx.boost_round(packed, bits, n, F, ms, nb, cuts, y, torch.zeros_like(m), m, gp, ok)
    assert t["n_nodes"] >= 1
