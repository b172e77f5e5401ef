"""GPU parity of whole trees and of the boosting loop against the CPU oracle
(-m gpu).  Every input goes through the GPU's own quantise -> compress first, and
each stage is compared with the oracle before the next one is trusted."""
import numpy as np
import pytest
import torch

import synth
from gpu_util import dev, host_u32, judge_on_grid, oracle_prep, tree_kw

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    import paper_1806_11248_amd as g
    c = g.Context(0)
    yield c
    c.close()


def _say(msg):
    print(msg, flush=True)


def gpu_prep(ctx, oracle, d, use_csr=False):
    """GPU quantise + compress of workload d, checked bit-exactly against the oracle."""
    X = d["X"]
    B = d["params"]["max_bins"]
    o = oracle_prep(oracle, X, B)
    if use_csr:
        indptr, indices, values = synth.dense_to_csr(X)
        cuts, nb, sym, mv, ms = ctx.quantise(csr=(dev(indptr), dev(indices), dev(values)), max_bins=B,
                                             n=X.shape[0], F=X.shape[1])
    else:
        cuts, nb, sym, mv, ms = ctx.quantise(dev(X), max_bins=B)
    assert np.array_equal(nb.cpu().numpy(), o["nb"])
    assert np.array_equal(cuts.cpu().numpy(), o["cuts"])
    assert (mv, ms) == (o["max_value"], o["missing"])
    packed, bits = ctx.compress(sym, mv)
    assert bits == o["bits"]
    assert np.array_equal(host_u32(packed), o["words"])
    del sym
    return o, dict(cuts=cuts, nb=nb, packed=packed, bits=bits, missing=ms)


def grow_and_judge(ctx, oracle, o, gdev, gp, p, n, F, nodes=None, grid_only=False):
    import paper_1806_11248_amd as g
    params = g.make_params(max_depth=p["max_depth"], max_bins=p["max_bins"], lam=p["lam"], gamma=p["gamma"],
                           min_child_weight=p["min_child_weight"])
    gp_t = dev(gp)
    tree, row_idx, leaf = ctx.grow_tree(gdev["packed"], gdev["bits"], n, F, gdev["missing"], gdev["nb"],
                                        gdev["cuts"], gp_t, params)
    _, scale = ctx.gpair_fixed(gp_t)
    rep = judge_on_grid(oracle, oracle.replay_tree, tree, o, gp, scale, **tree_kw(p), nodes=nodes)
    if not grid_only:   # and against the unrounded pairs, within the stated bound of one rounding per row
        rep = oracle.replay_tree(tree, o["sym"], o["nb"], o["missing"], gp, **tree_kw(p),
                                 sum_atol_per_row=0.5 / min(scale), nodes=nodes)
        assert rep["ok"], rep["errors"][:5]
    assert np.array_equal(host_u32(row_idx), rep["row_idx"])           # partitions: bit-exact
    assert np.array_equal(leaf.cpu().numpy(), rep["leaf_of_row"])
    nn = tree["n_nodes"]
    for i in range(nn):                                                  # thresholds are the cuts
        if tree["feature"][i] >= 0:
            f, b = tree["feature"][i], tree["bin"][i]
            want = o["cuts"][f, b] if b < p["max_bins"] - 1 else np.inf
            assert tree["threshold"][i] == want
    rep["scale"] = scale
    # the same tree when row ids are not carried along
    bare, none_rows, leaf2 = ctx.grow_tree(gdev["packed"], gdev["bits"], n, F, gdev["missing"], gdev["nb"],
                                           gdev["cuts"], gp_t, params, want_rows=False)
    assert none_rows is None and bare["n_nodes"] == nn
    assert np.array_equal(leaf2.cpu().numpy(), rep["leaf_of_row"])    # leaf ids from a walk of the finished tree
    only_tree = ctx.grow_tree(gdev["packed"], gdev["bits"], n, F, gdev["missing"], gdev["nb"], gdev["cuts"], gp_t,
                              params, want_rows=False, want_leaf=False)
    assert only_tree[1] is None and only_tree[2] is None and only_tree[0]["n_nodes"] == nn
    for k in ("feature", "bin", "default_left", "left", "right", "n_rows", "threshold", "weight", "gain",
              "sumG", "sumH"):
        assert np.array_equal(bare[k][:nn], tree[k][:nn]), k
    return tree, rep


CASES = [  # config, rows, kwargs, csr
    (1, None, {}, False),                 # the tiny workload at its full size: 10,000 x 8, 4-bit, depth 3
    (2, 60_000, {}, False),               # 8-bit, 28 features, depth 6
    (3, 60_000, {}, True),                # 9-bit with missing values, CSR input, depth 8
    (4, 200_000, {}, False),              # 8-bit, 13 features (skewed categorical columns), depth 8
    (5, 6_000, {"F": 300}, False),        # 6-bit, wide, depth 10: many small nodes, feature tiles
    (5, 4_000, {"F": 500}, False),        # rows of 375 bytes: the row-parallel histogram kernel
]


@pytest.mark.parametrize("cfg,n,kw,csr", CASES)
def test_tree_matches_oracle(ctx, oracle, cfg, n, kw, csr):
    d = synth.make(cfg, n, **kw)
    p = d["params"]
    X = d["X"]
    n, F = X.shape
    _say(f"tree C{cfg} n={n} F={F} depth={p['max_depth']}")
    o, gdev = gpu_prep(ctx, oracle, d, use_csr=csr)
    wide = F * gdev["bits"] > 8 * 32       # such rows are not moved: id lists are partitioned instead
    assert (ctx.grow_tree_path(F, gdev["bits"], p["max_bins"], track_rows=True) == 3) == wide
    if p["objective"] == "given":
        gp = np.stack([d["g"], d["h"]], 1)
    else:
        gp = oracle.gradients(p["objective"], np.zeros(n, np.float32), d["y"])
        gp_gpu = ctx.gradients(p["objective"], dev(np.zeros(n, np.float32)), dev(d["y"])).cpu().numpy()
        assert np.allclose(gp_gpu, gp, rtol=1e-6, atol=1e-7)
    tree, rep = grow_and_judge(ctx, oracle, o, gdev, gp, p, n, F)
    # an independently grown oracle tree has the same structure unless a legal tie intervened
    t_ref, rows_ref, leaf_ref = oracle.grow_tree(o["sym"], o["nb"], o["cuts"], o["missing"], gp, **tree_kw(p))
    if rep["identical"]:
        nn = t_ref["n_nodes"]
        assert tree["n_nodes"] == nn
        for k in ("feature", "bin", "default_left", "left", "right", "n_rows"):
            assert np.array_equal(tree[k][:nn], t_ref[k][:nn]), k
        # leaf weights: 1e-5 relative, plus the fixed-point rounding bound of the node's rows
        w_atol = 2.0 * t_ref["n_rows"][:nn] * (0.5 / min(rep["scale"])) / (t_ref["sumH"][:nn] + p["lam"])
        assert np.all(np.abs(tree["weight"][:nn] - t_ref["weight"][:nn])
                      <= 1e-5 * np.abs(t_ref["weight"][:nn]) + w_atol + 1e-12)
        assert np.allclose(tree["gain"][:nn], t_ref["gain"][:nn], rtol=1e-5, atol=1e-7)
    _say(f"  nodes={tree['n_nodes']} identical={rep['identical']} ties={len(rep['ties'])}")

    # prediction: packed symbols, raw floats, oracle -- same leaves, same margins
    m0 = np.zeros(n, np.float32)
    ref = oracle.predict_sym(tree, o["sym"], o["missing"], 0.3, m0)
    got_p = ctx.predict([tree], dev(m0), 0.3, packed=gdev["packed"], bits=gdev["bits"], missing_sym=gdev["missing"],
                        n=n, F=F).cpu().numpy()
    got_x = ctx.predict([tree], dev(m0), 0.3, X=dev(X)).cpu().numpy()
    assert np.array_equal(got_p, ref) and np.array_equal(got_x, ref)


@pytest.fixture()
def ctx_env(monkeypatch):
    """A context created under tuning variables (they are read when a context is created)."""
    made = []

    def make(**env):
        import paper_1806_11248_amd as g
        for k, v in env.items():
            monkeypatch.setenv(k, str(v))
        c = g.Context(0)
        made.append(c)
        return c
    yield make
    for c in made:
        c.close()


@pytest.mark.parametrize("cfg,n,kw", [(4, 150_000, {}), (3, 40_000, {}), (5, 5_000, {"F": 200}), (5, 4_000, {"F": 500})])
def test_three_launch_partition_path(ctx_env, oracle, cfg, n, kw):
    """The record partition normally takes its one-launch form (rows wider than 8 words: only ids
    move); switched off, the flag / scan / move form that carries whole records must grow the same trees."""
    c = ctx_env(GBT_TUNE_PART_FUSED=0, GBT_TUNE_PART_IDS=0, GBT_TUNE_HIST_FIX=0)   # and the separate fixed-point conversion pass
    d = synth.make(cfg, n, **kw)
    p = d["params"]
    n, F = d["X"].shape
    _say(f"three-launch partition C{cfg} n={n} F={F}")
    o, gdev = gpu_prep(c, oracle, d)
    assert c.grow_tree_path(F, gdev["bits"], p["max_bins"], track_rows=True) == 0
    gp = (np.stack([d["g"], d["h"]], 1) if p["objective"] == "given"
          else oracle.gradients(p["objective"], np.zeros(n, np.float32), d["y"]))
    grow_and_judge(c, oracle, o, gdev, gp, p, n, F)


@pytest.mark.parametrize("F,B,miss", [(1, 256, 0.0), (3, 256, 0.0), (4, 256, 0.0), (7, 256, 0.0), (8, 200, 0.1),
                                      (11, 256, 0.0), (12, 128, 0.3), (13, 256, 0.0), (14, 255, 0.05),
                                      (16, 256, 0.0)])
def test_byte_symbols_up_to_16_features(ctx, oracle, F, B, miss):
    """8-bit rows of one to four words: without row ids the partition pass also builds one child's
    histogram; the trees must equal the tracked ones (separate kernels) and the oracle's."""
    n = 70_001
    d = synth.make(4, n)
    rng = np.random.default_rng(1000 * F + B)
    X = d["X"][:, rng.integers(0, d["X"].shape[1], F)].copy()
    X += rng.normal(0, 0.01, X.shape).astype(np.float32)      # columns drawn twice differ a little
    if miss > 0:
        X[rng.random(X.shape) < miss] = np.nan
    p = dict(d["params"], max_bins=B, max_depth=6)
    dd = dict(X=X, params=p)
    _say(f"byte symbols F={F} B={B} missing={miss}")
    o, gdev = gpu_prep(ctx, oracle, dd)
    assert gdev["bits"] == 8
    gp = oracle.gradients(p["objective"], np.zeros(n, np.float32), d["y"])
    grow_and_judge(ctx, oracle, o, gdev, gp, p, n, F)


@pytest.mark.parametrize("F,n,kind", [(1, 5_000, "general"), (4, 70_001, "uniform"), (5, 70_001, "general"), (8, 3_001, "tiny"),
                                      (9, 70_001, "general"), (12, 70_001, "tiny-uniform"), (13, 2_300_003, "general"),
                                      (13, 70_001, "huge"), (14, 70_001, "general"), (16, 2_300_003, "uniform"),
                                      (16, 40_000, "general"), (13, 200, "general"), (7, 300, "uniform")])
def test_root_histogram_forms(ctx, oracle, F, n, kind):
    """The root's histogram kernel for byte symbols: every slot class (1..16 features), pairs with one common
    hessian (count word, no tests) and without (packed word with carry / wrap bookkeeping), fp32 pairs rounded
    in fp32 and, where the scales leave the range in which that is exact, through fp64; inputs short enough
    for one workgroup and long enough for unequal slices per compute unit.  Judged through the tree: the
    root's totals, its split and the gains reported come from that histogram."""
    d = synth.make(4, max(n, 400))
    rng = np.random.default_rng(31 * F + n % 1000)
    X = d["X"][:n, rng.integers(0, d["X"].shape[1], F)].copy()
    X += rng.normal(0, 0.01, X.shape).astype(np.float32)
    p = dict(d["params"], max_bins=256, max_depth=2, min_child_weight=0.0 if "tiny" in kind else 1.0)
    o, gdev = gpu_prep(ctx, oracle, dict(X=X, params=p))
    g_ = rng.standard_normal(n) + (X[:, 0] > np.median(X[:, 0])) * 0.7
    h_ = np.ones(n) if "uniform" in kind else rng.uniform(0.05, 1.0, n)
    mag = {"tiny": 2.0 ** -100, "tiny-uniform": 2.0 ** -100, "huge": 2.0 ** 90}.get(kind, 1.0)
    gp = np.stack([g_ * mag, h_ * mag], 1).astype(np.float32)
    _say(f"root histogram forms: F={F} n={n} {kind} bits={gdev['bits']}")
    if p["min_child_weight"] == 0.0:
        p["lam"] = float(mag)
    grow_and_judge(ctx, oracle, o, gdev, gp, p, n, F, grid_only=True)


@pytest.mark.parametrize("F", [13, 16, 5])
def test_pass_with_carries_and_wraps_everywhere(ctx, ctx_env, oracle, F):
    """Extreme same-sign pairs piled into few bins: in the partition + histogram pass the packed LDS
    words carry and wrap every few hundred adds.  The tree must equal, to the last bit of every sum,
    the one grown through the separate histogram kernels on row lists."""
    import paper_1806_11248_amd as g
    n, B = 1_200_007, 256
    rng = np.random.default_rng(40 + F)
    sym = np.zeros((n, F), np.uint16)
    sym[:, 0] = rng.integers(0, 3, n)                       # three heavy bins
    sym[:, 1] = (np.arange(n) // 7) % B
    for f in range(2, F):
        sym[:, f] = rng.integers(0, 1 + f, n) * (B // (1 + f))
    run = (np.arange(n) // 50_000) % 2 == 0                 # long runs of one sign, then the other
    gmag = np.where(rng.random(n) < 0.5, 1.999, 1.3).astype(np.float32)
    gp = np.stack([np.where(run, gmag, -gmag), np.where(rng.random(n) < 0.7, 1.999, 0.9)], 1).astype(np.float32)
    gp[:, 0] += (sym[:, 0] == 1) * np.float32(0.5)          # something to split on
    nb = np.full(F, B, np.int32)
    cuts = np.tile(np.arange(1, B, dtype=np.float32), (F, 1))
    packed = dev(oracle.pack(sym, 8).view(np.int32))
    params = g.make_params(max_depth=4, max_bins=B)
    _say(f"carries and wraps in the pass, F={F}")
    assert ctx.grow_tree_path(F, 8, B, track_rows=False) == 2
    tree, _, leaf = ctx.grow_tree(packed, 8, n, F, B, dev(nb), dev(cuts), dev(gp), params, want_rows=False)
    other = ctx_env(GBT_TUNE_PART_HIST=0, GBT_TUNE_PART_FUSED=0, GBT_TUNE_ORDER_ROWS=0)
    assert other.grow_tree_path(F, 8, B, track_rows=True) == 0
    ref, _, leaf_ref = other.grow_tree(packed, 8, n, F, B, dev(nb), dev(cuts), dev(gp), params)
    nn = tree["n_nodes"]
    assert nn > 3 and ref["n_nodes"] == nn
    for k in ("feature", "bin", "default_left", "left", "right", "n_rows", "weight", "gain", "sumG", "sumH"):
        assert np.array_equal(ref[k][:nn], tree[k][:nn]), k
    assert torch.equal(leaf, leaf_ref)
    # and the root's sums against plain fp64 arithmetic on the fixed-point pairs
    gq, scale = ctx.gpair_fixed(dev(gp))
    q = gq.cpu().numpy().astype(np.int64)
    assert tree["sumG"][0] == q[:, 0].sum() / scale[0] and tree["sumH"][0] == q[:, 1].sum() / scale[1]


@pytest.mark.parametrize("F,B,miss", [(16, 200, 0.05), (6, 256, 0.0)])
def test_byte_symbols_many_tiles(ctx, oracle, F, B, miss):
    """The partition + histogram pass over millions of rows: spans of several tiles, cursors handed
    out to hundreds of workgroups, the slot classes other than the 13-feature one."""
    n = 2_500_003
    d = synth.make(4, n)
    rng = np.random.default_rng(77 + F)
    X = d["X"][:, rng.integers(0, d["X"].shape[1], F)].copy()
    X += rng.normal(0, 0.01, X.shape).astype(np.float32)
    if miss > 0:
        X[rng.random(X.shape) < miss] = np.nan
    p = dict(d["params"], max_bins=B, max_depth=5)
    _say(f"byte symbols, many tiles: n={n} F={F} B={B} missing={miss}")
    o, gdev = gpu_prep(ctx, oracle, dict(X=X, params=p))
    assert gdev["bits"] == 8 and ctx.grow_tree_path(F, 8, B, track_rows=False) == 2
    gp = oracle.gradients(p["objective"], np.zeros(n, np.float32), d["y"])
    grow_and_judge(ctx, oracle, o, gdev, gp, p, n, F, nodes={0, 1, 2, 5, 12, 20, 31, 40})


def test_depth_zero_and_gamma(ctx, oracle):
    d = synth.make(1)
    p = dict(d["params"])
    n, F = d["X"].shape
    o, gdev = gpu_prep(ctx, oracle, d)
    gp = np.stack([d["g"], d["h"]], 1)
    for change in (dict(max_depth=0), dict(gamma=1e9), dict(min_child_weight=1e9)):
        q = dict(p); q.update(change)
        _say(f"degenerate tree {change}")
        tree, rep = grow_and_judge(ctx, oracle, o, gdev, gp, q, n, F)
        assert tree["n_nodes"] == 1 and tree["feature"][0] == -1


@pytest.mark.parametrize("cfg,n,kw", [(4, 60_000, {}), (5, 7_000, {"F": 40})])
def test_a_few_huge_pairs_set_the_fixed_point_scale(ctx, oracle, cfg, n, kw):
    # One row in a thousand carries pairs a thousand times the rest and half the hessians are zero: the largest pair
    # fixes the quantum, the ordinary rows keep about 16 of their bits, and leaves with |weight| far above 1
    # appear.  Sums stay within half a quantum per row; the weights within what that bound implies.
    d = synth.make(cfg, n, **kw)
    p = dict(d["params"], max_depth=6, lam=1.0, gamma=0.0, min_child_weight=3.3)
    n, F = d["X"].shape
    rng = np.random.default_rng(n)
    gp = np.stack([rng.standard_normal(n) * 400.0, np.where(rng.random(n) < 0.5, 0.0, rng.uniform(0, 1, n) * 2.5)], 1)
    gp[rng.integers(0, n, n // 1000)] *= 1000.0
    gp = gp.astype(np.float32)
    o, gdev = gpu_prep(ctx, oracle, d)
    _say(f"huge pairs: config {cfg}, {n} x {F}")
    tree, rep = grow_and_judge(ctx, oracle, o, gdev, gp, p, n, F)
    nn = tree["n_nodes"]
    assert nn > 15 and np.abs(tree["weight"][:nn]).max() > 50.0


def test_boosting_rounds_in_lock_step(ctx, oracle):
    """Each round: the GPU's gradients are checked against the oracle's, then the
    SAME fp32 pairs feed both tree builders; margins are compared after the update."""
    import paper_1806_11248_amd as g
    for cfg, n, rounds, csr in ((2, 50_000, 4, False), (3, 50_000, 3, True)):
        d = synth.make(cfg, n)
        p = d["params"]
        n, F = d["X"].shape
        o, gdev = gpu_prep(ctx, oracle, d, use_csr=csr)
        y_t = dev(d["y"])
        margin_gpu = torch.zeros(n, dtype=torch.float32, device="cuda")
        margin_ref = np.zeros(n, np.float32)
        for r in range(rounds):
            _say(f"boost C{cfg} round {r}")
            gp_ref = oracle.gradients(p["objective"], margin_ref, d["y"])
            gp_gpu = ctx.gradients(p["objective"], margin_gpu, y_t).cpu().numpy()
            assert np.allclose(gp_gpu, gp_ref, rtol=1e-5, atol=1e-6)
            tree, rep = grow_and_judge(ctx, oracle, o, gdev, gp_ref, p, n, F)
            ctx.predict([tree], margin_gpu, p["eta"], packed=gdev["packed"], bits=gdev["bits"],
                        missing_sym=gdev["missing"], n=n, F=F)
            margin_ref = oracle.predict_sym(tree, o["sym"], o["missing"], p["eta"], margin_ref)
            assert np.allclose(margin_gpu.cpu().numpy(), margin_ref, rtol=1e-5, atol=1e-6)


@pytest.mark.parametrize("depth,F,miss", [(1, 13, 0.0), (2, 13, 0.0), (3, 13, 0.0), (4, 13, 0.0), (5, 13, 0.0),
                                          (6, 13, 0.0), (8, 13, 0.0), (7, 16, 0.1), (6, 3, 0.0), (9, 8, 0.3),
                                          (10, 13, 0.0), (11, 5, 0.2), (13, 12, 0.0)])
def test_last_levels_without_moving_rows(ctx, ctx_env, oracle, depth, F, miss):
    """Byte symbols, at most 16 features: the last two levels that need histograms are built without
    moving rows (the second of them with two histograms per workgroup over the first one's segments)
    and the leaves' row counts come from a count over up to three levels of splits (depth 2:
    straight from the packed matrix).  From depth 7 on, levels further up also leave the rows in place two at a
    time and a third pass moves them over three levels of splits at once (depth 10 and 13: twice and three times
    in a tree).  Same trees as with one such level, as with the rows moved at every level, and as without those
    cycles."""
    n = 120_000
    d = synth.make(4, n)
    rng = np.random.default_rng(100 * depth + F)
    X = d["X"] if F == 13 and miss == 0.0 else d["X"][:, rng.integers(0, d["X"].shape[1], F)].copy()
    if miss > 0:
        X = X + rng.normal(0, 0.01, X.shape).astype(np.float32)
        X[rng.random(X.shape) < miss] = np.nan
    p = dict(d["params"], max_depth=depth)
    n, F = X.shape
    _say(f"no-move last levels, depth {depth} F={F} missing={miss}")
    o, gdev = gpu_prep(ctx, oracle, dict(X=X, params=p))
    gp = oracle.gradients(p["objective"], np.zeros(n, np.float32), d["y"])
    tree, rep = grow_and_judge(ctx, oracle, o, gdev, gp, p, n, F)
    import paper_1806_11248_amd as g
    params = g.make_params(max_depth=depth, max_bins=p["max_bins"], lam=p["lam"], gamma=p["gamma"],
                           min_child_weight=p["min_child_weight"])
    nn = tree["n_nodes"]
    # (a variable stays set for the contexts made after it: the cycles need both in-place levels anyway)
    for env in ({"GBT_TUNE_PART_CYCLE": 0}, {"GBT_TUNE_PART_NOMOVE": 0}, {"GBT_TUNE_PART_NOMOVE": 1}):
        other, _, _ = ctx_env(**env).grow_tree(gdev["packed"], gdev["bits"], n, F, gdev["missing"], gdev["nb"], gdev["cuts"],
                                               dev(gp), params, want_rows=False, want_leaf=False)
        assert other["n_nodes"] == nn
        for k in ("feature", "bin", "default_left", "left", "right", "n_rows", "weight", "gain", "sumG", "sumH"):
            assert np.array_equal(other[k][:nn], tree[k][:nn]), (env, k)
