"""Edge cases and randomised small cases of the GPU path against the oracle (-m gpu)."""
import numpy as np
import pytest
import torch
from hypothesis import HealthCheck, given, settings, strategies as st

from gpu_util import dev, host_u32, judge_on_grid, oracle_prep, tree_kw

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    import paper_1806_11248_amd as g
    c = g.Context(0)
    yield c
    c.close()


def _grow_and_judge(ctx, oracle, X, gp, p):
    import paper_1806_11248_amd as g
    n, F = X.shape
    B = p["max_bins"]
    o = oracle_prep(oracle, X, B)
    cuts, nb, sym, mv, ms = ctx.quantise(dev(X), max_bins=B)
    assert np.array_equal(sym.cpu().numpy(), o["sym"]) and (mv, ms) == (o["max_value"], o["missing"])
    assert np.array_equal(cuts.cpu().numpy(), o["cuts"]) and np.array_equal(nb.cpu().numpy(), o["nb"])
    packed, bits = ctx.compress(sym, mv)
    assert np.array_equal(host_u32(packed), o["words"])
    params = g.make_params(max_depth=p["max_depth"], max_bins=B, lam=p["lam"], gamma=p["gamma"],
                           min_child_weight=p["min_child_weight"])
    gp_t = dev(gp)
    tree, row_idx, leaf = ctx.grow_tree(packed, bits, n, F, ms, nb, cuts, gp_t, params)
    _, scale = ctx.gpair_fixed(gp_t)
    judge_on_grid(oracle, oracle.replay_tree, tree, o, gp, scale, **tree_kw(p))
    rep = oracle.replay_tree(tree, o["sym"], o["nb"], o["missing"], gp, **tree_kw(p),
                             sum_atol_per_row=0.5 / min(scale))
    assert rep["ok"], rep["errors"][:5]
    assert np.array_equal(host_u32(row_idx), rep["row_idx"])
    assert np.array_equal(leaf.cpu().numpy(), rep["leaf_of_row"])
    return tree, o, dict(packed=packed, bits=bits, missing=ms)


P0 = dict(max_depth=3, max_bins=16, lam=1.0, gamma=0.0, min_child_weight=1.0)


def test_single_row_and_single_feature(ctx, oracle):
    print("n=1", flush=True)
    tree, _, _ = _grow_and_judge(ctx, oracle, np.array([[0.5]], np.float32), np.array([[1.0, 1.0]], np.float32), P0)
    assert tree["n_nodes"] == 1
    print("n=65, F=1", flush=True)
    rng = np.random.default_rng(0)
    X = rng.random((65, 1)).astype(np.float32)
    gp = np.stack([np.where(X[:, 0] > 0.5, 1.0, -1.0), np.ones(65)], 1).astype(np.float32)
    tree, _, _ = _grow_and_judge(ctx, oracle, X, gp, P0)
    assert tree["n_nodes"] >= 3


def test_no_hessian_mass_under_lambda_zero(ctx, oracle):
    # lambda = 0 and every hessian 0: no candidate has a finite gain and the root's weight is defined as 0
    print("no curvature at all", flush=True)
    rng = np.random.default_rng(3)
    X = rng.random((500, 3)).astype(np.float32)
    gp = np.stack([rng.standard_normal(500), np.zeros(500)], 1).astype(np.float32)
    p = dict(P0, lam=0.0, min_child_weight=0.0)
    tree, _, _ = _grow_and_judge(ctx, oracle, X, gp, p)
    assert tree["n_nodes"] == 1 and tree["weight"][0] == 0.0 and tree["sumH"][0] == 0.0
    m = ctx.predict([tree], dev(np.ones(500, np.float32)), 0.5, X=dev(X), n=500, F=3).cpu().numpy()
    assert np.array_equal(m, np.ones(500, np.float32))
    # some rows with curvature, some without: whatever is grown, both sides agree on it and no weight is NaN
    print("half the rows without curvature", flush=True)
    gp[::2, 1] = 1.0
    tree, _, _ = _grow_and_judge(ctx, oracle, X, gp, p)
    assert not np.isnan(tree["weight"][: tree["n_nodes"]]).any()


def test_identical_rows_and_constant_features(ctx, oracle):
    print("identical rows", flush=True)
    X = np.tile(np.array([[1.0, 2.0, 3.0]], np.float32), (1000, 1))
    rng = np.random.default_rng(1)
    gp = np.stack([rng.standard_normal(1000), np.ones(1000)], 1).astype(np.float32)
    tree, _, _ = _grow_and_judge(ctx, oracle, X, gp, P0)
    assert tree["n_nodes"] == 1                       # one bin per feature: nothing to split on
    print("all missing but one column", flush=True)
    X = np.full((3000, 4), np.nan, np.float32)
    X[:, 2] = rng.random(3000)
    gp = np.stack([np.where(X[:, 2] > 0.3, 1.0, -1.0), np.ones(3000)], 1).astype(np.float32)
    tree, _, _ = _grow_and_judge(ctx, oracle, X, gp, P0)
    assert tree["feature"][0] == 2


def test_two_bins_and_many_bins(ctx, oracle):
    rng = np.random.default_rng(2)
    X = rng.standard_normal((5000, 5)).astype(np.float32)
    gp = np.stack([rng.standard_normal(5000) + (X[:, 1] > 0), rng.random(5000) + 0.5], 1).astype(np.float32)
    for B in (2, 3, 1000, 4096):
        print(f"max_bins={B}", flush=True)
        p = dict(P0, max_bins=B, max_depth=4)
        _grow_and_judge(ctx, oracle, X, gp, p)


def test_predict_several_trees_in_order(ctx, oracle):
    rng = np.random.default_rng(3)
    n, F = 20_000, 6
    X = rng.standard_normal((n, F)).astype(np.float32)
    X[rng.random((n, F)) < 0.2] = np.nan
    y = (rng.random(n) < 0.5).astype(np.float32)
    p = dict(P0, max_bins=32, max_depth=4)
    margin = np.zeros(n, np.float32)
    trees = []
    for r in range(3):
        gp = oracle.gradients("logistic", margin, y)
        tree, o, gdev = _grow_and_judge(ctx, oracle, X, gp, p)
        trees.append(tree)
        margin = oracle.predict_sym(tree, o["sym"], o["missing"], 0.3, margin)
    print("predict 3 trees", flush=True)
    got = ctx.predict(trees, dev(np.zeros(n, np.float32)), 0.3, packed=gdev["packed"], bits=gdev["bits"],
                      missing_sym=gdev["missing"], n=n, F=F).cpu().numpy()
    got_raw = ctx.predict(trees, dev(np.zeros(n, np.float32)), 0.3, X=dev(X)).cpu().numpy()
    assert np.array_equal(got, margin) and np.array_equal(got_raw, margin)


# (rows, features, bins, missing): row widths on both sides of every switch between the walks over packed rows --
# up to 128 bits in registers, 8-bit rows of at most 16 bytes by byte selectors, 33 to 128 bytes staged through LDS a
# wave's 64 rows at a time, anything else gathered level by level -- and row counts around a wave and a block of rows
PREDICT_WIDTHS = [
    (1, 40, 300, 0.3), (63, 40, 300, 0.3), (65, 40, 300, 0.0), (4097, 40, 300, 0.5),     # 9 bits x 40 = 45 bytes
    (5000, 29, 256, 0.0), (5000, 29, 257, 0.2),                                          # 29 and 33 bytes
    (777, 100, 1000, 0.1), (3000, 102, 1000, 0.1), (2000, 103, 1000, 0.0),               # 125, 127.5, 128.75 bytes
    (6000, 16, 256, 0.0), (6000, 17, 256, 0.1), (4000, 12, 700, 0.2),                    # 16, 17 bytes; 15 bytes of 10 bits
]


@pytest.mark.parametrize("n,F,B,miss", PREDICT_WIDTHS)
def test_predict_over_packed_rows_of_every_width(ctx, oracle, n, F, B, miss):
    import paper_1806_11248_amd as g
    rng = np.random.default_rng(n * 131 + F)
    X = rng.standard_normal((n, F)).astype(np.float32)
    X[rng.random((n, F)) < miss] = np.nan
    print(f"predict over packed rows n={n} F={F} B={B} miss={miss}", flush=True)
    o = oracle_prep(oracle, X, B)
    packed = dev(oracle.pack(o["sym"], o["bits"]).view(np.int32))
    # two trees that need not be good, only deep and different: grown by the oracle on random pairs
    trees = []
    for k in range(2):
        gp = np.stack([rng.standard_normal(n), rng.random(n) + 0.5], 1).astype(np.float32)
        t, _, _ = oracle.grow_tree(o["sym"], o["nb"], o["cuts"], o["missing"], gp, max_depth=5 + k, max_bins=B, lam=1.0, gamma=0.0,
                                   min_child_weight=0.0)
        trees.append(t)
    m0 = rng.standard_normal(n).astype(np.float32)
    ref = m0
    for t in trees:
        ref = oracle.predict_sym(t, o["sym"], o["missing"], 0.3, ref)
    got = ctx.predict(trees, dev(m0), 0.3, packed=packed, bits=o["bits"], missing_sym=o["missing"], n=n, F=F).cpu().numpy()
    assert np.array_equal(got, ref)
    one = ctx.predict(trees[:1], dev(m0), 0.3, packed=packed, bits=o["bits"], missing_sym=o["missing"], n=n, F=F).cpu().numpy()
    assert np.array_equal(one, oracle.predict_sym(trees[0], o["sym"], o["missing"], 0.3, m0))


@settings(max_examples=30, deadline=None, suppress_health_check=list(HealthCheck), derandomize=True)
@given(seed=st.integers(0, 2 ** 31 - 1), n=st.integers(1, 3000), F=st.integers(1, 20),
       B=st.sampled_from([2, 5, 16, 33, 64, 256]), miss=st.sampled_from([0.0, 0.0, 0.3, 0.9]),
       depth=st.integers(0, 5), lam=st.sampled_from([0.0, 1.0, 10.0]), gamma=st.sampled_from([0.0, 0.5]),
       mcw=st.sampled_from([0.0, 1.0, 20.0]), ties=st.booleans())
def test_random_small_trees(ctx, oracle, seed, n, F, B, miss, depth, lam, gamma, mcw, ties):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((n, F)).astype(np.float32)
    if ties:
        X = np.round(X * 2) / 2                         # few distinct values, duplicated features
        if F > 1:
            X[:, F - 1] = X[:, 0]
    if miss:
        X[rng.random((n, F)) < miss] = np.nan
    g = rng.standard_normal(n) * rng.choice([1e-3, 1.0, 50.0])
    h = rng.random(n) * rng.choice([1e-2, 1.0]) + 1e-3
    if ties:
        g, h = np.sign(g) * 0.5, np.full(n, 0.25)        # exactly representable: exact gain ties
    gp = np.stack([g, h], 1).astype(np.float32)
    print(f"random tree seed={seed} n={n} F={F} B={B} miss={miss} depth={depth} lam={lam} gamma={gamma} mcw={mcw} ties={ties}",
          flush=True)
    _grow_and_judge(ctx, oracle, X, gp, dict(max_depth=depth, max_bins=B, lam=lam, gamma=gamma, min_child_weight=mcw))


@settings(max_examples=25, deadline=None, suppress_health_check=list(HealthCheck), derandomize=True)
@given(seed=st.integers(0, 2 ** 31 - 1), n=st.integers(1, 6000), F=st.integers(1, 40),
       B=st.sampled_from([2, 7, 32, 256, 1000]), miss=st.sampled_from([0.0, 0.5, 0.9, 1.0]),
       depth=st.integers(0, 9), max_leaves=st.integers(1, 60), ties=st.booleans())
def test_random_sparse_rows_and_lossguide(ctx, oracle, seed, n, F, B, miss, depth, max_leaves, ties):
    """Random small shapes through the other two growth entry points: the sparse-row form must give
    the packed form's tree, row order and leaves bit for bit (the packed form is judged above), and
    loss-guided growth in rounds must pass the oracle's replay of the sequential rule."""
    import paper_1806_11248_amd as g
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((n, F)).astype(np.float32)
    if ties:
        X = np.round(X * 2) / 2
    if miss:
        X[rng.random((n, F)) < miss] = np.nan
    gv = rng.standard_normal(n) * rng.choice([1e-2, 1.0, 20.0])
    hv = rng.random(n) + 1e-3
    if ties:
        gv, hv = np.sign(gv) * 0.5, np.full(n, 0.25)
    gp = np.stack([gv, hv], 1).astype(np.float32)
    print(f"random sparse/lossguide seed={seed} n={n} F={F} B={B} miss={miss} depth={depth} leaves={max_leaves} ties={ties}",
          flush=True)
    p = dict(max_depth=depth, max_bins=B, lam=1.0, gamma=0.0, min_child_weight=1.0)
    o = oracle_prep(oracle, X, B)
    cuts, nb, sym, mv, ms = ctx.quantise(dev(X), max_bins=B)
    packed, bits = ctx.compress(sym, mv)
    params = g.make_params(max_depth=depth, max_bins=B, lam=1.0, gamma=0.0, min_child_weight=1.0)
    gp_t = dev(gp)
    tree, row_idx, leaf = ctx.grow_tree(packed, bits, n, F, ms, nb, cuts, gp_t, params)
    nn = tree["n_nodes"]
    if F * B <= 65536:
        rowptr, ent, nnz = ctx.compress_sparse(sym, B, ms)
        assert nnz == int((o["sym"] != o["missing"]).sum())
        st_, srows, sleaf = ctx.grow_tree_sparse(rowptr, ent, n, nnz, F, nb, cuts, gp_t, params)
        assert st_["n_nodes"] == nn
        for k in ("feature", "bin", "default_left", "left", "right", "n_rows", "threshold", "weight", "gain",
                  "sumG", "sumH"):
            assert np.array_equal(st_[k][:nn], tree[k][:nn]), k
        assert torch.equal(srows, row_idx) and torch.equal(sleaf, leaf)
        m = ctx.predict_sparse([tree], dev(np.zeros(n, np.float32)), 0.5, rowptr, ent, n, F, B)
        m2 = ctx.predict([tree], dev(np.zeros(n, np.float32)), 0.5, packed=packed, bits=bits, missing_sym=ms, n=n, F=F)
        assert torch.equal(m, m2)
    lg, lrows, lleaf = ctx.grow_tree_lossguide(packed, bits, n, F, ms, nb, cuts, gp_t, params, max_leaves)
    _, scale = ctx.gpair_fixed(gp_t)
    judge_on_grid(oracle, oracle.replay_tree_lossguide, lg, o, gp, scale, max_leaves=max_leaves, **tree_kw(p))
    rep = oracle.replay_tree_lossguide(lg, o["sym"], o["nb"], o["missing"], gp, max_leaves=max_leaves, **tree_kw(p),
                                       sum_atol_per_row=0.5 / min(scale))
    assert rep["ok"], rep["errors"][:5]
    assert np.array_equal(host_u32(lrows), rep["row_idx"])
    assert np.array_equal(lleaf.cpu().numpy(), rep["leaf_of_row"])


@settings(max_examples=15, deadline=None, suppress_health_check=list(HealthCheck), derandomize=True)
@given(seed=st.integers(0, 2 ** 31 - 1), n=st.integers(5_000, 250_000), F=st.integers(1, 40),
       B=st.sampled_from([16, 64, 255, 256]), miss=st.sampled_from([0.0, 0.0, 0.2]), depth=st.integers(1, 9),
       skew=st.booleans())
def test_random_medium_trees(ctx, oracle, seed, n, F, B, miss, depth, skew):
    """Shapes of a few tiles to a few dozen tiles through whichever growth path their width selects
    (fused partition + histogram up to 16 byte-wide features, one-launch partition, id lists), with and
    without the final row order, against the oracle's replay."""
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((n, F)).astype(np.float32)
    if skew:   # low-cardinality columns with one dominant value, like categorical data
        k = max(1, F // 2)
        X[:, :k] = np.floor(np.abs(X[:, :k]) * 1.5)
    if miss:
        X[rng.random((n, F)) < miss] = np.nan
    y = (X[:, 0] > 0).astype(np.float64) + 0.3 * rng.standard_normal(n)
    gp = np.stack([rng.standard_normal(n) * 0.1 - np.nan_to_num(y), rng.random(n) * 0.5 + 0.5], 1).astype(np.float32)
    print(f"random medium tree seed={seed} n={n} F={F} B={B} miss={miss} depth={depth} skew={skew}", flush=True)
    import paper_1806_11248_amd as g
    p = dict(max_depth=depth, max_bins=B, lam=1.0, gamma=0.0, min_child_weight=1.0)
    tree, o, gdev = _grow_and_judge(ctx, oracle, X, gp, p)
    params = g.make_params(max_depth=depth, max_bins=B, lam=1.0, gamma=0.0, min_child_weight=1.0)
    cuts, nb, sym, mv, ms = ctx.quantise(dev(X), max_bins=B)
    bare, _, _ = ctx.grow_tree(gdev["packed"], gdev["bits"], n, F, ms, nb, cuts, dev(gp), params, want_rows=False,
                               want_leaf=False)
    nn = tree["n_nodes"]
    assert bare["n_nodes"] == nn
    for k in ("feature", "bin", "default_left", "left", "right", "n_rows", "weight", "gain"):
        assert np.array_equal(bare[k][:nn], tree[k][:nn]), k
