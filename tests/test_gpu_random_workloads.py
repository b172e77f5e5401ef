"""GPU parity on RANDOM small workloads (-m gpu): shapes, bin counts, missing rates, gradient-pair
distributions and parameters drawn per seed, far outside what the named configurations cover (1 to 250 000
rows, 1 to 400 features, 2 to 4096 bins, up to 90% missing, pairs spanning eight decades with zero hessians
and outliers, lambda = 0, min_child_weight = 0, depth 0 to 9).  Everything is judged in the GPU library's own
precision (pairs moved onto its fixed-point grid, where the oracle's sums are exact): histograms and gains
equal to the last bit, the oracle's exhaustive best split at every node, partitions and predictions bit-exact.

A fixed set of seeds runs by default.  GBT_TEST_SWEEP_SECONDS=<s> adds fresh seeds for that long (seeds start
at GBT_TEST_SWEEP_SEED, default 1000000), printing each case before it runs (give pytest -s to see them as
they come).
"""
import os
import time

import numpy as np
import pytest
import torch

import grid
from gpu_util import dev, host_u32, judge_on_grid, tree_kw
from test_gpu_lossguide import _judge as lossguide_judge
from test_gpu_tree import gpu_prep, grow_and_judge

pytestmark = pytest.mark.gpu

# Contexts are created under one of these settings in turn: every path the growers can take (the default
# choices, rows moved at every level or not at the last one or two or only every third level, the three-launch partition, histograms
# apart from the partition, pairs rounded in a pass of their own, row ids carried along, one loss-guided
# expansion per round, run-time bit widths, other workgroup shapes and LDS tile sizes, rows of up to 64 words moved instead of listed,
# the 8-bit root histogram by the general kernel, every histogram job a single merge-free piece or many short ones)
VARIANTS = [
    {},
    {"GBT_TUNE_PART_NOMOVE": "0"},
    {"GBT_TUNE_PART_NOMOVE": "1"},
    {"GBT_TUNE_PART_CYCLE": "0"},
    {"GBT_TUNE_PART_FUSED": "0"},
    {"GBT_TUNE_PART_HIST": "0"},
    {"GBT_TUNE_HIST_FIX": "0"},
    {"GBT_TUNE_ORDER_ROWS": "0"},
    {"GBT_TUNE_LOSSGUIDE_BATCH": "1"},
    {"GBT_TUNE_HIST_RUNTIME_BITS": "1"},
    {"GBT_TUNE_HIST_BLOCK": "256", "GBT_TUNE_HIST_LDS_KB": "16", "GBT_TUNE_HIST_JOBS": "3"},
    {"GBT_TUNE_HIST_LDS_KB": "128"},
    {"GBT_TUNE_PART_IDS": "0"},
    {"GBT_TUNE_MOVE_MAX_WORDS": "64"},
    {"GBT_TUNE_HIST8": "0"},
    {"GBT_TUNE_HIST_MERGE_RATIO": "100000"},
    {"GBT_TUNE_HIST_MERGE_RATIO": "1", "GBT_TUNE_HIST_JOBS": "32"},
]


def _say(msg):
    print(msg, flush=True)


def column(rng, n, kind):
    """One feature column: smooth, few integer levels, constant, Zipf categories, heavy-tailed, coarse grid."""
    if kind == 0:
        return rng.standard_normal(n)
    if kind == 1:
        return rng.integers(0, rng.integers(2, 40), n).astype(float)
    if kind == 2:
        return np.full(n, 3.25)
    if kind == 3:
        K = int(rng.integers(3, 400))
        w = np.arange(1, K + 1) ** -1.2
        return rng.choice(K, n, p=w / w.sum()).astype(float) + 1
    if kind == 4:
        return np.exp(rng.standard_normal(n) * 2)
    return np.round(rng.standard_normal(n) * 3) / 3


def random_workload(seed):
    """(workload, pairs, parameters, n, F, description) drawn from the seed."""
    rng = np.random.default_rng(seed)
    n = int(rng.choice([1, 2, 63, 64, 65, 500, 2047, 2049, 7000, 30000, 90000, 250000]))
    if n > 10:
        n = max(1, n + int(rng.integers(-3, 4)))
    F = int(rng.choice([1, 2, 3, 5, 8, 12, 13, 16, 17, 28, 40, 70, 150, 400]))
    B = int(rng.choice([2, 3, 4, 16, 17, 64, 100, 255, 256, 257, 512, 1024, 4096]))
    n = min(n, 4_000_000 // F)          # (keeps the oracle's sorts short; rows wider than 64 words stay in)
    miss = float(rng.choice([0.0, 0.0, 0.02, 0.3, 0.9]))
    X = np.stack([column(rng, n, int(rng.integers(0, 6))) for _ in range(F)], 1).astype(np.float32)
    if miss > 0:
        X[rng.random((n, F)) < miss] = np.nan
    sg, sh = 10.0 ** rng.uniform(-4, 4), 10.0 ** rng.uniform(-4, 4)
    mode = int(rng.integers(0, 4))
    if mode == 0:     # anything
        gp = np.stack([rng.standard_normal(n) * sg, rng.uniform(0, 1, n) * sh], 1)
    elif mode == 1:   # the first tree of a logistic model
        gp = np.stack([rng.choice([-0.5, 0.5], n), np.full(n, 0.25)], 1)
    elif mode == 2:   # squared error
        gp = np.stack([rng.standard_normal(n) * sg + sg, np.ones(n)], 1)
    else:             # half the hessians zero, one row in a thousand a thousand times the rest
        gp = np.stack([rng.standard_normal(n) * sg, np.where(rng.random(n) < 0.5, 0.0, rng.uniform(0, 1, n) * sh)], 1)
        gp[rng.integers(0, n, max(1, n // 1000))] *= 1000.0
    gp = gp.astype(np.float32)
    lam = float(rng.choice([0.0, 1.0, 10.0]))
    mcw = float(rng.choice([0.0, 1.0, 5.0])) * (sh if mode == 0 else 1.0)
    if mode == 3:     # (no child weight a sum could equal; lambda = 0 with rows that have no curvature is in)
        lam, mcw = float(rng.choice([0.0, 1.0])), float(rng.choice([0.0, 1.7321])) * sh
    p = dict(max_depth=int(rng.integers(0, 10)), max_bins=B, lam=lam, gamma=float(rng.choice([0.0, 0.0, 1e-3, 1.0])),
             min_child_weight=mcw)
    desc = dict(seed=seed, n=n, F=F, B=B, miss=miss, mode=mode, sg=float(f"{sg:.3g}"), sh=float(f"{sh:.3g}"),
                depth=p["max_depth"], lam=lam, gamma=p["gamma"], mcw=float(f"{mcw:.4g}"))
    return dict(X=X, params=p), gp, p, n, F, desc


def check_growers(oracle, monkeypatch, seed):
    import paper_1806_11248_amd as g
    d, gp, p, n, F, desc = random_workload(seed)
    variant = VARIANTS[seed % len(VARIANTS)]
    for v in VARIANTS:
        for k in v:
            monkeypatch.delenv(k, raising=False)
    for k, v in variant.items():
        monkeypatch.setenv(k, v)
    lossguide = seed % 4 == 3
    _say(f"random workload {desc} {variant} lossguide={lossguide}")
    ctx = g.Context(0)
    try:
        o, gdev = gpu_prep(ctx, oracle, d, use_csr=(seed % 5 == 0))
        if lossguide:
            max_leaves = int(np.random.default_rng(seed).integers(1, 40))
            lossguide_judge(ctx, oracle, o, gdev, gp, dict(p, max_depth=max(p["max_depth"], 1)), n, F, max_leaves,
                            grid_only=True)
        else:
            grow_and_judge(ctx, oracle, o, gdev, gp, p, n, F, grid_only=True)
    finally:
        ctx.close()


def check_steps_sparse_predict(ctx, oracle, seed):
    import paper_1806_11248_amd as g
    d, gp, p, n, F, desc = random_workload(seed)
    B = p["max_bins"]
    _say(f"random workload {desc}: steps, sparse rows, prediction")
    o, gdev = gpu_prep(ctx, oracle, d)
    params = g.make_params(max_depth=p["max_depth"], max_bins=B, lam=p["lam"], gamma=p["gamma"],
                           min_child_weight=p["min_child_weight"])
    gp_t = dev(gp)
    gq, scale = ctx.gpair_fixed(gp_t)
    og = grid.on_grid(gp)
    # the steps on a random half of the rows: histogram, totals, best split, partition.  On the grid the
    # oracle's sums are exact, so "equal" means equal
    rng = np.random.default_rng(seed)
    rows = np.sort(rng.choice(n, max(1, n // 2), replace=False)).astype(np.uint32)
    rows_t = dev(rows.view(np.int32))
    h = ctx.build_hist(gdev["packed"], gdev["bits"], n, F, B, gdev["missing"], gq, rows_t)
    ref, cnt, G, H = oracle.hist(o["sym"], B, o["missing"], rows, og)
    hf = ctx.hist_export_f64(h, scale).cpu().numpy()
    assert np.array_equal(hf, ref)
    Gq, Hq = ctx.sum_gpair(gq, rows_t)
    assert (Gq / scale[0], Hq / scale[1]) == (G, H)
    sp = ctx.eval_split(h, gdev["nb"], Gq, Hq, scale, params)
    spo = oracle.eval_split(ref, cnt, o["nb"], G, H, len(rows), p["lam"], p["min_child_weight"])
    if spo["valid"] and spo["gain"] > 0:
        where = (spo["feature"], spo["bin"], spo["default_left"])
        assert (sp["feature"], sp["bin"], sp["default_left"]) == where and sp["gain"] == spo["gain"], (sp, spo)
        out, nl = oracle.partition(o["sym"], rows, *where, o["missing"])
        r2 = rows_t.clone()
        nl2 = ctx.partition(gdev["packed"], gdev["bits"], n, F, r2, 0, len(rows), *where, gdev["missing"])
        assert nl2 == nl and np.array_equal(host_u32(r2), out)
    else:   # nothing worth a split: the GPU may name a candidate without gain (it does not count rows), no more
        assert not sp["valid"] or not sp["gain"] > 0, (sp, spo)
    # one boosting iteration as one call and as three: the same pairs, tree and margins to the last bit
    objective = ("squared", "logistic")[seed % 2]
    y_t = dev((rng.standard_normal(n) if objective == "squared" else (rng.random(n) < 0.4)).astype(np.float32))
    m_in = dev((rng.standard_normal(n) * (3.0 if seed % 3 else 0.0)).astype(np.float32))
    bparams = g.make_params(max_depth=p["max_depth"], max_bins=B, lam=p["lam"], gamma=p["gamma"],
                            min_child_weight=p["min_child_weight"], eta=0.3, objective=objective)
    gp3 = ctx.gradients(objective, m_in, y_t)
    t3, _, _ = ctx.grow_tree(gdev["packed"], gdev["bits"], n, F, gdev["missing"], gdev["nb"], gdev["cuts"], gp3, bparams,
                             want_rows=False, want_leaf=False)
    m3 = ctx.predict([t3], m_in.clone(), 0.3, packed=gdev["packed"], bits=gdev["bits"], missing_sym=gdev["missing"], n=n, F=F)
    gp1, m1 = torch.empty_like(gp3), torch.empty_like(m_in)
    t1 = ctx.boost_round(gdev["packed"], gdev["bits"], n, F, gdev["missing"], gdev["nb"], gdev["cuts"], y_t, m_in, m1, gp1,
                         bparams)
    assert torch.equal(gp1, gp3) and torch.equal(m1, m3) and t1["n_nodes"] == t3["n_nodes"]
    for k in ("feature", "bin", "default_left", "left", "right", "n_rows", "threshold", "weight", "gain", "sumG", "sumH"):
        assert np.array_equal(t1[k][:t3["n_nodes"]], t3[k][:t3["n_nodes"]]), k
    # sparse rows: the same tree as the oracle's and as the dense layout's, to the last bit
    sym_t = dev(o["sym"])
    rowptr, ent, nnz = ctx.compress_sparse(sym_t, B, gdev["missing"])
    tree, row_idx, leaf = ctx.grow_tree_sparse(rowptr, ent, n, nnz, F, gdev["nb"], gdev["cuts"], gp_t, params)
    rep = judge_on_grid(oracle, oracle.replay_tree, tree, o, gp, scale, **tree_kw(p))
    assert np.array_equal(host_u32(row_idx), rep["row_idx"]) and np.array_equal(leaf.cpu().numpy(), rep["leaf_of_row"])
    nn = tree["n_nodes"]
    dense, _, _ = ctx.grow_tree(gdev["packed"], gdev["bits"], n, F, gdev["missing"], gdev["nb"], gdev["cuts"], gp_t,
                                params, want_rows=False, want_leaf=False)
    assert dense["n_nodes"] == nn
    for k in ("feature", "bin", "default_left", "left", "right", "n_rows", "threshold", "weight", "gain", "sumG",
              "sumH"):
        assert np.array_equal(dense[k][:nn], tree[k][:nn]), k
    # two trees' worth of prediction from sparse rows, packed symbols and raw floats
    m0 = rng.standard_normal(n).astype(np.float32)
    ref = oracle.predict_sym(tree, o["sym"], o["missing"], 0.3, m0)
    ref = oracle.predict_sym(tree, o["sym"], o["missing"], 0.3, ref)
    got = ctx.predict_sparse([tree, tree], dev(m0), 0.3, rowptr, ent, n, F, B).cpu().numpy()
    assert np.array_equal(got, ref)
    got = ctx.predict([tree, tree], dev(m0), 0.3, packed=gdev["packed"], bits=gdev["bits"],
                      missing_sym=gdev["missing"], n=n, F=F).cpu().numpy()
    assert np.array_equal(got, ref)
    got = ctx.predict([tree, tree], dev(m0), 0.3, X=dev(d["X"]), n=n, F=F).cpu().numpy()
    refr = oracle.predict_raw(tree, d["X"], 0.3, oracle.predict_raw(tree, d["X"], 0.3, m0))
    assert np.array_equal(refr, ref) and np.array_equal(got, ref)


# the sparse-row histogram with all global bin ids in LDS at once (default where they fit) or in tiles, and
# with other job counts
SPARSE_VARIANTS = [{}, {"GBT_TUNE_SPARSE_TILED": "1"}, {"GBT_TUNE_SPARSE_TILED": "1", "GBT_TUNE_SPARSE_JOBS": "4",
                                                        "GBT_TUNE_HIST_LDS_KB": "16"}]


@pytest.fixture(scope="module")
def ctxs():
    """One context per entry of SPARSE_VARIANTS (the variables are read when a context is created)."""
    import paper_1806_11248_amd as g
    made = []
    for variant in SPARSE_VARIANTS:
        saved = {k: os.environ.get(k) for k in variant}
        os.environ.update(variant)
        try:
            made.append(g.Context(0))
        finally:
            for k, v in saved.items():
                if v is None:
                    os.environ.pop(k, None)
                else:
                    os.environ[k] = v
    yield made
    for c in made:
        c.close()


@pytest.mark.parametrize("seed", range(1000, 1066))
def test_random_workload_growers(oracle, monkeypatch, seed):
    check_growers(oracle, monkeypatch, seed)


@pytest.mark.parametrize("seed", range(100000, 100032))
def test_random_workload_steps_sparse_predict(ctxs, oracle, seed):
    check_steps_sparse_predict(ctxs[seed % len(ctxs)], oracle, seed)


def test_random_workload_sweep(ctxs, oracle, monkeypatch):
    budget = float(os.environ.get("GBT_TEST_SWEEP_SECONDS", "0"))
    if budget <= 0:
        pytest.skip("set GBT_TEST_SWEEP_SECONDS to sweep fresh seeds")
    seed = int(os.environ.get("GBT_TEST_SWEEP_SEED", "1000000"))
    t0, k = time.time(), 0
    while time.time() - t0 < budget:
        check_growers(oracle, monkeypatch, seed + k)
        check_steps_sparse_predict(ctxs[(seed + k) % len(ctxs)], oracle, seed + k)
        k += 1
    _say(f"swept {k} seeds from {seed}")
