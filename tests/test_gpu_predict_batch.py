"""Prediction with many trees on raw floats (Sec. 2.4: trees in order, one instance per thread) in the
form that reads the rows once and takes the trees through LDS in groups (-m gpu).  The oracle walks
one tree at a time over the same floats; margins must be bit-identical (fp32 rounding after every
tree on both sides), on new data as well as on the training matrix."""
import numpy as np
import pytest
import torch

from gpu_util import dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    import paper_1806_11248_amd as g
    c = g.Context(0)
    yield c
    c.close()


def _boost(ctx, X, y, B, rounds, depth, lossguide_every=0):
    """rounds trees grown on the GPU (each judged elsewhere); returns trees as numpy dicts."""
    import paper_1806_11248_amd as g
    n, F = X.shape
    cuts, nb, sym, mv, ms = ctx.quantise(dev(X), max_bins=B)
    packed, bits = ctx.compress(sym, mv)
    margin = torch.zeros(n, device="cuda")
    trees = []
    for r in range(rounds):
        d = 1 + (r * 3) % depth                      # trees of different depths inside one group
        params = g.make_params(max_depth=d, max_bins=B, lam=1.0, eta=0.3, objective="logistic")
        gp = ctx.gradients("logistic", margin, dev(y))
        if lossguide_every and r % lossguide_every == 1:
            big = g.make_params(max_depth=12, max_bins=B, lam=1.0, eta=0.3, objective="logistic")
            t, _, _ = ctx.grow_tree_lossguide(packed, bits, n, F, ms, nb, cuts, gp, big, 24, want_rows=False,
                                              want_leaf=False)
        else:
            t, _, _ = ctx.grow_tree(packed, bits, n, F, ms, nb, cuts, gp, params, want_rows=False, want_leaf=False)
        ctx.predict([t], margin, 0.3, packed=packed, bits=bits, missing_sym=ms, n=n, F=F)
        trees.append(t)
    return trees, margin.cpu().numpy()


@pytest.mark.parametrize("n,F,B,rounds,depth,miss", [
    (30_011, 28, 256, 45, 6, 0.0),      # three groups of trees (2048 nodes of LDS each)
    (9_000, 7, 64, 20, 5, 0.3),         # missing values, an odd number of features
    (5_003, 95, 32, 6, 4, 0.1),         # the widest row tile the kernel takes
    (300, 3, 16, 2, 3, 0.0),            # two trees, one partial tile
])
def test_many_trees_on_raw_floats(ctx, oracle, n, F, B, rounds, depth, miss):
    rng = np.random.default_rng(n + F)
    X = rng.standard_normal((n, F)).astype(np.float32)
    X[:, 0] = np.round(X[:, 0] * 3)
    if miss:
        X[rng.random((n, F)) < miss] = np.nan
    y = (rng.random(n) < 1 / (1 + np.exp(-(X[:, 0] + np.nan_to_num(X[:, 1]))))).astype(np.float32)
    print(f"batched predict n={n} F={F} trees={rounds}", flush=True)
    trees, boosted = _boost(ctx, X, y, B, rounds, depth, lossguide_every=4)
    # the training matrix: the margins the boosting loop accumulated tree by tree over packed symbols
    got = ctx.predict(trees, dev(np.zeros(n, np.float32)), 0.3, X=dev(X)).cpu().numpy()
    assert np.array_equal(got, boosted)
    # new rows, with infinities and values equal to thresholds, against the oracle's walk
    m = 4_099
    Z = rng.standard_normal((m, F)).astype(np.float32) * 2
    Z[rng.random((m, F)) < 0.15] = np.nan
    Z[rng.random((m, F)) < 0.02] = np.inf
    Z[rng.random((m, F)) < 0.02] = -np.inf
    thr = np.concatenate([t["threshold"][:t["n_nodes"]][t["feature"][:t["n_nodes"]] >= 0] for t in trees])
    thr = thr[np.isfinite(thr)]
    if len(thr):
        Z[np.arange(0, m, 7), 0] = thr[np.arange(0, m, 7) % len(thr)]     # x == threshold goes right
    start = rng.standard_normal(m).astype(np.float32)
    ref = start.copy()
    for t in trees:
        ref = oracle.predict_raw(t, Z, 0.3, ref)
    got = ctx.predict(trees, dev(start), 0.3, X=dev(Z)).cpu().numpy()
    assert np.array_equal(got, ref)
    # one tree at a time through the single-tree kernels gives the same
    step = dev(start)
    for t in trees:
        ctx.predict([t], step, 0.3, X=dev(Z))
    assert np.array_equal(step.cpu().numpy(), ref)
