"""The final row order of Alg. 1 (RepartitionInstances applied level after level) when the rows are
not followed through the levels: it is made from the finished tree as a stable sort of the row ids
by their leaf's place in the tree's left-to-right order (-m gpu).

The whole-tree tests compare that order with the oracle's at sizes the oracle replays.  Here trees
with more leaves than one 8-bit sorting pass covers are grown, too large to replay node by node:
the order is compared with numpy's stable sort of the leaf ranks (leaf ids and trees of these
shapes are judged against the oracle elsewhere) and with the order the id-carrying partitions give."""
import numpy as np
import pytest
import torch

from gpu_util import dev, host_u32

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


@pytest.fixture()
def ctx_env(monkeypatch):
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


def leaf_ranks(tree):
    """rank[node] = place of a leaf in left-to-right order (children: left first)."""
    rank = np.full(tree["n_nodes"], -1, np.int64)
    stack, k = [0], 0
    while stack:
        i = stack.pop()
        if tree["feature"][i] < 0:
            rank[i] = k
            k += 1
        else:
            stack.append(int(tree["right"][i]))
            stack.append(int(tree["left"][i]))
    return rank, k


def random_symbols(ctx, n, F, B, seed):
    rng = np.random.default_rng(seed)
    sym = rng.integers(0, B, size=(n, F), dtype=np.uint16)
    packed, bits = ctx.compress(dev(sym), B - 1)
    nb = dev(np.full(F, B, np.int32))
    cuts = dev(np.tile(np.arange(1, B, dtype=np.float32), (F, 1)))
    gp = np.stack([rng.standard_normal(n).astype(np.float32), np.ones(n, np.float32)], 1)
    return packed, bits, nb, cuts, dev(gp)


def check_order(tree, row_idx, leaf, n):
    rank, n_leaves = leaf_ranks(tree)
    leaf = leaf.cpu().numpy()
    assert leaf.min() >= 0 and leaf.max() < tree["n_nodes"] and np.all(rank[leaf] >= 0)
    want = np.argsort(rank[leaf], kind="stable").astype(np.uint32)
    got = host_u32(row_idx)
    assert np.array_equal(got, want)
    # each leaf's run has the length the tree records
    counts = np.bincount(rank[leaf], minlength=n_leaves)
    leaves = np.flatnonzero(rank >= 0)
    assert np.array_equal(counts[rank[leaves]], tree["n_rows"][leaves])
    return n_leaves


@pytest.mark.parametrize("F,B,n,depth", [(4, 256, 1_500_000, 14),    # 8-bit records: partition + histogram pass
                                         (3, 64, 300_000, 16),        # 18-bit rows: staged one-launch partition
                                         (5, 200, 9_000, 0)])         # one leaf
def test_depthwise_order_beyond_one_pass(ctx_env, F, B, n, depth):
    import paper_1806_11248_amd as g
    c = ctx_env()
    packed, bits, nb, cuts, gp = random_symbols(c, n, F, B, 11 + F)
    params = g.make_params(max_depth=depth, max_bins=B, lam=0.0, gamma=0.0, min_child_weight=0.0)
    _say(f"row order F={F} B={B} n={n} depth={depth} path={c.grow_tree_path(F, bits, B, track_rows=True)}")
    tree, row_idx, leaf = c.grow_tree(packed, bits, n, F, B, nb, cuts, gp, params)
    n_leaves = check_order(tree, row_idx, leaf, n)
    _say(f"  {tree['n_nodes']} nodes, {n_leaves} leaves")
    assert depth == 0 or n_leaves > 256
    # rows only (the leaf ids then live in the workspace)
    t2, rows2, none_leaf = c.grow_tree(packed, bits, n, F, B, nb, cuts, gp, params, want_leaf=False)
    assert none_leaf is None and torch.equal(rows2, row_idx)
    # the id-carrying three-launch partitions end with the same list
    c0 = ctx_env(GBT_TUNE_ORDER_ROWS=0)
    assert c0.grow_tree_path(F, bits, B, track_rows=True) == 0
    t0, rows0, leaf0 = c0.grow_tree(packed, bits, n, F, B, nb, cuts, gp, params)
    assert t0["n_nodes"] == tree["n_nodes"]
    for k in ("feature", "bin", "default_left", "left", "right", "n_rows"):
        assert np.array_equal(t0[k][:t0["n_nodes"]], tree[k][:t0["n_nodes"]]), k
    assert torch.equal(rows0, row_idx) and torch.equal(leaf0, leaf)


def test_lossguide_order_three_passes(ctx_env):
    """More than 65,536 leaves: three 8-bit passes over (rank, row) pairs."""
    import paper_1806_11248_amd as g
    c = ctx_env()
    F, B, n, max_leaves = 3, 64, 400_000, 70_000
    packed, bits, nb, cuts, gp = random_symbols(c, n, F, B, 5)
    params = g.make_params(max_depth=64, max_bins=B, lam=0.0, gamma=0.0, min_child_weight=0.0)
    _say(f"row order, loss-guided, {max_leaves} leaves")
    tree, row_idx, leaf = c.grow_tree_lossguide(packed, bits, n, F, B, nb, cuts, gp, params, max_leaves)
    n_leaves = check_order(tree, row_idx, leaf, n)
    _say(f"  {tree['n_nodes']} nodes, {n_leaves} leaves")
    assert n_leaves > 65_536
