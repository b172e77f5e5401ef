"""GPU parity of loss-guided growth (Sec. 2.3: nodes opened "highest gain first") against the CPU
oracle (-m gpu): every tree is replayed by the oracle's judge, which re-derives the expansion order."""
import numpy as np
import pytest
import torch

import synth
from gpu_util import dev, host_u32, judge_on_grid, tree_kw
from test_gpu_tree import gpu_prep

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    import paper_1806_11248_amd as g
    c = g.Context(0)
    yield c
    c.close()


def _say(msg):
    print(msg, flush=True)


def _judge(ctx, oracle, o, gdev, gp, p, n, F, max_leaves, grid_only=False):
    import paper_1806_11248_amd as g
    params = g.make_params(max_depth=p["max_depth"], max_bins=p["max_bins"], lam=p["lam"], gamma=p["gamma"],
                           min_child_weight=p["min_child_weight"])
    gp_t = dev(gp)
    tree, row_idx, leaf = ctx.grow_tree_lossguide(gdev["packed"], gdev["bits"], n, F, gdev["missing"], gdev["nb"],
                                                  gdev["cuts"], gp_t, params, max_leaves)
    _, scale = ctx.gpair_fixed(gp_t)
    rep = judge_on_grid(oracle, oracle.replay_tree_lossguide, tree, o, gp, scale, max_leaves=max_leaves, **tree_kw(p))
    if not grid_only:
        rep = oracle.replay_tree_lossguide(tree, o["sym"], o["nb"], o["missing"], gp, max_leaves=max_leaves,
                                           **tree_kw(p), sum_atol_per_row=0.5 / min(scale))
        assert rep["ok"], rep["errors"][:5]
    assert np.array_equal(host_u32(row_idx), rep["row_idx"])           # partitions: bit-exact
    assert np.array_equal(leaf.cpu().numpy(), rep["leaf_of_row"])
    nn = tree["n_nodes"]
    # the same tree when row ids are not carried along (one-launch partition paths)
    bare, r2, l2 = ctx.grow_tree_lossguide(gdev["packed"], gdev["bits"], n, F, gdev["missing"], gdev["nb"],
                                           gdev["cuts"], gp_t, params, max_leaves, want_rows=False)
    assert r2 is None and bare["n_nodes"] == nn
    assert np.array_equal(l2.cpu().numpy(), rep["leaf_of_row"])
    for k in ("feature", "bin", "default_left", "left", "right", "n_rows", "threshold", "weight", "gain",
              "sumG", "sumH"):
        assert np.array_equal(bare[k][:nn], tree[k][:nn]), k
    # over sparse rows: the same tree, row order and leaves
    if True:
        rowptr, ent, nnz = ctx.compress_sparse(dev(o["sym"]), p["max_bins"], gdev["missing"])
        for want_rows in (True, False):
            st, s_rows, s_leaf = ctx.grow_tree_sparse_lossguide(rowptr, ent, n, nnz, F, gdev["nb"], gdev["cuts"], gp_t,
                                                                params, max_leaves, want_rows=want_rows)
            assert st["n_nodes"] == nn
            for k in ("feature", "bin", "default_left", "left", "right", "n_rows", "threshold", "weight", "gain",
                      "sumG", "sumH"):
                assert np.array_equal(st[k][:nn], tree[k][:nn]), ("sparse rows", k)
            assert np.array_equal(s_leaf.cpu().numpy(), rep["leaf_of_row"])
            if want_rows:
                assert np.array_equal(host_u32(s_rows), rep["row_idx"])
    # an independently grown oracle tree is the same unless a legal tie intervened
    t_ref, rows_ref, leaf_ref = oracle.grow_tree_lossguide(o["sym"], o["nb"], o["cuts"], o["missing"], gp,
                                                           max_leaves=max_leaves, **tree_kw(p))
    if rep["identical"] and not grid_only:
        assert t_ref["n_nodes"] == nn
        for k in ("feature", "bin", "default_left", "left", "right", "n_rows"):
            assert np.array_equal(tree[k][:nn], t_ref[k][:nn]), k
        assert np.allclose(tree["gain"][:nn], t_ref["gain"][:nn], rtol=1e-5, atol=1e-7)
    # prediction walks the (unbalanced) tree: packed symbols and the oracle agree
    m0 = np.zeros(n, np.float32)
    ref = oracle.predict_sym(tree, o["sym"], o["missing"], 0.3, m0)
    got = ctx.predict([tree], dev(m0), 0.3, packed=gdev["packed"], bits=gdev["bits"], missing_sym=gdev["missing"],
                      n=n, F=F).cpu().numpy()
    assert np.array_equal(got, ref)
    return tree, rep


CASES = [  # config, rows, kwargs, csr, max_leaves, max_depth
    (1, None, {}, False, 6, 8),
    (2, 60_000, {}, False, 40, 7),            # 8-bit, 28 features: one-launch partition without ids
    (3, 50_000, {}, True, 25, 12),            # 9-bit with missing values, CSR input, a deep narrow tree allowed
    (4, 200_000, {}, False, 64, 10),          # 8-bit, 13 features: partition + histogram in one pass without ids
    (5, 5_000, {"F": 300}, False, 30, 6),     # wide rows
    (4, 30_000, {}, False, 1, 5),             # a budget of one leaf: the root alone
    (4, 30_000, {}, False, 2, 5),             # one split
    (2, 20_000, {}, False, 300, 3),           # the depth cap, not the budget, ends the growth: 8 leaves
]


@pytest.mark.parametrize("cfg,n,kw,csr,max_leaves,max_depth", CASES)
def test_lossguide_tree_matches_oracle(ctx, oracle, cfg, n, kw, csr, max_leaves, max_depth):
    d = synth.make(cfg, n, **kw)
    p = dict(d["params"], max_depth=max_depth)
    X = d["X"]
    n, F = X.shape
    _say(f"loss-guided C{cfg} n={n} F={F} leaves={max_leaves} depth<={max_depth}")
    o, gdev = gpu_prep(ctx, oracle, dict(d, params=p), use_csr=csr)
    gp = (np.stack([d["g"], d["h"]], 1) if p["objective"] == "given"
          else oracle.gradients(p["objective"], np.zeros(n, np.float32), d["y"]))
    tree, rep = _judge(ctx, oracle, o, gdev, gp, p, n, F, max_leaves)
    n_leaves = (tree["n_nodes"] + 1) // 2
    assert n_leaves <= max_leaves
    _say(f"  nodes={tree['n_nodes']} identical={rep['identical']} ties={len(rep['ties'])}")


def test_lossguide_argument_errors(ctx):
    import paper_1806_11248_amd as g
    d = synth.make(1)
    n, F = d["X"].shape
    cuts, nb, sym, mv, ms = ctx.quantise(dev(d["X"]), max_bins=16)
    packed, bits = ctx.compress(sym, mv)
    gp = dev(np.stack([d["g"], d["h"]], 1))
    params = g.make_params(max_depth=3, max_bins=16)
    with pytest.raises(g.GbtError) as e:
        ctx.grow_tree_lossguide(packed, bits, n, F, ms, nb, cuts, gp, params, 0)
    assert e.value.code == g.binding.EINVAL
    # a tree with too little room is refused before anything runs
    import ctypes as C
    from paper_1806_11248_amd.binding import _ptr, _tree_struct
    t = g.new_tree_leaves(4)
    ws = ctx.workspace("grow", ctx.lib.gbt_grow_tree_lossguide_workspace_bytes(n, F, bits, 16, 8))
    rc = ctx.lib.gbt_grow_tree_lossguide(ctx.h, _ptr(packed), bits, n, F, ms, _ptr(nb), _ptr(cuts), _ptr(gp),
                                         C.byref(params), 8, C.byref(_tree_struct(t)), None, None, _ptr(ws), ws.numel())
    assert rc == g.binding.EINVAL


def test_rounds_of_several_leaves_keep_the_sequential_rule(oracle, monkeypatch):
    """Several open leaves are expanded per round ahead of their turn; with one expansion per round the
    library follows the rule step by step.  Both must give the same tree, node numbers included, also
    when the depth cap stops some of a round's leaves and when the budget ends inside a round."""
    import paper_1806_11248_amd as g
    d = synth.make(4, 150_000)
    n, F = d["X"].shape
    ctxs = []
    for batch in (1, 16, 32):
        monkeypatch.setenv("GBT_TUNE_LOSSGUIDE_BATCH", str(batch))
        ctxs.append(g.Context(0))
    o, gdev = gpu_prep(ctxs[1], oracle, d)
    gp = dev(oracle.gradients("logistic", np.zeros(n, np.float32), d["y"]))
    for max_leaves, depth in ((37, 64), (100, 5), (3, 64), (200, 9)):
        params = g.make_params(max_depth=depth, max_bins=d["params"]["max_bins"])
        print(f"lossguide batches, {max_leaves} leaves, depth cap {depth}", flush=True)
        got = [c.grow_tree_lossguide(gdev["packed"], gdev["bits"], n, F, gdev["missing"], gdev["nb"], gdev["cuts"], gp,
                                     params, max_leaves) for c in ctxs]
        nn = got[0][0]["n_nodes"]
        for t, rows, leaf in got[1:]:
            assert t["n_nodes"] == nn
            for k in ("feature", "bin", "default_left", "left", "right", "n_rows", "threshold", "weight", "gain",
                      "sumG", "sumH"):
                assert np.array_equal(t[k][:nn], got[0][0][k][:nn]), k
            assert torch.equal(rows, got[0][1]) and torch.equal(leaf, got[0][2])
    for c in ctxs:
        c.close()
