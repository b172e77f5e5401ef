"""GPU parity of the sparse-row storage form (Sec. 1: sparse input; Sec. 2.2: compressed storage)
against the CPU oracle (-m gpu).  The oracle knows nothing of the layout: it works on the dense
symbol matrix with its missing symbol, and the sparse rows must give the same histograms,
partitions and trees."""
import numpy as np
import pytest
import torch

import synth
from gpu_util import dev, hist_tolerance, host_u32, judge_on_grid, tree_kw

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    import paper_1806_11248_amd as g
    c = g.Context(0)
    yield c
    c.close()


def _say(msg):
    print(msg, flush=True)


def sparse_case(seed, n, F, B, miss):
    rng = np.random.default_rng(seed)
    nb = rng.integers(max(1, B // 2), B + 1, F).astype(np.int32)
    nb[0] = B
    missing = int(nb.max())
    sym = np.stack([rng.integers(0, nb[f], n) for f in range(F)], 1).astype(np.uint16)
    sym[rng.random((n, F)) < miss] = missing
    if F > 2:
        sym[:, 2] = missing                      # a feature with nothing present
    if n > 10:
        sym[3, :] = missing                      # an empty row
        sym[n - 1, :] = np.minimum(nb - 1, 1)    # a full last row
    gp = np.stack([rng.standard_normal(n), rng.random(n) * 0.9 + 0.1], 1).astype(np.float32)
    return sym, nb, missing, gp


def reference_rows(sym, B, missing):
    """The layout written out on the CPU: ascending global bin ids of the present elements."""
    n, F = sym.shape
    present = sym != missing
    rowptr = np.zeros(n + 1, np.int64)
    np.cumsum(present.sum(1), out=rowptr[1:])
    gid = (np.arange(F, dtype=np.int64)[None, :] * B + sym.astype(np.int64))[present]   # row-major: ascending per row
    return rowptr, gid.astype(np.uint16 if F * B <= 65536 else np.uint32)   # wider matrices: 32-bit ids


LAYOUT_CASES = [  # n, F, B, miss
    (20_011, 50, 256, 0.8),
    (5_000, 13, 256, 0.0),       # nothing missing: every row has F entries
    (3_000, 200, 64, 0.95),
    (4_099, 7, 1000, 0.5),
    (1, 3, 4, 0.0),
    (70, 5, 16, 1.0),            # nothing present at all
    (6_007, 300, 256, 0.9),      # 76,800 global bin ids: 32-bit entries, the histogram in id-range tiles
    (2_500, 1100, 64, 0.97),     # 70,400 ids over many features
    (1_201, 90, 1000, 0.0),      # 90,000 ids, every row with 90 entries
    (40, 257, 256, 1.0),         # 32-bit entries, nothing present
]


@pytest.mark.parametrize("n,F,B,miss", LAYOUT_CASES)
def test_compress_sparse_and_hist(ctx, oracle, n, F, B, miss):
    sym, nb, missing, gp = sparse_case(n + F, n, F, B, miss)
    _say(f"sparse rows n={n} F={F} B={B} miss={miss}")
    rowptr, ent, nnz = ctx.compress_sparse(dev(sym), B, missing)
    ref_ptr, ref_ent = reference_rows(sym, B, missing)
    assert nnz == ref_ptr[-1]
    assert np.array_equal(host_u32(rowptr).astype(np.int64), ref_ptr)
    assert ent.element_size() == ref_ent.itemsize
    assert np.array_equal(ent.cpu().view(torch.int16 if ref_ent.itemsize == 2 else torch.int32).numpy()[:nnz].view(ref_ent.dtype),
                          ref_ent)
    gq, scale = ctx.gpair_fixed(dev(gp))
    for b, m in ((0, n), (n // 3, n - n // 3 - n // 5), (n // 2, 1 if n > 1 else 0), (0, 0)):
        rows = np.arange(b, b + m, dtype=np.uint32)
        h = ctx.build_hist_sparse(rowptr, ent, n, F, B, gq, row_begin=b, n_rows=m)
        assert torch.equal(h, ctx.build_hist_sparse(rowptr, ent, n, F, B, gq, row_begin=b, n_rows=m))
        ref, cnt, G, H = oracle.hist(sym, B, missing, rows, gp)
        hf = ctx.hist_export_f64(h, scale).cpu().numpy()
        assert np.all(np.abs(hf - ref) <= hist_tolerance(ref, cnt, scale))
        # the fixed-point sums themselves, exactly: the dense-layout kernel on the packed matrix
        bits = oracle.bits_for(int(sym.max()))
        packed = dev(oracle.pack(sym, bits).view(np.int32))
        hd = ctx.build_hist(packed, bits, n, F, B, missing, gq, dev(rows.view(np.int32)))
        assert torch.equal(h, hd)


def test_sparse_hist_extreme_pile_up(ctx, oracle):
    """Same-sign extreme pairs piled into single bins: carries and wraps of the packed LDS word."""
    n, F, B = 2_000_003, 4, 64
    rng = np.random.default_rng(8)
    sym = np.full((n, F), B, np.uint16)
    sym[:, 0] = 0
    sym[:, 1] = rng.integers(0, 2, n) * (B - 1)
    sym[:, 3] = np.where(rng.random(n) < 0.3, np.arange(n) % B, B)
    g = np.where(rng.random(n) < 0.5, 1.999, 1.5).astype(np.float32)
    g[n // 2:] *= -1.0
    h = np.where(rng.random(n) < 0.5, 1.999, 0.7).astype(np.float32)
    gp = np.stack([g, h], 1)
    rowptr, ent, nnz = ctx.compress_sparse(dev(sym), B, B)
    gq, scale = ctx.gpair_fixed(dev(gp))
    _say("sparse hist extreme pile-up")
    hi = ctx.build_hist_sparse(rowptr, ent, n, F, B, gq).cpu().numpy()
    hq = gq.cpu().numpy().astype(np.int64)
    for f in range(F):
        ok = sym[:, f] != B
        for c in range(2):
            want = np.zeros(B, np.int64)
            np.add.at(want, sym[ok, f], hq[ok, c])
            assert np.array_equal(hi[f, :, c], want)


TREE_CASES = [  # config, rows, kwargs, max_depth override
    (3, 30_000, {"F": 300}, None),        # 300 x 256 = 76,800 global bin ids: 32-bit entries, 80% missing
    (5, 6_000, {"F": 1200}, 6),           # 76,800 ids, nothing missing: rows of 1200 entries (no tile fits LDS)
    (3, 60_000, {}, None),                # the sparse workload: 50 features, 80% missing, depth 8
    (3, 9_000, {}, 11),                   # deep: more than 256 leaves, tiny nodes, many leaves above the last level
    (2, 40_000, {}, 13),                  # a tree too large for the walk's LDS: nodes are read from memory
    (4, 100_000, {}, 6),                  # nothing missing: 13 entries in every row
    (2, 30_000, {}, None),                # 28 features, dense
]


@pytest.mark.parametrize("cfg,n,kw,depth", TREE_CASES)
def test_sparse_tree_matches_oracle(ctx, oracle, cfg, n, kw, depth):
    import paper_1806_11248_amd as g
    from test_gpu_tree import gpu_prep
    d = synth.make(cfg, n, **kw)
    p = dict(d["params"])
    if depth is not None:
        p["max_depth"] = depth
    X = d["X"]
    n, F = X.shape
    B = p["max_bins"]
    _say(f"sparse tree C{cfg} n={n} F={F} depth={p['max_depth']}")
    o, gdev = gpu_prep(ctx, oracle, d)
    sym_t = dev(o["sym"])
    rowptr, ent, nnz = ctx.compress_sparse(sym_t, B, gdev["missing"])
    gp = (np.stack([d["g"], d["h"]], 1) if p["objective"] == "given"
          else oracle.gradients(p["objective"], np.zeros(n, np.float32), d["y"]))
    gp_t = dev(gp)
    params = g.make_params(max_depth=p["max_depth"], max_bins=B, lam=p["lam"], gamma=p["gamma"],
                           min_child_weight=p["min_child_weight"])
    tree, row_idx, leaf = ctx.grow_tree_sparse(rowptr, ent, n, nnz, F, gdev["nb"], gdev["cuts"], gp_t, params)
    _, scale = ctx.gpair_fixed(gp_t)
    judge_on_grid(oracle, oracle.replay_tree, tree, o, gp, scale, **tree_kw(p))
    rep = oracle.replay_tree(tree, o["sym"], o["nb"], o["missing"], gp, **tree_kw(p),
                             sum_atol_per_row=0.5 / min(scale))
    assert rep["ok"], rep["errors"][:5]
    assert np.array_equal(host_u32(row_idx), rep["row_idx"])           # partitions: bit-exact
    assert np.array_equal(leaf.cpu().numpy(), rep["leaf_of_row"])
    nn = tree["n_nodes"]
    _say(f"  nodes={nn} identical={rep['identical']} ties={len(rep['ties'])}")
    # the dense-layout path grows the very same tree (integer sums: equal to the last bit)
    dense, _, _ = ctx.grow_tree(gdev["packed"], gdev["bits"], n, F, gdev["missing"], gdev["nb"], gdev["cuts"], gp_t,
                                params, want_rows=False, want_leaf=False)
    assert dense["n_nodes"] == nn
    for k in ("feature", "bin", "default_left", "left", "right", "n_rows", "threshold", "weight", "gain",
              "sumG", "sumH"):
        assert np.array_equal(dense[k][:nn], tree[k][:nn]), k
    # tree only
    bare, r2, l2 = ctx.grow_tree_sparse(rowptr, ent, n, nnz, F, gdev["nb"], gdev["cuts"], gp_t, params,
                                        want_leaf=False, want_rows=False)
    assert r2 is None and l2 is None and bare["n_nodes"] == nn
    assert np.array_equal(bare["feature"][:nn], tree["feature"][:nn])
    # prediction over the sparse rows: the oracle's margins
    m0 = np.zeros(n, np.float32)
    ref = oracle.predict_sym(tree, o["sym"], o["missing"], 0.3, m0)
    got = ctx.predict_sparse([tree, tree], dev(m0), 0.3, rowptr, ent, n, F, B).cpu().numpy()
    ref2 = oracle.predict_sym(tree, o["sym"], o["missing"], 0.3, ref)
    assert np.array_equal(got, ref2)


def test_sparse_tree_depth_zero(ctx, oracle):
    import paper_1806_11248_amd as g
    sym, nb, missing, gp = sparse_case(3, 5_000, 6, 32, 0.5)
    rowptr, ent, nnz = ctx.compress_sparse(dev(sym), 32, missing)
    params = g.make_params(max_depth=0, max_bins=32)
    cuts = dev(np.tile(np.arange(1, 32, dtype=np.float32), (6, 1)))
    tree, row_idx, leaf = ctx.grow_tree_sparse(rowptr, ent, 5_000, nnz, 6, dev(nb), cuts, dev(gp), params)
    assert tree["n_nodes"] == 1 and tree["n_rows"][0] == 5_000
    assert np.array_equal(host_u32(row_idx), np.arange(5_000, dtype=np.uint32)) and not leaf.any()


def test_sparse_argument_errors(ctx):
    import paper_1806_11248_amd as g
    from paper_1806_11248_amd import binding
    sym = dev(np.zeros((10, 5000), np.uint16))
    with pytest.raises(g.GbtError) as e:
        ctx.compress_sparse(sym, 60_000, 60_000)    # 3 * 10^8 global bin ids: more than the form takes
    assert e.value.code == binding.EUNSUPPORTED
    assert ctx.lib.gbt_sparse_entry_bytes(256, 256) == 2 and ctx.lib.gbt_sparse_entry_bytes(257, 256) == 4
    assert ctx.lib.gbt_sparse_entry_bytes(5000, 60_000) == 0
