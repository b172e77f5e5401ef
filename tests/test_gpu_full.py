"""GPU parity at the workloads' FULL sizes, in the launch configuration bench.py
times (-m gpu).  The oracle checks every row's final position, every node's
totals and leaf weight, the gain the GPU reports for every split, and repeats
the exhaustive best-split search at EVERY node (every leaf included: none may
have had a split due)."""
import time

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


def _full_case(ctx, oracle, cfg, csr, rounds, check_root_hist=True, sparse_rows=False):
    import paper_1806_11248_amd as g
    t0 = time.time()
    d = synth.make(cfg)
    p = d["params"]
    X = d["X"]
    n, F = X.shape
    B = p["max_bins"]
    _say(f"C{cfg} full size {n} x {F}: generated in {time.time() - t0:.1f} s")

    # ---- quantise + compress on the GPU, the oracle's on the CPU
    t0 = time.time()
    if csr:
        indptr, indices, values = synth.dense_to_csr(X)
        cuts, nb, sym, mv, ms = ctx.quantise(csr=(dev(indptr), dev(indices), dev(values)), max_bins=B, n=n, F=F)
        del indptr, indices, values
    else:
        cuts, nb, sym, mv, ms = ctx.quantise(dev(X), max_bins=B)
    packed, bits = ctx.compress(sym, mv)
    torch.cuda.synchronize()
    _say(f"  gpu quantise+compress {time.time() - t0:.2f} s (bits={bits})")
    t0 = time.time()
    o_cuts, o_nb = oracle.cuts(X, B)
    o_sym, o_missing, o_mx = oracle.bin_matrix(X, o_cuts, o_nb)
    _say(f"  oracle quantise {time.time() - t0:.1f} s")
    assert np.array_equal(nb.cpu().numpy(), o_nb)
    assert np.array_equal(cuts.cpu().numpy(), o_cuts)
    assert (mv, ms) == (o_mx, o_missing) and bits == oracle.bits_for(o_mx)
    # symbols: bit-exact, compared in slabs to bound host memory
    step = max(1, (64 << 20) // max(F, 1))
    for lo in range(0, n, step):
        assert np.array_equal(sym[lo:lo + step].cpu().numpy(), o_sym[lo:lo + step]), f"symbols differ in rows {lo}.."
    if sparse_rows:   # the same matrix in the sparse-row form
        sp_rowptr, sp_ent, sp_nnz = ctx.compress_sparse(sym, B, ms)
        assert sp_nnz == int((o_sym != o_missing).sum())
    del sym
    # packed words: whole rows that start on a word boundary, packed by the oracle
    period = 32 // np.gcd(32, F * bits)                # rows per word-aligned group
    words = host_u32(packed)
    rng = np.random.default_rng(cfg)
    for r0 in list(rng.integers(0, max(1, n // period - 64), 6) * period) + [0, (n // period - 1) * period]:
        r0 = int(r0)
        r1 = min(n, r0 + 37 * period)
        w0 = r0 * F * bits // 32
        ref = oracle.pack(o_sym[r0:r1], bits)[:-1]
        if r1 < n and ((r1 - r0) * F * bits) % 32:
            ref = ref[:-1]                              # the last word also holds bits of the next row
        assert np.array_equal(words[w0:w0 + len(ref)], ref)
    assert words[-1] == 0 and len(words) == oracle.packed_words(n * F, bits)
    del words

    margin_gpu = torch.zeros(n, dtype=torch.float32, device="cuda")
    margin_ref = np.zeros(n, np.float32)
    y_t = dev(d["y"])
    params = g.make_params(max_depth=p["max_depth"], max_bins=B, lam=p["lam"], gamma=p["gamma"],
                           min_child_weight=p["min_child_weight"])
    for r in range(rounds):
        gp_ref = oracle.gradients(p["objective"], margin_ref, d["y"])
        gp_t = ctx.gradients(p["objective"], margin_gpu, y_t)
        gp_gpu = gp_t.cpu().numpy()
        assert np.allclose(gp_gpu, gp_ref, rtol=1e-5, atol=1e-6)
        gp_t = dev(gp_ref)                               # the same fp32 pairs feed both sides
        gq, scale = ctx.gpair_fixed(gp_t)
        if check_root_hist and r == 0:
            t0 = time.time()
            h = ctx.build_hist(packed, bits, n, F, B, ms, gq)
            hf = ctx.hist_export_f64(h, scale).cpu().numpy()
            ref, cnt, G, H = oracle.hist(o_sym, B, o_missing, None, gp_ref)
            assert np.all(np.abs(hf - ref) <= hist_tolerance(ref, cnt, scale))
            quantum = 0.5 / np.array(scale)
            big = np.abs(ref) >= np.maximum(cnt, 1)[..., None] * quantum / 1e-5
            assert np.all(np.abs(hf - ref)[big] <= 1e-5 * np.abs(ref)[big])
            _say(f"  root histogram checked in {time.time() - t0:.1f} s ({big[cnt > 0].mean():.3f} of bins to plain 1e-5)")
        del gq
        t0 = time.time()
        tree, row_idx, leaf = ctx.grow_tree(packed, bits, n, F, ms, nb, cuts, gp_t, params)
        torch.cuda.synchronize()
        t_gpu = time.time() - t0
        t0 = time.time()
        rep = oracle.replay_tree(tree, o_sym, o_nb, o_missing, gp_ref, **tree_kw(p),
                                 sum_atol_per_row=0.5 / min(scale))
        _say(f"  round {r}: gpu tree {t_gpu * 1e3:.1f} ms, {tree['n_nodes']} nodes; oracle replay {time.time() - t0:.1f} s, "
             f"{rep['checked_splits']} exhaustive searches, identical={rep['identical']}, ties={len(rep['ties'])}")
        assert rep["ok"], rep["errors"][:5]
        assert np.array_equal(host_u32(row_idx), rep["row_idx"])
        assert np.array_equal(leaf.cpu().numpy(), rep["leaf_of_row"])
        del row_idx, leaf
        if r == 0:   # and in the library's own precision: exact totals and gains, the exhaustive best split at every node
            t0 = time.time()
            judge_on_grid(oracle, oracle.replay_tree, tree, dict(sym=o_sym, nb=o_nb, missing=o_missing), gp_ref, scale,
                          **tree_kw(p))
            _say(f"  judged on the fixed-point grid in {time.time() - t0:.1f} s")
        # the launch configuration the benchmark times: no row order asked for (one-launch partition,
        # with one child's histogram in the same pass where the shape allows) -- the same tree
        t0 = time.time()
        bare, _, leaf2 = ctx.grow_tree(packed, bits, n, F, ms, nb, cuts, gp_t, params, want_rows=False)
        torch.cuda.synchronize()
        nn = tree["n_nodes"]
        assert np.array_equal(leaf2.cpu().numpy(), rep["leaf_of_row"])
        del leaf2
        _say(f"  round {r}: same tree without row ids in {(time.time() - t0) * 1e3:.1f} ms "
             f"(path {ctx.grow_tree_path(F, bits, B, track_rows=False)})")
        assert bare["n_nodes"] == nn
        for k in ("feature", "bin", "default_left", "left", "right", "n_rows", "threshold", "weight", "gain",
                  "sumG", "sumH"):
            assert np.array_equal(bare[k][:nn], tree[k][:nn]), k
        # ... and as bench.py calls it: the whole iteration in one call (gradients of the GPU's own margins, tree,
        # margin update).  Its pairs are the GPU's; where those equal the oracle's bit for bit its tree must be the
        # tree judged above, else the tree the separate calls grow on the same pairs.
        t0 = time.time()
        gp_b = torch.empty((n, 2), dtype=torch.float32, device="cuda")
        m_b = torch.empty_like(margin_gpu)
        bparams = g.make_params(max_depth=p["max_depth"], max_bins=B, lam=p["lam"], gamma=p["gamma"],
                                min_child_weight=p["min_child_weight"], eta=p["eta"], objective=p["objective"])
        tree_b = ctx.boost_round(packed, bits, n, F, ms, nb, cuts, y_t, margin_gpu, m_b, gp_b, bparams)
        torch.cuda.synchronize()
        same_pairs = bool(torch.equal(gp_b, gp_t))
        assert np.array_equal(gp_b.cpu().numpy(), gp_gpu)
        want = bare if same_pairs else ctx.grow_tree(packed, bits, n, F, ms, nb, cuts, gp_b, params, want_rows=False,
                                                     want_leaf=False)[0]
        assert tree_b["n_nodes"] == want["n_nodes"]
        for k in ("feature", "bin", "default_left", "left", "right", "n_rows", "threshold", "weight", "gain",
                  "sumG", "sumH"):
            assert np.array_equal(tree_b[k][:want["n_nodes"]], want[k][:want["n_nodes"]]), k
        m_want = margin_gpu.clone()
        ctx.predict([want], m_want, p["eta"], packed=packed, bits=bits, missing_sym=ms, n=n, F=F)
        assert torch.equal(m_b, m_want)
        del gp_b, m_b, m_want
        _say(f"  round {r}: the same iteration as one call in {(time.time() - t0) * 1e3:.1f} ms "
             f"(pairs {'equal to' if same_pairs else 'differ in rounding from'} the oracle's)")
        if sparse_rows:   # the sparse-row kernels: the same tree, row order and leaves, the same margins
            t0 = time.time()
            st, s_rows, s_leaf = ctx.grow_tree_sparse(sp_rowptr, sp_ent, n, sp_nnz, F, nb, cuts, gp_t, params)
            torch.cuda.synchronize()
            _say(f"  round {r}: same tree over sparse rows in {(time.time() - t0) * 1e3:.1f} ms")
            assert st["n_nodes"] == nn
            for k in ("feature", "bin", "default_left", "left", "right", "n_rows", "threshold", "weight", "gain",
                      "sumG", "sumH"):
                assert np.array_equal(st[k][:nn], tree[k][:nn]), k
            assert np.array_equal(host_u32(s_rows), rep["row_idx"])
            assert np.array_equal(s_leaf.cpu().numpy(), rep["leaf_of_row"])
            del s_rows, s_leaf
            m2 = margin_gpu.clone()
            ctx.predict_sparse([tree], m2, p["eta"], sp_rowptr, sp_ent, n, F, B)
        ctx.predict([tree], margin_gpu, p["eta"], packed=packed, bits=bits, missing_sym=ms, n=n, F=F)
        if sparse_rows:
            assert torch.equal(m2, margin_gpu)
            del m2
        margin_ref = oracle.predict_sym(tree, o_sym, o_missing, p["eta"], margin_ref)
        assert np.allclose(margin_gpu.cpu().numpy(), margin_ref, rtol=1e-5, atol=1e-6)


def test_full_c2_lossguide(ctx, oracle):
    """Loss-guided growth (Sec. 2.3) at C2's full size, 64 leaves, judged by the oracle's replay."""
    import paper_1806_11248_amd as g
    d = synth.make(2)
    p = dict(d["params"], max_depth=12)
    X = d["X"]
    n, F = X.shape
    B = p["max_bins"]
    _say(f"full C2 loss-guided: {n} x {F}, 64 leaves")
    cuts, nb, sym, mv, ms = ctx.quantise(dev(X), max_bins=B)
    packed, bits = ctx.compress(sym, mv)
    del sym
    o_cuts, o_nb = oracle.cuts(X, B)
    o_sym, o_missing, o_mx = oracle.bin_matrix(X, o_cuts, o_nb)
    assert np.array_equal(cuts.cpu().numpy(), o_cuts) and ms == o_missing
    gp = oracle.gradients(p["objective"], np.zeros(n, np.float32), d["y"])
    gp_t = dev(gp)
    params = g.make_params(max_depth=12, max_bins=B, lam=p["lam"], gamma=p["gamma"],
                           min_child_weight=p["min_child_weight"])
    for want_rows in (True, False):
        t0 = time.time()
        tree, row_idx, leaf = ctx.grow_tree_lossguide(packed, bits, n, F, ms, nb, cuts, gp_t, params, 64,
                                                      want_rows=want_rows)
        torch.cuda.synchronize()
        _say(f"  gpu tree (row ids {want_rows}) {1e3 * (time.time() - t0):.1f} ms, {tree['n_nodes']} nodes")
        if want_rows:
            _, scale = ctx.gpair_fixed(gp_t)
            rep = oracle.replay_tree_lossguide(tree, o_sym, o_nb, o_missing, gp, max_leaves=64, **tree_kw(p),
                                               sum_atol_per_row=0.5 / min(scale))
            assert rep["ok"], rep["errors"][:5]
            assert np.array_equal(host_u32(row_idx), rep["row_idx"])
            assert np.array_equal(leaf.cpu().numpy(), rep["leaf_of_row"])
            first = tree
        else:
            nn = first["n_nodes"]
            assert tree["n_nodes"] == nn
            for k in ("feature", "bin", "default_left", "left", "right", "n_rows", "weight", "gain"):
                assert np.array_equal(tree[k][:nn], first[k][:nn]), k


def test_full_c2_dense_classification(ctx, oracle):
    _full_case(ctx, oracle, 2, csr=False, rounds=10)


def test_full_c3_sparse_regression(ctx, oracle):
    _full_case(ctx, oracle, 3, csr=True, rounds=5, sparse_rows=True)


def test_full_c5_wide(ctx, oracle):
    _full_case(ctx, oracle, 5, csr=False, rounds=1)


def test_full_c4_large_tabular(ctx, oracle):
    _full_case(ctx, oracle, 4, csr=False, rounds=1)
