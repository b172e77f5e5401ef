"""GPU parity, one C-ABI call at a time, against the CPU oracle (-m gpu)."""
import numpy as np
import pytest
import torch

import grid
import synth
from gpu_util import dev, hist_tolerance, host_u32, oracle_prep

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    import paper_1806_11248_amd as g
    c = g.Context(0)
    yield c
    c.close()


def _say(msg):
    print(msg, flush=True)


# ------------------------------------------------------------------ gradients --
@pytest.mark.parametrize("objective", ["logistic", "squared"])
def test_gradients(ctx, oracle, objective):
    rng = np.random.default_rng(0)
    n = 100_003
    m = (rng.standard_normal(n) * 3).astype(np.float32)
    y = (rng.random(n) < 0.5).astype(np.float32) if objective == "logistic" else rng.standard_normal(n).astype(np.float32)
    _say(f"gradients {objective} n={n}")
    gp = ctx.gradients(objective, dev(m), dev(y)).cpu().numpy()
    ref = oracle.gradients(objective, m, y)
    assert np.allclose(gp, ref, rtol=1e-6, atol=1e-7)
    assert (gp != ref).mean() < 1e-3      # both sides evaluate in fp64 and round once
    assert ctx.gradients(objective, dev(m[:0]), dev(y[:0])).shape == (0, 2)
    # arrays that do not start on a 16-byte boundary, and lengths around the four instances a thread takes at once
    mt, yt = dev(m), dev(y)
    for off, k in ((1, 1), (1, 6), (2, 4099), (3, 1001), (0, 3), (0, 7)):
        out = torch.empty((k + 1, 2), dtype=torch.float32, device="cuda")[1:] if off & 1 else None
        got = ctx.gradients(objective, mt[off:off + k], yt[off:off + k], out=out).cpu().numpy()
        assert np.array_equal(got, gp[off:off + k]), (off, k)


# ------------------------------------------------------------------- quantise --
def _quantise_case(seed, n, F, B):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((n, F)).astype(np.float32)
    X[:, 1] = np.round(X[:, 1] * 2)                    # few distinct values
    if F > 2:
        X[:, 2] = np.abs(np.where(rng.random(n) < 0.7, 0.0, X[:, 2]))   # a huge tie at the minimum
    if F > 3:
        X[:, 3] = rng.integers(0, 1000, n)             # integer valued, more distinct than bins
    X[rng.random((n, F)) < 0.1] = np.nan
    if F > 4:
        X[:, 4] = np.nan                               # nothing present
    if F > 5:
        X[:, 5] = 7.25                                 # one value
    return X


@pytest.mark.parametrize("n,F,B", [(5000, 8, 16), (70_001, 13, 256), (9_000, 70, 64), (300, 3, 256), (1, 2, 4)])
def test_quantise_dense(ctx, oracle, n, F, B):
    X = _quantise_case(n + F, n, F, B)
    _say(f"quantise dense n={n} F={F} B={B}")
    cuts, nb, sym, mv, ms = ctx.quantise(dev(X), max_bins=B)
    o = oracle_prep(oracle, X, B)
    assert np.array_equal(nb.cpu().numpy(), o["nb"])
    assert np.array_equal(cuts.cpu().numpy(), o["cuts"])
    assert (mv, ms) == (o["max_value"], o["missing"])
    assert np.array_equal(sym.cpu().numpy(), o["sym"])


def test_quantise_csr_matches_dense_oracle(ctx, oracle):
    d = synth.make(3, 30_011)
    X = d["X"]
    indptr, indices, values = synth.dense_to_csr(X)
    _say(f"quantise csr n={X.shape[0]} nnz={len(values)}")
    cuts, nb, sym, mv, ms = ctx.quantise(csr=(dev(indptr), dev(indices), dev(values)), max_bins=256,
                                         n=X.shape[0], F=X.shape[1])
    o = oracle_prep(oracle, X, 256)
    assert np.array_equal(nb.cpu().numpy(), o["nb"])
    assert np.array_equal(cuts.cpu().numpy(), o["cuts"])
    assert (mv, ms) == (o["max_value"], o["missing"]) and o["bits"] == 9
    assert np.array_equal(sym.cpu().numpy(), o["sym"])


def test_quantise_csr_with_nothing_stored(ctx, oracle):
    # every value missing: the index and value arrays are empty (no address to give), all symbols are the missing one
    n, F = 37, 5
    X = np.full((n, F), np.nan, np.float32)
    indptr, indices, values = synth.dense_to_csr(X)
    assert len(values) == 0
    cuts, nb, sym, mv, ms = ctx.quantise(csr=(dev(indptr), dev(indices), dev(values)), max_bins=16, n=n, F=F)
    o = oracle_prep(oracle, X, 16)
    assert np.array_equal(nb.cpu().numpy(), o["nb"]) and np.array_equal(cuts.cpu().numpy(), o["cuts"])
    assert (mv, ms) == (o["max_value"], o["missing"]) == (1, 1)
    assert np.array_equal(sym.cpu().numpy(), o["sym"])


# ------------------------------------------------- quantise + compress in one call --
@pytest.mark.parametrize("n,F,B,nan", [(5000, 8, 16, True), (70_001, 13, 256, True), (9_000, 70, 64, True),
                                       (300, 3, 256, False), (1, 2, 4, False), (4096, 1, 2, False), (4097, 5, 255, False),
                                       (12_289, 31, 1000, True), (2_000, 600, 8, False)])
def test_quantise_packed_dense(ctx, oracle, n, F, B, nan):
    """Cuts and bit stream of the one-call form: equal to the oracle's cuts, symbols and packing, bit for bit, and to
    gbt_quantise followed by gbt_compress; with and without missing values (the width depends on whether the
    missing symbol occurs), tiles that end inside a word."""
    X = _quantise_case(n + F, n, F, B) if nan else np.random.default_rng(n + F).standard_normal((n, F)).astype(np.float32)
    _say(f"quantise+pack dense n={n} F={F} B={B} missing={nan}")
    cuts, nb, packed, bits, mv, ms = ctx.quantise_packed(dev(X), max_bins=B)
    o = oracle_prep(oracle, X, B)
    assert np.array_equal(nb.cpu().numpy(), o["nb"])
    assert np.array_equal(cuts.cpu().numpy(), o["cuts"])
    assert (mv, ms, bits) == (o["max_value"], o["missing"], o["bits"])
    assert np.array_equal(host_u32(packed), oracle.pack(o["sym"], o["bits"]))
    _, _, sym, mv2, _ = ctx.quantise(dev(X), max_bins=B)
    packed2, bits2 = ctx.compress(sym, mv2)
    assert bits2 == bits and torch.equal(packed2, packed)


@pytest.mark.parametrize("cfg,n,kw", [(3, 30_011, {}), (3, 257, {}), (2, 5_000, {})])
def test_quantise_packed_csr(ctx, oracle, cfg, n, kw):
    d = synth.make(cfg, n, **kw)
    X = d["X"]
    indptr, indices, values = synth.dense_to_csr(X)
    _say(f"quantise+pack csr n={X.shape[0]} F={X.shape[1]} nnz={len(values)}")
    cuts, nb, packed, bits, mv, ms = ctx.quantise_packed(csr=(dev(indptr), dev(indices), dev(values)), max_bins=256,
                                                         n=X.shape[0], F=X.shape[1])
    o = oracle_prep(oracle, X, 256)
    assert np.array_equal(nb.cpu().numpy(), o["nb"]) and np.array_equal(cuts.cpu().numpy(), o["cuts"])
    assert (mv, ms, bits) == (o["max_value"], o["missing"], o["bits"])
    assert np.array_equal(host_u32(packed), oracle.pack(o["sym"], o["bits"]))


def test_quantise_packed_refuses_what_it_cannot_do(ctx):
    import paper_1806_11248_amd as g
    n, F = 64, 1200          # CSR rows too wide for the packing tile
    X = np.random.default_rng(0).standard_normal((n, F)).astype(np.float32)
    indptr, indices, values = synth.dense_to_csr(X)
    with pytest.raises(g.GbtError) as e:
        ctx.quantise_packed(csr=(dev(indptr), dev(indices), dev(values)), max_bins=16, n=n, F=F)
    assert e.value.code == g.binding.EUNSUPPORTED


# ------------------------------------------------------------------- compress --
@pytest.mark.parametrize("bits", list(range(1, 17)))
def test_compress(ctx, oracle, bits):
    rng = np.random.default_rng(bits)
    n, F = 1237, 13
    sym = rng.integers(0, 1 << bits, (n, F)).astype(np.uint16)
    sym[0, 0] = (1 << bits) - 1
    _say(f"compress bits={bits}")
    packed, b = ctx.compress(dev(sym), int(sym.max()))
    assert b == bits == oracle.bits_for(int(sym.max()))
    assert np.array_equal(host_u32(packed), oracle.pack(sym, bits))


def test_compress_empty_and_errors(ctx):
    import paper_1806_11248_amd as g
    packed, b = ctx.compress(ctx.empty((0, 5), torch.uint16), 3)
    assert b == 2 and packed.numel() == 1
    with pytest.raises(g.GbtError) as e:
        ctx.compress(ctx.empty((4, 5), torch.uint16), 1 << 16)     # needs 17 bits
    assert e.value.code == g.binding.EUNSUPPORTED


# ------------------------------------------------------------------ histogram --
def _node_case(seed, n, F, B, bits_target, miss):
    rng = np.random.default_rng(seed)
    nb = rng.integers(max(1, B // 2), B + 1, F).astype(np.int32)
    nb[0] = B
    missing = int(nb.max())
    sym = np.stack([rng.integers(0, nb[f], n) for f in range(F)], 1).astype(np.uint16)
    # a heavy bin, like a skewed categorical column
    heavy = rng.random(n) < 0.4
    sym[heavy, F - 1] = 0
    if miss > 0:
        sym[rng.random((n, F)) < miss] = missing
        if F > 2:
            sym[:, 2] = missing               # a feature with nothing present
    gp = np.stack([rng.standard_normal(n), rng.random(n) * 0.9 + 0.1], 1).astype(np.float32)
    return sym, nb, missing, gp


HIST_CASES = [
    # n, F, B, miss
    (10_000, 8, 16, 0.0),        # 4-bit
    (50_003, 13, 256, 0.0),      # 8-bit, rows of 13 bytes
    (20_001, 28, 256, 0.0),      # 8-bit, 112 KB of LDS
    (30_007, 50, 256, 0.8),      # 9-bit with the missing symbol, two feature tiles
    (5_003, 300, 64, 0.0),       # 6-bit, several feature tiles
    (3_001, 400, 64, 0.0),       # 6-bit, rows of 300 bytes: lanes share a row
    (2_003, 260, 256, 0.5),      # 9-bit wide rows with the missing symbol
    (4_097, 7, 1000, 0.1),       # 10-bit
    (63, 3, 2, 0.0),             # 1-bit, less than a wave
]


@pytest.mark.parametrize("n,F,B,miss", HIST_CASES)
def test_build_hist(ctx, oracle, n, F, B, miss):
    sym, nb, missing, gp = _node_case(n * 7 + F, n, F, B, None, miss)
    bits = oracle.bits_for(int(sym.max()))
    words = oracle.pack(sym, bits)
    _say(f"build_hist n={n} F={F} B={B} bits={bits} missing={missing}")
    packed = dev(words.view(np.int32))
    gq, scale = ctx.gpair_fixed(dev(gp))
    rng = np.random.default_rng(n)
    subset = np.sort(rng.choice(n, max(1, n // 3), replace=False)).astype(np.uint32)
    for rows in (None, subset, subset[:1], subset[:0]):
        rows_t = None if rows is None else dev(rows.view(np.int32))
        h = ctx.build_hist(packed, bits, n, F, B, missing, gq, rows_t)
        h2 = ctx.build_hist(packed, bits, n, F, B, missing, gq, rows_t)
        assert torch.equal(h, h2)                      # integer sums: run-to-run identical
        hf = ctx.hist_export_f64(h, scale).cpu().numpy()
        ref, cnt, G, H = oracle.hist(sym, B, missing, rows, gp)
        assert np.all(np.abs(hf - ref) <= hist_tolerance(ref, cnt, scale))
        # plain 1e-5 relative holds wherever the bin's |mean| is at least 5e4 quanta
        quantum = 0.5 / np.array(scale)
        big = np.abs(ref) >= np.maximum(cnt, 1)[..., None] * quantum / 1e-5
        if rows is None and n > 1000:
            assert big[cnt > 0].mean() > 0.5
        assert np.all(np.abs(hf - ref)[big] <= 1e-5 * np.abs(ref)[big])
        Gq, Hq = ctx.sum_gpair(gq, rows_t)
        nr = n if rows is None else len(rows)
        assert abs(Gq / scale[0] - G) <= 1e-5 * abs(G) + nr * 0.5 / scale[0]
        assert abs(Hq / scale[1] - H) <= 1e-5 * abs(H) + nr * 0.5 / scale[1]
        # bins + missing mass = node total, exactly in fixed point
        hi = h.cpu().numpy()
        for f in range(F):
            s = sym[:, f] if rows is None else sym[rows, f]
            if not (s == missing).any():
                assert hi[f, :, 0].sum() == Gq and hi[f, :, 1].sum() == Hq


@pytest.mark.parametrize("bits_case", ["b8", "b3"])
def test_build_hist_many_rows_in_one_bin(ctx, oracle, bits_case):
    # Extreme, same-sign gradient pairs piled into single bins: the sums pass the
    # range of any 32-bit partial accumulator many times over and must stay exact.
    n, F = 3_000_017, 3
    B = 256 if bits_case == "b8" else 8
    rng = np.random.default_rng(3)
    sym = np.zeros((n, F), np.uint16)
    sym[:, 1] = rng.integers(0, 2, n) * (B - 1)
    sym[:, 2] = np.arange(n) % B
    gmag = np.where(rng.random(n) < 0.5, 1.999, 1.5).astype(np.float32)
    g = gmag.copy()
    g[n // 2:] *= -1.0                                   # long runs of one sign, then the other
    h = np.where(rng.random(n) < 0.5, 1.999, 0.7).astype(np.float32)
    gp = np.stack([g, h], 1)
    bits = oracle.bits_for(int(sym.max()))
    packed = dev(oracle.pack(sym, bits).view(np.int32))
    gq, scale = ctx.gpair_fixed(dev(gp))
    _say(f"hist extreme pile-up bits={bits}")
    hq = gq.cpu().numpy().astype(np.int64)
    for rows in (None, np.arange(0, n, 2, dtype=np.uint32)):
        rows_t = None if rows is None else dev(rows.view(np.int32))
        hi = ctx.build_hist(packed, bits, n, F, B, B, gq, rows_t).cpu().numpy()
        ref, cnt, G, H = oracle.hist(sym, B, B, rows, gp)
        hf = hi / np.array(scale)
        assert np.all(np.abs(hf - ref) <= 1e-5 * np.abs(ref) + cnt[..., None] * 0.5 / np.array(scale) + 1e-300)
        sel = slice(None) if rows is None else rows
        for f in range(F):                               # the fixed-point sums themselves, exactly
            for c in range(2):
                want = np.bincount(sym[sel, f], weights=None, minlength=B) * 0
                want = np.zeros(B, np.int64)
                np.add.at(want, sym[sel, f], hq[sel, c])
                assert np.array_equal(hi[f, :, c], want)


def test_sibling_subtraction_is_exact(ctx, oracle):
    n, F, B = 40_000, 13, 256
    sym, nb, missing, gp = _node_case(5, n, F, B, None, 0.05)
    bits = oracle.bits_for(int(sym.max()))
    packed = dev(oracle.pack(sym, bits).view(np.int32))
    gq, scale = ctx.gpair_fixed(dev(gp))
    rows = np.arange(n, dtype=np.uint32)
    out, nl = oracle.partition(sym, rows, 0, 100, 1, missing)
    _say("sibling subtraction")
    hp = ctx.build_hist(packed, bits, n, F, B, missing, gq, None)
    hl = ctx.build_hist(packed, bits, n, F, B, missing, gq, dev(out[:nl].view(np.int32)))
    hr = ctx.build_hist(packed, bits, n, F, B, missing, gq, dev(out[nl:].view(np.int32)))
    assert torch.equal(ctx.hist_subtract(hp, hl), hr)
    assert torch.equal(ctx.hist_subtract(hp, hr), hl)


def test_gpair_fixed_scale_and_errors(ctx, oracle):
    import paper_1806_11248_amd as g
    gp = np.array([[0.75, 0.25], [-3.0, 0.0], [1e-3, 1.0]], np.float32)
    gq, scale = ctx.gpair_fixed(dev(gp))
    assert scale == (2.0 ** 24, 2.0 ** 21)            # 3.0 < 2^2, 1.0 < 2^1: |g|*scale <= 2^26, h*scale <= 2^22
    assert np.array_equal(gq.cpu().numpy(), np.rint(gp.astype(np.float64) * np.array(scale)).astype(np.int32))
    # the oracle's restatement of the grid, on ties, tiny and huge magnitudes
    rng = np.random.default_rng(9)
    for sg, sh in ((1.0, 1.0), (3e-7, 2e5), (9e6, 1e-4)):
        gp2 = np.stack([rng.standard_normal(70_001) * sg, rng.uniform(0, 1, 70_001) * sh], 1).astype(np.float32)
        gp2[5] = [2.5 * 2.0 ** -25 * sg, 3.5 * 2.0 ** -21 * sh]
        gq, scale = ctx.gpair_fixed(dev(gp2))
        q, scale_o = grid.fixed_point(gp2)
        assert scale == scale_o and np.array_equal(gq.cpu().numpy(), q)
    bad = gp.copy(); bad[1, 0] = np.inf
    with pytest.raises(g.GbtError) as e:
        ctx.gpair_fixed(dev(bad))
    assert e.value.code == g.binding.EINVAL
    bad = gp.copy(); bad[2, 1] = -0.5                  # hessians must not be negative
    with pytest.raises(g.GbtError) as e:
        ctx.gpair_fixed(dev(bad))
    assert e.value.code == g.binding.EINVAL
    gq, scale = ctx.gpair_fixed(dev(np.zeros((5, 2), np.float32)))
    assert scale == (1.0, 1.0) and not gq.any()


@pytest.mark.parametrize("n", [1, 2, 7, 4096, 100_003, 2_500_001])
@pytest.mark.parametrize("src_off,dst_off", [(0, 0), (1, 0), (1, 1), (0, 1)])
def test_gpair_fixed_any_alignment(ctx, n, src_off, dst_off):
    """Pairs are 8 bytes; the kernels work in 16-byte pieces and must serve pointers of either
    alignment, on both sides, with odd and even counts."""
    import ctypes as C
    from paper_1806_11248_amd.binding import _ptr
    rng = np.random.default_rng(n * 4 + src_off * 2 + dst_off)
    gp = np.stack([rng.normal(0, 2, n), rng.uniform(0, 1, n)], 1).astype(np.float32)
    src = torch.zeros((n + 1, 2), dtype=torch.float32, device="cuda")
    src[src_off:src_off + n] = torch.from_numpy(gp).cuda()
    dst = torch.full((n + 2, 2), -7, dtype=torch.int32, device="cuda")
    scale = (C.c_double * 2)()
    ws = ctx.workspace("small", 4096)
    _say(f"gpair_fixed n={n} src+{src_off} dst+{dst_off}")
    ctx._check(ctx.lib.gbt_gpair_fixed(ctx.h, _ptr(src[src_off:]), n, _ptr(dst[dst_off:]), scale, _ptr(ws), ws.numel()))
    want = np.rint(gp.astype(np.float64) * np.array([scale[0], scale[1]])).astype(np.int32)
    got = dst.cpu().numpy()
    assert np.array_equal(got[dst_off:dst_off + n], want)
    assert (got[:dst_off] == -7).all() and (got[dst_off + n:] == -7).all()      # nothing written outside
    sums = ctx.sum_gpair(dst[dst_off:dst_off + n].contiguous())
    assert sums == (int(want[:, 0].astype(np.int64).sum()), int(want[:, 1].astype(np.int64).sum()))


# ---------------------------------------------------------------------- split --
@pytest.mark.parametrize("n,F,B,miss", [(10_000, 8, 16, 0.0), (30_007, 50, 256, 0.8), (5_003, 300, 64, 0.0),
                                        (700, 5, 256, 0.3)])
@pytest.mark.parametrize("lam,mcw", [(1.0, 1.0), (0.0, 5.0)])
def test_eval_split(ctx, oracle, n, F, B, miss, lam, mcw):
    import paper_1806_11248_amd as g
    sym, nb, missing, gp = _node_case(n + 1, n, F, B, None, miss)
    bits = oracle.bits_for(int(sym.max()))
    packed = dev(oracle.pack(sym, bits).view(np.int32))
    gq, scale = ctx.gpair_fixed(dev(gp))
    _say(f"eval_split n={n} F={F} B={B} lam={lam} mcw={mcw}")
    h = ctx.build_hist(packed, bits, n, F, B, missing, gq, None)
    Gq, Hq = ctx.sum_gpair(gq)
    sp = ctx.eval_split(h, dev(nb), Gq, Hq, scale, g.make_params(max_depth=1, max_bins=B, lam=lam, min_child_weight=mcw))
    ref_h, cnt, G, H = oracle.hist(sym, B, missing, None, gp)
    ref = oracle.eval_split(ref_h, cnt, nb, G, H, n, lam, mcw)
    assert bool(sp["valid"]) == bool(ref["valid"])
    if not ref["valid"]:
        return
    same = (sp["feature"], sp["bin"], sp["default_left"]) == (ref["feature"], ref["bin"], ref["default_left"])
    g_own, sides = oracle.candidate_gain(ref_h, sp["feature"], sp["bin"], sp["default_left"], G, H, lam, mcw,
                                         cnt=cnt, n_rows=n)
    assert same or abs(g_own - ref["gain"]) <= 1e-6 * abs(ref["gain"])
    assert abs(sp["gain"] - g_own) <= 1e-5 * abs(g_own) + 1e-9
    assert np.allclose([sp["GL"], sp["HL"], sp["GR"], sp["HR"]], sides, rtol=1e-5, atol=n * 0.5 / min(scale))
    assert sp["GLq"] == round(sp["GL"] * scale[0]) and sp["HLq"] == round(sp["HL"] * scale[1])


def test_eval_split_exact_ties_follow_candidate_order(ctx, oracle):
    # g = +-0.5, h = 0.25 are exact in fixed point and in fp64: duplicated
    # features tie exactly and the first one must win on both sides.
    import paper_1806_11248_amd as g
    rng = np.random.default_rng(11)
    n, B = 20_000, 32
    col = rng.integers(0, B, n)
    sym = np.stack([rng.integers(0, B, n), col, col, rng.integers(0, B, n), col], 1).astype(np.uint16)
    y = (col > 20) ^ (rng.random(n) < 0.2)
    gp = np.stack([np.where(y, -0.5, 0.5), np.full(n, 0.25)], 1).astype(np.float32)
    nb = np.full(5, B, np.int32)
    packed = dev(oracle.pack(sym, 5).view(np.int32))
    gq, scale = ctx.gpair_fixed(dev(gp))
    h = ctx.build_hist(packed, 5, n, 5, B, B, gq, None)
    Gq, Hq = ctx.sum_gpair(gq)
    sp = ctx.eval_split(h, dev(nb), Gq, Hq, scale, g.make_params(max_depth=1, max_bins=B))
    ref_h, cnt, G, H = oracle.hist(sym, B, B, None, gp)
    ref = oracle.eval_split(ref_h, cnt, nb, G, H, n, 1.0, 1.0)
    assert (sp["feature"], sp["bin"], sp["default_left"]) == (ref["feature"], ref["bin"], ref["default_left"]) == (1, 20, 0)
    assert sp["gain"] == ref["gain"]                   # same inputs, same sequence of fp64 operations
    assert np.array_equal(ctx.hist_export_f64(h, scale).cpu().numpy(), ref_h)


# ------------------------------------------------------------------ partition --
@pytest.mark.parametrize("n,F,B,miss", [(10_000, 8, 16, 0.0), (100_003, 13, 256, 0.0), (30_007, 50, 256, 0.8),
                                        (2049, 300, 64, 0.0), (5, 3, 4, 0.5)])
def test_partition(ctx, oracle, n, F, B, miss):
    sym, nb, missing, gp = _node_case(n + 2, n, F, B, None, miss)
    bits = oracle.bits_for(int(sym.max()))
    packed = dev(oracle.pack(sym, bits).view(np.int32))
    rng = np.random.default_rng(n)
    rows = np.sort(rng.choice(n, max(1, (2 * n) // 3), replace=False)).astype(np.uint32)
    m = len(rows)
    for (f, b, dl, lo, hi) in [(F - 1, int(nb[F - 1]) // 2, 0, 0, m), (1 % F, 0, 1, m // 4, m - m // 5),
                               (0, B + 5, 1, 0, m), (0, 0, 0, 3 % m, 3 % m)]:
        _say(f"partition n={n} F={F} bits={bits} split=({f},{b},{dl}) seg=[{lo},{hi})")
        t = dev(rows.view(np.int32))
        nl = ctx.partition(packed, bits, n, F, t, lo, hi, f, b, dl, missing)
        out, nl_ref = oracle.partition(sym, rows[lo:hi], f, b, dl, missing)
        got = host_u32(t)
        assert nl == nl_ref
        assert np.array_equal(got[lo:hi], out)
        assert np.array_equal(got[:lo], rows[:lo]) and np.array_equal(got[hi:], rows[hi:])


def test_argument_errors_return_codes(ctx, oracle):
    import paper_1806_11248_amd as g
    E = g.binding
    sym, nb, missing, gp = _node_case(1, 1000, 4, 16, None, 0.0)
    packed = dev(oracle.pack(sym, 4).view(np.int32))
    gq, scale = ctx.gpair_fixed(dev(gp))
    with pytest.raises(g.GbtError) as e:
        ctx.build_hist(packed, 17, 1000, 4, 16, missing, gq)
    assert e.value.code == E.EUNSUPPORTED
    with pytest.raises(g.GbtError) as e:
        ctx.build_hist(packed, 0, 1000, 4, 16, missing, gq)
    assert e.value.code == E.EINVAL
    with pytest.raises(g.GbtError) as e:
        ctx.build_hist(packed, 4, 1000, 4, 8192, missing, gq, out=ctx.empty((4, 16, 2), torch.int64))
    assert e.value.code == E.EINVAL
    rows = dev(np.arange(1000, dtype=np.int32))
    with pytest.raises(g.GbtError) as e:
        ctx.partition(packed, 4, 1000, 4, rows, 10, 5, 0, 1, 0, missing)
    assert e.value.code == E.EINVAL
    with pytest.raises(g.GbtError) as e:
        ctx.partition(packed, 4, 1000, 4, rows, 0, 1000, 4, 1, 0, missing)      # feature out of range
    assert e.value.code == E.EINVAL
    # a workspace that is too small is refused, nothing is enqueued
    import ctypes as C
    nl = C.c_int64()
    st = ctx.lib.gbt_partition(ctx.h, packed.data_ptr(), 4, 1000, 4, rows.data_ptr(), 0, 1000, 0, 1, 0, missing,
                               ctx.workspace("small", 4096).data_ptr(), 16, C.byref(nl))
    assert st == E.ENOMEM
    assert "workspace" in ctx.lib.gbt_last_error(ctx.h).decode()
