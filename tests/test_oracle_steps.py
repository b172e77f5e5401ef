"""Pins for the oracle's gradients, histogram, split search and partition
(paper Sec. 2.3, 2.5, Eq. 1-2, Alg. 1)."""
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------- gradients --
def test_logistic_gradients_closed_forms(oracle):
    from scipy.special import expit
    rng = np.random.default_rng(0)
    m = (rng.standard_normal(1000) * 4).astype(np.float32)
    y = (rng.random(1000) < 0.5).astype(np.float32)
    gp = oracle.gradients("logistic", m, y).astype(np.float64)
    p = expit(m.astype(np.float64))
    assert np.allclose(gp[:, 0], p - y, rtol=2e-7, atol=1e-9)
    assert np.allclose(gp[:, 1], p * (1 - p), rtol=2e-7, atol=1e-12)
    assert np.all(gp[:, 1] <= 0.25 + 1e-7)
    # margin 0: g = 0.5 - y, h = 0.25 exactly
    g0 = oracle.gradients("logistic", np.zeros(4, np.float32), np.array([0, 1, 0, 1], np.float32))
    assert np.array_equal(g0, np.array([[.5, .25], [-.5, .25], [.5, .25], [-.5, .25]], np.float32))
    # sigmoid(-x) = 1 - sigmoid(x): g(-m, 1-y) = -g(m, y), h even
    gm = oracle.gradients("logistic", -m, 1 - y).astype(np.float64)
    assert np.allclose(gm[:, 0], -gp[:, 0], atol=1e-7) and np.allclose(gm[:, 1], gp[:, 1], atol=1e-7)
    # Eq. 1-2 are the first and second derivative of log(1+e^m) - y*m
    md = m.astype(np.float64)
    loss = lambda z: np.logaddexp(0, z) - y * z
    eps = 1e-4
    assert np.allclose((loss(md + eps) - loss(md - eps)) / (2 * eps), gp[:, 0], atol=1e-6)
    assert np.allclose((loss(md + eps) - 2 * loss(md) + loss(md - eps)) / eps ** 2, gp[:, 1], atol=1e-5)


def test_squared_error_gradients(oracle):
    m = np.array([0.0, 1.5, -2.0], np.float32)
    y = np.array([1.0, 1.0, 3.0], np.float32)
    assert np.array_equal(oracle.gradients("squared", m, y),
                          np.array([[-1, 1], [.5, 1], [-5, 1]], np.float32))


# ----------------------------------------------------------------- histogram --
def _random_node(seed, n=4000, F=6, B=32, miss=0.15):
    rng = np.random.default_rng(seed)
    nb = rng.integers(1, B + 1, F).astype(np.int32)
    nb[0] = B
    missing = int(nb.max())
    sym = np.stack([rng.integers(0, nb[f], n) for f in range(F)], 1).astype(np.uint16)
    sym[rng.random((n, F)) < miss] = missing
    gp = np.stack([rng.standard_normal(n), rng.random(n) + 0.1], 1).astype(np.float32)
    return sym, nb, missing, gp


@pytest.mark.parametrize("seed", [0, 1])
def test_hist_is_bincount(oracle, seed):
    sym, nb, missing, gp = _random_node(seed)
    n, F = sym.shape
    B = 32
    rng = np.random.default_rng(seed + 10)
    rows = np.sort(rng.choice(n, n // 3, replace=False)).astype(np.uint32)
    for rsel in (None, rows):
        h, cnt, G, H = oracle.hist(sym, B, missing, rsel, gp)
        idx = np.arange(n) if rsel is None else rsel
        for f in range(F):
            s = sym[idx, f]
            keep = s != missing
            for c in range(2):
                ref = np.bincount(s[keep], weights=gp[idx, c][keep].astype(np.float64), minlength=B)
                assert np.allclose(h[f, :, c], ref, rtol=1e-12, atol=1e-12)
            assert np.array_equal(cnt[f], np.bincount(s[keep], minlength=B))
            assert cnt[f].sum() == keep.sum()
            # bins + missing mass = node totals
            gm = gp[idx, 0][~keep].astype(np.float64).sum()
            assert np.isclose(h[f, :, 0].sum() + gm, G, rtol=1e-12, atol=1e-9)
        assert np.isclose(G, gp[idx, 0].astype(np.float64).sum(), rtol=1e-13)
        assert np.isclose(H, gp[idx, 1].astype(np.float64).sum(), rtol=1e-13)


def test_hist_constant_gradient_counts_rows(oracle):
    sym, nb, missing, _ = _random_node(3)
    gp = np.ones((sym.shape[0], 2), np.float32)
    h, cnt, G, H = oracle.hist(sym, 32, missing, None, gp)
    assert np.array_equal(h[:, :, 0], cnt) and np.array_equal(h[:, :, 1], cnt)
    assert G == H == sym.shape[0]


def test_hist_parent_is_sum_of_children(oracle):
    sym, nb, missing, gp = _random_node(4)
    n = sym.shape[0]
    rows = np.arange(n, dtype=np.uint32)
    out, nl = oracle.partition(sym, rows, 0, 11, 1, missing)
    hp, cp, G, H = oracle.hist(sym, 32, missing, rows, gp)
    hl, cl, GL, HL = oracle.hist(sym, 32, missing, out[:nl], gp)
    hr, cr, GR, HR = oracle.hist(sym, 32, missing, out[nl:], gp)
    assert np.allclose(hl + hr, hp, rtol=1e-12, atol=1e-10)
    assert np.array_equal(cl + cr, cp)
    assert np.isclose(GL + GR, G, rtol=1e-12) and np.isclose(HL + HR, H, rtol=1e-12)


# --------------------------------------------------------------------- split --
def _brute_force_best(sym, nb, missing, gp, lam, mcw):
    """Every (feature, bin, direction) priced directly from the rows: no
    histogram, no prefix sums."""
    n, F = sym.shape
    g = gp[:, 0].astype(np.float64)
    h = gp[:, 1].astype(np.float64)
    G, H = g.sum(), h.sum()
    best = (-np.inf, None)
    for f in range(F):
        s = sym[:, f].astype(int)
        has_missing = bool((s == missing).any())
        for b in range(nb[f]):
            for d in ((0, 1) if has_missing else (0,)):
                left = ((s <= b) & (s != missing)) | ((s == missing) & (d == 1))
                if not left.any() or left.all():
                    continue
                GL, HL = g[left].sum(), h[left].sum()
                GR, HR = g[~left].sum(), h[~left].sum()
                if HL < mcw or HR < mcw:
                    continue
                term = lambda g_, h_: g_ * g_ / (h_ + lam) if h_ + lam > 0 else 0.0   # no curvature: no step, no gain
                gain = term(GL, HL) + term(GR, HR) - term(G, H)
                if gain > best[0] + 1e-12 * max(1.0, abs(gain)):
                    best = (gain, (f, b, d))
    return best


@pytest.mark.parametrize("seed", range(12))
def test_split_against_brute_force(oracle, seed):
    rng = np.random.default_rng(100 + seed)
    n, F, B = int(rng.integers(8, 65)), int(rng.integers(1, 5)), 8
    nb = rng.integers(1, B + 1, F).astype(np.int32)
    missing = int(nb.max())
    sym = np.stack([rng.integers(0, nb[f], n) for f in range(F)], 1).astype(np.uint16)
    if seed % 2:
        sym[rng.random((n, F)) < 0.3] = missing
    gp = np.stack([rng.standard_normal(n), rng.random(n) + 0.05], 1).astype(np.float32)
    lam, mcw = float(rng.choice([0.0, 1.0, 3.0])), float(rng.choice([0.0, 1.0, 2.5]))
    h, cnt, G, H = oracle.hist(sym, B, missing, None, gp)
    sp = oracle.eval_split(h, cnt, nb, G, H, n, lam, mcw)
    gain, where = _brute_force_best(sym, nb, missing, gp, lam, mcw)
    if where is None:
        assert not sp["valid"] and sp["feature"] == -1
        return
    assert sp["valid"]
    assert np.isclose(sp["gain"], gain, rtol=1e-10, atol=1e-12)
    assert (sp["feature"], sp["bin"], sp["default_left"]) == where
    assert sp["gain"] >= -1e-12          # lambda >= 0: the best valid candidate never loses
    g2, sides = oracle.candidate_gain(h, *where, G, H, lam, mcw, cnt=cnt, n_rows=len(sym))
    assert np.isclose(g2, gain, rtol=1e-10, atol=1e-12)
    assert np.allclose(sides, [sp["GL"], sp["HL"], sp["GR"], sp["HR"]], rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("seed", range(6))
def test_split_never_leaves_a_side_without_rows(oracle, seed):
    # lambda = 0 and min_child_weight = 0, the node's rows all in the low bins, large gradients: priced from
    # G - GL, a right side without rows is rounding noise squared over zero.  No such candidate may win, and the
    # winner is the brute-force one (which sums each side from its rows).
    rng = np.random.default_rng(seed)
    n, F, B = 4000, 3, 16
    nb = np.array([16, 12, 9], np.int32)
    sym = np.stack([rng.integers(2, 6, n), rng.integers(0, 5, n), rng.integers(3, 4, n)], 1).astype(np.uint16)
    missing = 16
    if seed % 2:
        sym[rng.random((n, F)) < 0.2] = missing
    gp = np.stack([rng.standard_normal(n) * 10.0 ** rng.uniform(-8, 8, n), np.ones(n)], 1).astype(np.float32)
    h, cnt, G, H = oracle.hist(sym, B, missing, None, gp)
    if seed % 2 == 0:   # the trap is really set: nothing is missing, some right side without rows has G - GL != 0
        assert any(G - np.cumsum(h[f, :, 0])[b] != 0.0 for f in range(F) for b in range(int(sym[:, f].max()), nb[f] - 1))
    sp = oracle.eval_split(h, cnt, nb, G, H, n, 0.0, 0.0)
    gain, where = _brute_force_best(sym, nb, missing, gp, 0.0, 0.0)
    assert sp["valid"] and np.isfinite(sp["gain"]) and (sp["feature"], sp["bin"], sp["default_left"]) == where
    assert np.isclose(sp["gain"], gain, rtol=1e-9)
    out, nl = oracle.partition(sym, np.arange(n, dtype=np.uint32), sp["feature"], sp["bin"], sp["default_left"], missing)
    assert 0 < nl < n
    # all rows in one bin of five, nothing missing, no weight asked of a child: still nothing to split on
    one = np.full((50, 1), 2, np.uint16)
    h1, cnt1, G1, H1 = oracle.hist(one, 8, 8, None, gp[:50])
    assert not oracle.eval_split(h1, cnt1, np.array([5], np.int32), G1, H1, 50, 1.0, 0.0)["valid"]


@pytest.mark.parametrize("seed", range(4))
def test_named_candidate_is_priced_by_the_search_rule(oracle, seed):
    # Pricing a candidate by name must follow the rule of the exhaustive search: valid iff BOTH sides hold a row
    # and both have H >= min_child_weight.  Validity and gain are re-derived here from the rows themselves.
    rng = np.random.default_rng(100 + seed)
    n, F, B = 300, 3, 8
    nb = np.array([8, 6, 4], np.int32)
    missing = 8
    sym = np.stack([rng.integers(1, 5, n), rng.integers(0, 3, n), rng.integers(2, 3, n)], 1).astype(np.uint16)
    if seed % 2:
        sym[rng.random((n, F)) < 0.15] = missing
    gp = np.stack([rng.standard_normal(n) * 10.0 ** rng.uniform(-6, 6, n), rng.integers(0, 2, n).astype(np.float64)],
                  1).astype(np.float32)
    h, cnt, G, H = oracle.hist(sym, B, missing, None, gp)
    g64 = gp.astype(np.float64)
    refused_for_rows = 0
    for lam, mcw in ((0.0, 0.0), (1.0, 3.0)):
        for f in range(F):
            for b in range(nb[f]):
                for dl in (0, 1):
                    left = (sym[:, f] <= b) | ((sym[:, f] == missing) & bool(dl))
                    HL, HR = g64[left, 1].sum(), g64[~left, 1].sum()
                    valid = 0 < left.sum() < n and HL >= mcw and HR >= mcw
                    got, _ = oracle.candidate_gain(h, f, b, dl, G, H, lam, mcw, cnt=cnt, n_rows=n)
                    assert np.isfinite(got) == bool(valid), (f, b, dl, lam, mcw, got)
                    if valid:
                        t = lambda g_, h_: g_ * g_ / (h_ + lam) if h_ + lam > 0 else 0.0
                        want = t(g64[left, 0].sum(), HL) + t(g64[~left, 0].sum(), HR) - t(g64[:, 0].sum(), g64[:, 1].sum())
                        assert np.isclose(got, want, rtol=1e-7, atol=1e-9 * abs(t(g64[:, 0].sum(), g64[:, 1].sum())))
                    elif HL >= mcw and HR >= mcw:
                        refused_for_rows += 1
    assert refused_for_rows > 0   # the case the rule exists for does occur here


def test_split_two_cluster_closed_form(oracle):
    for line in open(os.path.join(GOLDEN, "two_cluster_gain.txt")):
        if line.startswith("#") or not line.strip():
            continue
        n1, a, n2, c, lam, num, den = (int(t) for t in line.split())
        # the fixture's fraction is itself the closed form, recomputed exactly
        exact = (Fraction(n1 * a) ** 2 / (n1 + lam) + Fraction(n2 * c) ** 2 / (n2 + lam)
                 - Fraction(n1 * a - n2 * c) ** 2 / (n1 + n2 + lam))
        assert exact == Fraction(num, den)
        sym = np.array([[0]] * n1 + [[1]] * n2, np.uint16)
        gp = np.array([[a, 1]] * n1 + [[-c, 1]] * n2, np.float32)
        h, cnt, G, H = oracle.hist(sym, 4, 2, None, gp)
        sp = oracle.eval_split(h, cnt, np.array([2], np.int32), G, H, n1 + n2, float(lam), 1.0)
        assert (sp["feature"], sp["bin"], sp["default_left"]) == (0, 0, 0)
        assert np.isclose(sp["gain"], num / den, rtol=1e-14)
        assert (sp["GL"], sp["HL"], sp["GR"], sp["HR"]) == (n1 * a, n1, -n2 * c, n2)


def test_split_reduces_to_regression_stump(oracle):
    # h = 1, lambda = 0: gain = reduction of the sum of squared errors, so the
    # root split must separate the rows like a depth-1 least-squares tree on -g.
    from sklearn.tree import DecisionTreeRegressor
    rng = np.random.default_rng(7)
    n, F, B = 600, 3, 16
    X = rng.standard_normal((n, F)).astype(np.float32)
    y = (np.where(X[:, 1] > 0.3, 2.0, -1.0) + 0.3 * rng.standard_normal(n))
    cuts, nb = oracle.cuts(X, B)
    sym, missing, _ = oracle.bin_matrix(X, cuts, nb)
    gp = np.stack([-y, np.ones(n)], 1).astype(np.float32)
    h, cnt, G, H = oracle.hist(sym, B, missing, None, gp)
    sp = oracle.eval_split(h, cnt, nb, G, H, n, 0.0, 1.0)
    # scikit-learn sees the same candidate set when it is given the symbols
    stump = DecisionTreeRegressor(max_depth=1).fit(sym.astype(np.float64), -gp[:, 0].astype(np.float64))
    assert stump.tree_.feature[0] == sp["feature"] == 1
    left_sk = sym[:, sp["feature"]] <= stump.tree_.threshold[0]
    left_or = sym[:, sp["feature"]] <= sp["bin"]
    assert np.array_equal(left_sk, left_or)
    yy = -gp[:, 0].astype(np.float64)
    sse = lambda v: ((v - v.mean()) ** 2).sum()
    assert np.isclose(sp["gain"], sse(yy) - sse(yy[left_or]) - sse(yy[~left_or]), rtol=1e-9)
    # leaf weights = -mean(g) per side
    assert np.isclose(-sp["GL"] / sp["HL"], yy[left_or].mean(), rtol=1e-12)
    assert np.isclose(-sp["GR"] / sp["HR"], yy[~left_or].mean(), rtol=1e-12)


def test_default_direction_is_learned(oracle):
    # one feature, two bins; the missing rows look like bin 0 in one data set and
    # like bin 1 in its mirror image: the default direction must flip.
    base_sym = np.array([0] * 10 + [1] * 10 + [2] * 10, np.uint16).reshape(-1, 1)   # 2 = missing
    nb = np.array([2], np.int32)
    for like_left in (True, False):
        g = np.array([1.0] * 10 + [-1.0] * 10 + ([1.0] if like_left else [-1.0]) * 10)
        gp = np.stack([g, np.ones(30)], 1).astype(np.float32)
        h, cnt, G, H = oracle.hist(base_sym, 2, 2, None, gp)
        sp = oracle.eval_split(h, cnt, nb, G, H, 30, 1.0, 1.0)
        assert (sp["feature"], sp["bin"]) == (0, 0)
        assert sp["default_left"] == int(like_left)
    # "present left, missing right" is a candidate of its own (bin = last bin)
    g = np.array([1.0] * 10 + [1.0] * 10 + [-1.0] * 10)
    gp = np.stack([g, np.ones(30)], 1).astype(np.float32)
    h, cnt, G, H = oracle.hist(base_sym, 2, 2, None, gp)
    sp = oracle.eval_split(h, cnt, nb, G, H, 30, 1.0, 1.0)
    assert (sp["feature"], sp["bin"], sp["default_left"]) == (0, 1, 0)


def test_split_tie_break_and_min_child_weight(oracle):
    # two identical features: the first one wins; strict '>' keeps the first bin
    sym = np.array([[0, 0], [0, 0], [1, 1], [1, 1]], np.uint16)
    gp = np.array([[1, 1], [1, 1], [-1, 1], [-1, 1]], np.float32)
    nb = np.array([2, 2], np.int32)
    h, cnt, G, H = oracle.hist(sym, 2, 2, None, gp)
    sp = oracle.eval_split(h, cnt, nb, G, H, 4, 1.0, 1.0)
    assert (sp["feature"], sp["bin"], sp["default_left"]) == (0, 0, 0)
    # min_child_weight larger than either side's hessian mass: no valid candidate
    sp = oracle.eval_split(h, cnt, nb, G, H, 4, 1.0, 2.5)
    assert not sp["valid"]
    # and pricing that candidate by name says the same: a gain at weight 2 (each side holds exactly 2), none at 2.5
    assert np.isclose(oracle.candidate_gain(h, 0, 0, 0, G, H, 1.0, 2.0, cnt=cnt, n_rows=4)[0], 4 / 3 + 4 / 3)
    assert np.isnan(oracle.candidate_gain(h, 0, 0, 0, G, H, 1.0, 2.5, cnt=cnt, n_rows=4)[0])
    # a side without curvature under lambda = 0 counts nothing (not +inf): 2^2/2 + 0 - 8^2/2
    symz = np.array([[0], [0], [1], [1]], np.uint16)
    gpz = np.array([[1, 1], [1, 1], [-5, 0], [-5, 0]], np.float32)
    hz, cntz, Gz, Hz = oracle.hist(symz, 2, 2, None, gpz)
    spz = oracle.eval_split(hz, cntz, np.array([2], np.int32), Gz, Hz, 4, 0.0, 0.0)
    assert spz["valid"] and (spz["feature"], spz["bin"]) == (0, 0) and spz["gain"] == 2.0 + 0.0 - 32.0
    assert oracle.candidate_gain(hz, 0, 0, 0, Gz, Hz, 0.0, 0.0, cnt=cntz, n_rows=4)[0] == -30.0
    # a single-bin feature with nothing missing can never split
    sym1 = np.zeros((5, 1), np.uint16)
    gp1 = np.stack([np.arange(5) - 2.0, np.ones(5)], 1).astype(np.float32)
    h, cnt, G, H = oracle.hist(sym1, 2, 1, None, gp1)
    assert not oracle.eval_split(h, cnt, np.array([1], np.int32), G, H, 5, 1.0, 0.0)["valid"]


# ----------------------------------------------------------------- partition --
@pytest.mark.parametrize("dl", [0, 1])
def test_partition_is_stable_filter(oracle, dl):
    sym, nb, missing, _ = _random_node(8, n=3000)
    rng = np.random.default_rng(8)
    rows = np.sort(rng.choice(3000, 1700, replace=False)).astype(np.uint32)
    f, b = 2, int(nb[2] // 2)
    out, nl = oracle.partition(sym, rows, f, b, dl, missing)
    s = sym[rows, f].astype(int)
    m = np.where(s == missing, bool(dl), s <= b)
    assert np.array_equal(out, np.concatenate([rows[m], rows[~m]]))
    assert nl == int(m.sum())
    assert np.array_equal(np.sort(out), rows)
    assert np.all(np.diff(out[:nl].astype(np.int64)) > 0) and np.all(np.diff(out[nl:].astype(np.int64)) > 0)
    # degenerate: everything to one side, empty list
    out, nl = oracle.partition(sym, rows, 0, 10_000, 1, missing)
    assert nl == len(rows) and np.array_equal(out, rows)
    out, nl = oracle.partition(sym, rows[:0], 0, 3, 0, missing)
    assert nl == 0 and len(out) == 0
