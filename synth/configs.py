"""Seeded synthetic inputs for the five workloads.

This module only draws random inputs (feature matrices, labels, and for the
smallest workload the gradient pairs themselves).  It holds none of the
method's arithmetic: no quantisation, histograms, gains or gradients.  Both the
CPU oracle's tests and the GPU tests/benchmark read their inputs from here so
that the two sides see identical bytes.

Every workload is generated in row chunks of CHUNK rows, each chunk from its own
PCG64 stream keyed by (base seed + config number, tag, chunk index).  A run with
a smaller ``n`` is therefore an exact prefix of the full-size data set, and the
chunks can be drawn by several threads without changing the result.

The data sets the paper measures on (its Table 1) are public files that are not
available here; these generators stand in for them by shape only:
C2 ~ a 28-column classification set, C3 ~ the 10M-row synthetic regression made
sparse, C4 ~ the 115M x 13 classification set, C5 ~ a wide matrix.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

BASE_SEED = 180611248
CHUNK = 1 << 16

_TAG_PARAMS = 0
_TAG_ROWS = 1


def _rng(cfg: int, tag: int, idx: int = 0) -> np.random.Generator:
    ss = np.random.SeedSequence([BASE_SEED + cfg, tag, idx])
    return np.random.Generator(np.random.PCG64(ss))


def _threads() -> int:
    try:
        return max(1, min(16, len(os.sched_getaffinity(0))))
    except AttributeError:  # pragma: no cover
        return max(1, min(16, os.cpu_count() or 1))


def _run_chunks(n: int, fn):
    """Call fn(chunk_index, lo, hi) for every row chunk, on a thread pool."""
    spans = [(c, lo, min(n, lo + CHUNK)) for c, lo in enumerate(range(0, n, CHUNK))]
    if len(spans) <= 1:
        for s in spans:
            fn(*s)
        return
    with ThreadPoolExecutor(max_workers=_threads()) as ex:
        list(ex.map(lambda s: fn(*s), spans))


def _sigmoid(z):
    return 1.0 / (1.0 + np.exp(-z))


# --------------------------------------------------------------------------- C1
def config1(n: int = 10_000):
    """Tiny dense regression: n x 8 U[0,1) features, 16 bins; the gradient pairs
    are given directly (g ~ N(0,1), h ~ U[0.1,1]); one tree of depth 3."""
    F = 8
    X = np.empty((n, F), np.float32)
    g = np.empty(n, np.float32)
    h = np.empty(n, np.float32)

    def fill(c, lo, hi):
        r = _rng(1, _TAG_ROWS, c)
        m = CHUNK
        X[lo:hi] = r.random((m, F), dtype=np.float32)[: hi - lo]
        g[lo:hi] = r.standard_normal(m, dtype=np.float32)[: hi - lo]
        h[lo:hi] = (0.1 + 0.9 * r.random(m, dtype=np.float32))[: hi - lo]

    _run_chunks(n, fill)
    params = dict(max_bins=16, max_depth=3, rounds=1, eta=1.0, lam=1.0, gamma=0.0,
                  min_child_weight=1.0, objective="given")
    return dict(name="C1", X=X, y=None, g=g, h=h, params=params)


# --------------------------------------------------------------------------- C2
def config2(n: int = 1_000_000):
    """Dense binary classification: n x 28 N(0,1) features; labels Bernoulli of
    the sigmoid of five random pairwise products plus a linear term."""
    F = 28
    p = _rng(2, _TAG_PARAMS)
    a = p.standard_normal(5)
    pairs = []
    while len(pairs) < 5:
        i, j = (int(v) for v in p.integers(0, F, 2))
        if i != j and (i, j) not in pairs and (j, i) not in pairs:
            pairs.append((i, j))
    w = 0.5 * p.standard_normal(F)
    X = np.empty((n, F), np.float32)
    y = np.empty(n, np.float32)

    def fill(c, lo, hi):
        r = _rng(2, _TAG_ROWS, c)
        x = r.standard_normal((CHUNK, F), dtype=np.float32)[: hi - lo]
        u = r.random(CHUNK)[: hi - lo]
        xd = x.astype(np.float64)
        z = xd @ w
        for k, (i, j) in enumerate(pairs):
            z += a[k] * xd[:, i] * xd[:, j]
        X[lo:hi] = x
        y[lo:hi] = (u < _sigmoid(z)).astype(np.float32)

    _run_chunks(n, fill)
    params = dict(max_bins=256, max_depth=6, rounds=10, eta=0.1, lam=1.0, gamma=0.0,
                  min_child_weight=1.0, objective="logistic")
    return dict(name="C2", X=X, y=y, g=None, h=None, params=params)


# --------------------------------------------------------------------------- C3
def config3(n: int = 10_000_000, F: int = 50):
    """Sparse regression: each entry present with probability 0.2, present
    values lognormal(0,1); labels from a random depth-4 tree over the features
    (random default side for absent entries) plus N(0, 0.1) noise.  Returned
    both as CSR (int64 indptr, int32 indices, float32 values) and as a dense
    matrix with NaN for the absent entries."""
    p = _rng(3, _TAG_PARAMS)
    n_int = 15
    t_feat = p.integers(0, F, n_int)
    # threshold = a quantile of lognormal(0,1) at a random level in (0.1, 0.9)
    t_q = 0.1 + 0.8 * p.random(n_int)
    from math import erf, sqrt  # noqa: F401  (inverse normal CDF via bisection below)

    def norm_ppf(q):
        lo, hi = -8.0, 8.0
        for _ in range(80):
            mid = 0.5 * (lo + hi)
            if 0.5 * (1.0 + erf(mid / sqrt(2.0))) < q:
                lo = mid
            else:
                hi = mid
        return 0.5 * (lo + hi)

    t_thr = np.array([np.exp(norm_ppf(float(q))) for q in t_q])
    t_def_left = p.random(n_int) < 0.5
    leaves = p.standard_normal(16)

    X = np.empty((n, F), np.float32)
    y = np.empty(n, np.float32)

    def fill(c, lo, hi):
        r = _rng(3, _TAG_ROWS, c)
        m = hi - lo
        mask = (r.random((CHUNK, F), dtype=np.float32) < np.float32(0.2))[:m]
        vals = r.lognormal(0.0, 1.0, (CHUNK, F)).astype(np.float32)[:m]
        noise = 0.1 * r.standard_normal(CHUNK)[:m]
        x = np.where(mask, vals, np.float32(np.nan))
        node = np.zeros(m, np.int64)
        for _ in range(4):
            f = t_feat[node]
            v = x[np.arange(m), f]
            miss = np.isnan(v)
            go_left = np.where(miss, t_def_left[node], v < t_thr[node])
            node = 2 * node + np.where(go_left, 1, 2)
        X[lo:hi] = x
        y[lo:hi] = (leaves[node - n_int] + noise).astype(np.float32)

    _run_chunks(n, fill)
    params = dict(max_bins=256, max_depth=8, rounds=5, eta=0.1, lam=1.0, gamma=0.0,
                  min_child_weight=1.0, objective="squared")
    return dict(name="C3", X=X, y=y, g=None, h=None, params=params)


def dense_to_csr(X: np.ndarray):
    """CSR view (int64 indptr, int32 indices, float32 values) of a dense matrix
    whose absent entries are NaN."""
    present = ~np.isnan(X)
    counts = present.sum(axis=1, dtype=np.int64)
    indptr = np.zeros(X.shape[0] + 1, np.int64)
    np.cumsum(counts, out=indptr[1:])
    rows, cols = np.nonzero(present)
    del rows
    return indptr, cols.astype(np.int32), X[present].astype(np.float32)


# --------------------------------------------------------------------------- C4
def config4(n: int = 115_000_000):
    """Large tabular: 8 integer-valued columns with cardinality K_j in [7, 300]
    and P(k) ~ k^-1.2, stored as float32, plus 5 lognormal(0, 2) columns;
    binary labels from a logistic model of per-category effects and log
    features."""
    F_cat, F_num = 8, 5
    F = F_cat + F_num
    p = _rng(4, _TAG_PARAMS)
    K = p.integers(7, 301, F_cat)
    cdfs, effects = [], []
    for j in range(F_cat):
        k = np.arange(1, K[j] + 1, dtype=np.float64)
        pk = k ** -1.2
        cdfs.append(np.cumsum(pk / pk.sum()))
        effects.append(0.3 * p.standard_normal(K[j]))
    w = 0.5 * p.standard_normal(F_num)
    X = np.empty((n, F), np.float32)
    y = np.empty(n, np.float32)

    def fill(c, lo, hi):
        r = _rng(4, _TAG_ROWS, c)
        m = hi - lo
        z = np.zeros(m)
        blk = np.empty((m, F), np.float32)
        for j in range(F_cat):
            u = r.random(CHUNK)[:m]
            k = np.minimum(np.searchsorted(cdfs[j], u, side="right"), K[j] - 1)
            blk[:, j] = (k + 1).astype(np.float32)
            z += effects[j][k]
        for j in range(F_num):
            v = r.lognormal(0.0, 2.0, CHUNK)[:m].astype(np.float32)
            blk[:, F_cat + j] = v
            z += w[j] * np.log(np.maximum(v.astype(np.float64), 1e-300)) / 2.0
        u = r.random(CHUNK)[:m]
        X[lo:hi] = blk
        y[lo:hi] = (u < _sigmoid(z)).astype(np.float32)

    _run_chunks(n, fill)
    params = dict(max_bins=256, max_depth=8, rounds=1, eta=1.0, lam=1.0, gamma=0.0,
                  min_child_weight=1.0, objective="logistic")
    return dict(name="C4", X=X, y=y, g=None, h=None, params=params)


# --------------------------------------------------------------------------- C5
def config5(n: int = 500_000, F: int = 2000):
    """Wide/deep: 80% of the columns N(0,1), 20% copies of random source columns
    plus N(0, 0.05) noise (interleaved by a fixed permutation); labels from a
    20-sparse linear model plus N(0, 0.1) noise."""
    F_src = (F * 4) // 5
    F_dup = F - F_src
    p = _rng(5, _TAG_PARAMS)
    src = p.integers(0, F_src, F_dup)
    perm = p.permutation(F)
    n_coef = min(20, F)
    coef_idx = p.choice(F, n_coef, replace=False)
    coef = p.standard_normal(n_coef)
    X = np.empty((n, F), np.float32)
    y = np.empty(n, np.float32)

    def fill(c, lo, hi):
        r = _rng(5, _TAG_ROWS, c)
        m = hi - lo
        base = r.standard_normal((CHUNK, F_src), dtype=np.float32)[:m]
        dup = base[:, src] + np.float32(0.05) * r.standard_normal((CHUNK, F_dup), dtype=np.float32)[:m]
        blk = np.concatenate([base, dup], axis=1)[:, perm]
        noise = 0.1 * r.standard_normal(CHUNK)[:m]
        X[lo:hi] = blk
        y[lo:hi] = (blk[:, coef_idx].astype(np.float64) @ coef + noise).astype(np.float32)

    _run_chunks(n, fill)
    params = dict(max_bins=64, max_depth=10, rounds=1, eta=1.0, lam=1.0, gamma=0.0,
                  min_child_weight=1.0, objective="squared")
    return dict(name="C5", X=X, y=y, g=None, h=None, params=params)


CONFIGS = {1: config1, 2: config2, 3: config3, 4: config4, 5: config5}


def make(cfg: int, n: int | None = None, **kw):
    """Generate workload ``cfg`` (1..5), optionally with fewer rows."""
    fn = CONFIGS[cfg]
    return fn(**kw) if n is None else fn(n, **kw)
