"""CPU oracle for quantised-histogram tree construction (arXiv 1806.11248).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke``
and by the ``cpu_baseline`` leg of ``bench.py``.  The GPU library never imports
or links anything from this directory, and this directory never imports the GPU
package.

The arithmetic lives in ``gbt_oracle.c`` (plain C, fp64, compiled by
``oracle.build()``); this file marshals numpy arrays into it and holds the two
drivers that are easier to read in Python than in C:

* ``grow_tree``  -- Alg. 1 with the "closest to the root first" growth policy
  (Sec. 2.3): open nodes level by level, left to right; for every node build its
  histogram from its own rows (no sibling subtraction), search every split,
  partition its rows.
* ``replay_tree`` -- judges a tree grown elsewhere: on the oracle's own row
  lists it re-derives, node by node, the exhaustive best split and the fp64
  gain of the split the other side chose.

``leaf_weight`` holds the reading taken for a node without curvature.  Nothing
here knows how the GPU library represents its sums.

Pins (tests/test_oracle_*.py): closed forms, numpy/scipy/scikit-learn library
routines, brute-force enumeration on tiny inputs, conservation invariants.
tests/test_pins_kill_mutants.py plants single mistakes into copies of this
directory and demands that a pin fails for each.
Whole-workload trees have no printed example in the paper, so they are pinned
only through those per-step pins plus the invariants at full size.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gbt_oracle.c")
_LIB = os.path.join(_HERE, "libgbt_oracle.so")
_LIB_SAN = os.path.join(_HERE, "libgbt_oracle_san.so")
_lib = None

GAIN_FLOOR = 1e-6   # a split needs gain > max(gamma, GAIN_FLOOR)


def build(force: bool = False, sanitize: bool = False) -> str:
    """Compile gbt_oracle.c with gcc (no fast-math, no FMA contraction).

    sanitize: a second library, libgbt_oracle_san.so, built with -fsanitize=address,undefined (any undefined
    behaviour aborts).  `lib()` loads it instead of the plain one when GBT_ORACLE_SANITIZE=1 is in the environment;
    the process then also needs ASAN_OPTIONS=verify_asan_link_order=0:detect_leaks=0, since the interpreter itself
    is not instrumented (memory the oracle allocates is checked exactly, the caller's numpy buffers are not).  The
    whole CPU suite under it: GBT_ORACLE_SANITIZE=1 ASAN_OPTIONS=verify_asan_link_order=0:detect_leaks=0
    python -m pytest tests -m "not gpu"."""
    out = _LIB_SAN if sanitize else _LIB
    if force or not os.path.exists(out) or os.path.getmtime(out) < os.path.getmtime(_SRC):
        flags = (["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                  "-fno-omit-frame-pointer"] if sanitize else ["-O2"])
        subprocess.check_call(
            ["gcc", *flags, "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-o", out, _SRC, "-lm"])
    return out


class Split(C.Structure):
    _fields_ = [("feature", C.c_int32), ("bin", C.c_int32), ("default_left", C.c_int32),
                ("valid", C.c_int32), ("gain", C.c_double), ("GL", C.c_double), ("HL", C.c_double),
                ("GR", C.c_double), ("HR", C.c_double)]


def _p(a, t):
    return a.ctypes.data_as(C.POINTER(t))


def lib():
    global _lib
    if _lib is None:
        sanitize = os.environ.get("GBT_ORACLE_SANITIZE", "0") not in ("", "0")
        L = C.CDLL(build(sanitize=sanitize))
        L.gbto_cuts.restype = C.c_int32
        L.gbto_bits.restype = C.c_int32
        L.gbto_packed_words.restype = C.c_int64
        L.gbto_partition.restype = C.c_int64
        L.gbto_candidate_gain.restype = C.c_double
        L.gbto_candidate_gain.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int64, C.c_int32, C.c_int32,
                                          C.c_int32, C.c_double, C.c_double, C.c_double, C.c_double, C.c_void_p]
        L.gbto_eval_split.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                      C.c_double, C.c_double, C.c_int64, C.c_double, C.c_double,
                                      C.POINTER(Split)]
        _lib = L
    return _lib


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


# ------------------------------------------------------------------ quantise --
def cuts(X: np.ndarray, B: int):
    """Per-feature quantile cuts of a dense matrix (NaN = missing).
    Returns (cuts float32 [F][B-1] padded with +inf, nb int32 [F])."""
    X = _c(X, np.float32)
    n, F = X.shape
    out = np.empty((F, max(B - 1, 0)), np.float32)
    nb = np.empty(F, np.int32)
    lib().gbto_cuts_matrix(C.c_void_p(X.ctypes.data), C.c_int64(n), C.c_int32(F), C.c_int32(B),
                           C.c_void_p(out.ctypes.data), C.c_void_p(nb.ctypes.data))
    return out, nb


def bin_matrix(X: np.ndarray, cuts_: np.ndarray, nb: np.ndarray):
    """Symbols of X.  Returns (sym uint16 [n][F], missing_sym, max_value)."""
    X = _c(X, np.float32)
    n, F = X.shape
    B = cuts_.shape[1] + 1
    missing_sym = int(nb.max()) if F else 0
    sym = np.empty((n, F), np.uint16)
    lib().gbto_bin(C.c_void_p(X.ctypes.data), C.c_int64(n), C.c_int32(F),
                   C.c_void_p(_c(cuts_, np.float32).ctypes.data),
                   C.c_void_p(_c(nb, np.int32).ctypes.data), C.c_int32(B), C.c_int32(missing_sym),
                   C.c_void_p(sym.ctypes.data))
    max_value = int(sym.max()) if sym.size else 0
    return sym, missing_sym, max_value


def bits_for(max_value: int) -> int:
    return int(lib().gbto_bits(C.c_uint32(max_value)))


def packed_words(n_elems: int, bits: int) -> int:
    return int(lib().gbto_packed_words(C.c_int64(n_elems), C.c_int32(bits)))


def pack(sym: np.ndarray, bits: int) -> np.ndarray:
    s = _c(sym, np.uint16).reshape(-1)
    out = np.empty(packed_words(s.size, bits), np.uint32)
    lib().gbto_pack(C.c_void_p(s.ctypes.data), C.c_int64(s.size), C.c_int32(bits),
                    C.c_void_p(out.ctypes.data))
    return out


def unpack(words: np.ndarray, n_elems: int, bits: int) -> np.ndarray:
    w = _c(words, np.uint32)
    out = np.empty(n_elems, np.uint16)
    lib().gbto_unpack(C.c_void_p(w.ctypes.data), C.c_int64(n_elems), C.c_int32(bits),
                      C.c_void_p(out.ctypes.data))
    return out


# ----------------------------------------------------------------- gradients --
OBJECTIVES = {"squared": 0, "logistic": 1}


def gradients(objective: str, margin: np.ndarray, label: np.ndarray) -> np.ndarray:
    m = _c(margin, np.float32)
    y = _c(label, np.float32)
    out = np.empty((m.size, 2), np.float32)
    lib().gbto_gradients(C.c_int32(OBJECTIVES[objective]), C.c_void_p(m.ctypes.data),
                         C.c_void_p(y.ctypes.data), C.c_int64(m.size), C.c_void_p(out.ctypes.data))
    return out


# ----------------------------------------------------------------- histogram --
def hist(sym: np.ndarray, B: int, missing_sym: int, rows, gpair: np.ndarray):
    """Histogram of one node.  rows: uint32 row ids, or None for all rows.
    Returns (hist float64 [F][B][2], cnt int64 [F][B], G, H)."""
    n, F = sym.shape
    h = np.empty((F, B, 2), np.float64)
    cnt = np.empty((F, B), np.int64)
    GH = np.empty(2, np.float64)
    if rows is None:
        rp, nr = None, n
    else:
        rows = _c(rows, np.uint32)
        rp, nr = C.c_void_p(rows.ctypes.data), rows.size
    gp = _c(gpair, np.float32)
    lib().gbto_hist(C.c_void_p(sym.ctypes.data), C.c_int32(F), C.c_int32(B), C.c_int32(missing_sym),
                    rp, C.c_int64(nr), C.c_void_p(gp.ctypes.data), C.c_void_p(h.ctypes.data),
                    C.c_void_p(cnt.ctypes.data), C.c_void_p(GH.ctypes.data))
    return h, cnt, float(GH[0]), float(GH[1])


# --------------------------------------------------------------------- split --
def eval_split(hist_: np.ndarray, cnt: np.ndarray, nb: np.ndarray, G: float, H: float, n_rows: int,
               lam: float, min_child_weight: float) -> dict:
    F, B, _ = hist_.shape
    sp = Split()
    lib().gbto_eval_split(C.c_void_p(hist_.ctypes.data), C.c_void_p(cnt.ctypes.data),
                          C.c_void_p(_c(nb, np.int32).ctypes.data), F, B, G, H, n_rows, lam,
                          min_child_weight, C.byref(sp))
    return {k: getattr(sp, k) for k, _ in Split._fields_}


def candidate_gain(hist_: np.ndarray, f: int, b: int, default_left: int, G: float, H: float,
                   lam: float, min_child_weight: float, *, cnt: np.ndarray, n_rows: int):
    """fp64 gain of one named candidate, NaN if invalid (a side without rows, or lighter than
    min_child_weight: the rule of ``eval_split``); also (GL, HL, GR, HR).
    cnt, n_rows: the node's bin counts (from ``hist``) and its row count."""
    sides = np.empty(4, np.float64)
    cnt = _c(cnt, np.int64)
    g = lib().gbto_candidate_gain(C.c_void_p(hist_.ctypes.data), C.c_void_p(cnt.ctypes.data), hist_.shape[1],
                                  int(n_rows), f, b, default_left, G, H, lam, min_child_weight,
                                  C.c_void_p(sides.ctypes.data))
    return float(g), sides


# ----------------------------------------------------------------- partition --
def partition(sym: np.ndarray, rows: np.ndarray, f: int, b: int, default_left: int,
              missing_sym: int):
    rows = _c(rows, np.uint32)
    out = np.empty_like(rows)
    nl = lib().gbto_partition(C.c_void_p(sym.ctypes.data), C.c_int32(sym.shape[1]),
                              C.c_void_p(rows.ctypes.data), C.c_int64(rows.size), C.c_int32(f),
                              C.c_int32(b), C.c_int32(default_left), C.c_int32(missing_sym),
                              C.c_void_p(out.ctypes.data))
    return out, int(nl)


# ---------------------------------------------------------------------- tree --
def new_tree(max_depth: int) -> dict:
    cap = 2 ** (max_depth + 1) - 1
    return dict(
        n_nodes=0, capacity=cap,
        feature=np.full(cap, -1, np.int32), bin=np.zeros(cap, np.int32),
        threshold=np.full(cap, np.inf, np.float32), default_left=np.zeros(cap, np.int32),
        left=np.full(cap, -1, np.int32), right=np.full(cap, -1, np.int32),
        weight=np.zeros(cap, np.float64), gain=np.zeros(cap, np.float64),
        sumG=np.zeros(cap, np.float64), sumH=np.zeros(cap, np.float64),
        n_rows=np.zeros(cap, np.int64), depth=np.zeros(cap, np.int32))


def new_tree_leaves(max_leaves: int) -> dict:
    """A tree with room for max_leaves leaves (2*max_leaves - 1 nodes)."""
    t = new_tree(0)
    cap = 2 * max_leaves - 1
    for k, v in list(t.items()):
        if isinstance(v, np.ndarray):
            t[k] = np.resize(v, cap)
            t[k][:] = v[0]
    t["capacity"] = cap
    return t


def leaf_weight(G, H, lam):
    """w = -G / (H + lambda), the minimiser of G*w + (H + lambda)*w^2/2.  Without curvature (H + lambda = 0, only
    possible with lambda = 0 and no hessian mass) there is no minimiser; the reading taken is "no step": 0."""
    return -G / (H + lam) if H + lam > 0.0 else 0.0


def _threshold(cuts_, nb, f, b):
    # rows with symbol <= b are those with x < cuts[f][b]; the feature's last
    # bin has no cut to its right (only missing rows can be on the other side)
    return np.float32(cuts_[f, b]) if b < nb[f] - 1 else np.float32(np.inf)


def grow_tree(sym, nb, cuts_, missing_sym, gpair, *, max_depth, max_bins, lam=1.0, gamma=0.0,
              min_child_weight=1.0):
    """Alg. 1, depth-wise.  Returns (tree, row_idx, leaf_of_row): row_idx is the
    final row order (every node's rows are one contiguous, ascending run; a
    node's left child's run comes first), leaf_of_row the node id of each row's leaf."""
    n, F = sym.shape
    B = max_bins
    t = new_tree(max_depth)
    rows = np.arange(n, dtype=np.uint32)
    leaf_of_row = np.zeros(n, np.int32)
    queue = [(0, 0, n, 0)]           # node id, begin, end, depth  -- FIFO = level by level
    t["n_nodes"] = 1
    head = 0
    while head < len(queue):
        node, lo, hi, depth = queue[head]
        head += 1
        r = rows[lo:hi]
        h_, cnt, G, H = hist(sym, B, missing_sym, r, gpair)
        t["sumG"][node], t["sumH"][node], t["n_rows"][node] = G, H, hi - lo
        t["weight"][node] = leaf_weight(G, H, lam)
        t["depth"][node] = depth
        do_split = False
        if depth < max_depth:
            sp = eval_split(h_, cnt, nb, G, H, hi - lo, lam, min_child_weight)
            do_split = bool(sp["valid"]) and sp["gain"] > gamma and sp["gain"] > GAIN_FLOOR
        if not do_split:
            leaf_of_row[r] = node
            continue
        f, b, dl = sp["feature"], sp["bin"], sp["default_left"]
        out, nl = partition(sym, r, f, b, dl, missing_sym)
        rows[lo:hi] = out
        li, ri = t["n_nodes"], t["n_nodes"] + 1
        t["n_nodes"] += 2
        t["feature"][node], t["bin"][node], t["default_left"][node] = f, b, dl
        t["threshold"][node] = _threshold(cuts_, nb, f, b)
        t["left"][node], t["right"][node], t["gain"][node] = li, ri, sp["gain"]
        queue.append((li, lo, lo + nl, depth + 1))
        queue.append((ri, lo + nl, hi, depth + 1))
    return t, rows, leaf_of_row


def grow_tree_lossguide(sym, nb, cuts_, missing_sym, gpair, *, max_leaves, max_depth, max_bins, lam=1.0,
                        gamma=0.0, min_child_weight=1.0):
    """Alg. 1 with the loss-guided policy of Sec. 2.3: instead of the node closest to the
    root, the open leaf whose best split has the LARGEST gain is expanded next (the smaller
    node id on equal gains), until the tree has max_leaves leaves or no leaf is open.  A
    leaf is open iff it has a valid candidate with gain > max(gamma, GAIN_FLOOR) and its
    depth is below max_depth.  Children get the next two ids at the moment of the
    expansion.  Returns (tree, row_idx, leaf_of_row) like grow_tree."""
    n, F = sym.shape
    B = max_bins
    t = new_tree_leaves(max_leaves)
    rows = np.arange(n, dtype=np.uint32)
    leaf_of_row = np.zeros(n, np.int32)
    seg = {}      # node -> (lo, hi)
    open_ = {}    # node -> its best split

    def settle(node, lo, hi, depth):
        r = rows[lo:hi]
        h_, cnt, G, H = hist(sym, B, missing_sym, r, gpair)
        t["sumG"][node], t["sumH"][node], t["n_rows"][node] = G, H, hi - lo
        t["weight"][node] = leaf_weight(G, H, lam)
        t["depth"][node] = depth
        seg[node] = (lo, hi)
        if depth < max_depth:
            sp = eval_split(h_, cnt, nb, G, H, hi - lo, lam, min_child_weight)
            if bool(sp["valid"]) and sp["gain"] > gamma and sp["gain"] > GAIN_FLOOR:
                open_[node] = sp

    t["n_nodes"] = 1
    settle(0, 0, n, 0)
    n_leaves = 1
    while n_leaves < max_leaves and open_:
        node = min(open_, key=lambda k: (-open_[k]["gain"], k))
        sp = open_.pop(node)
        lo, hi = seg[node]
        f, b, dl = sp["feature"], sp["bin"], sp["default_left"]
        out, nl = partition(sym, rows[lo:hi], f, b, dl, missing_sym)
        rows[lo:hi] = out
        li, ri = t["n_nodes"], t["n_nodes"] + 1
        t["n_nodes"] += 2
        t["feature"][node], t["bin"][node], t["default_left"][node] = f, b, dl
        t["threshold"][node] = _threshold(cuts_, nb, f, b)
        t["left"][node], t["right"][node], t["gain"][node] = li, ri, sp["gain"]
        d = int(t["depth"][node]) + 1
        settle(li, lo, lo + nl, d)
        settle(ri, lo + nl, hi, d)
        n_leaves += 1
    for node in range(t["n_nodes"]):
        if t["feature"][node] < 0:
            lo, hi = seg[node]
            leaf_of_row[rows[lo:hi]] = node
    return t, rows, leaf_of_row


def predict_sym(tree, sym, missing_sym, eta, margin, want_leaf=False):
    n, F = sym.shape
    margin = _c(margin, np.float32).copy()
    leaf = np.empty(n, np.int32) if want_leaf else None
    lib().gbto_predict_sym(
        C.c_void_p(tree["feature"].ctypes.data), C.c_void_p(tree["bin"].ctypes.data),
        C.c_void_p(tree["default_left"].ctypes.data), C.c_void_p(tree["left"].ctypes.data),
        C.c_void_p(tree["right"].ctypes.data), C.c_void_p(tree["weight"].ctypes.data),
        C.c_void_p(sym.ctypes.data), C.c_int64(n), C.c_int32(F), C.c_int32(missing_sym),
        C.c_double(eta), C.c_void_p(margin.ctypes.data),
        C.c_void_p(leaf.ctypes.data) if want_leaf else None)
    return (margin, leaf) if want_leaf else margin


def predict_raw(tree, X, eta, margin, want_leaf=False):
    X = _c(X, np.float32)
    n, F = X.shape
    margin = _c(margin, np.float32).copy()
    leaf = np.empty(n, np.int32) if want_leaf else None
    lib().gbto_predict_raw(
        C.c_void_p(tree["feature"].ctypes.data), C.c_void_p(tree["threshold"].ctypes.data),
        C.c_void_p(tree["default_left"].ctypes.data), C.c_void_p(tree["left"].ctypes.data),
        C.c_void_p(tree["right"].ctypes.data), C.c_void_p(tree["weight"].ctypes.data),
        C.c_void_p(X.ctypes.data), C.c_int64(n), C.c_int32(F), C.c_double(eta),
        C.c_void_p(margin.ctypes.data), C.c_void_p(leaf.ctypes.data) if want_leaf else None)
    return (margin, leaf) if want_leaf else margin


def boost(sym, nb, cuts_, missing_sym, label, *, objective, rounds, eta, base_margin=0.0, **tree_kw):
    """The boosting loop of Fig. 1: gradients -> tree -> margin update."""
    n = sym.shape[0]
    margin = np.full(n, base_margin, np.float32)
    trees = []
    for _ in range(rounds):
        gp = gradients(objective, margin, label)
        t, _, _ = grow_tree(sym, nb, cuts_, missing_sym, gp, **tree_kw)
        margin = predict_sym(t, sym, missing_sym, eta, margin)
        trees.append(t)
    return trees, margin


# -------------------------------------------------------------------- replay --
def _weight_atol(w, denom, atol):
    """How far the leaf weight w = -G / denom (denom = H + lambda) can move when G and H each move by at
    most atol:  |-(G+dG)/(denom+dH) - w| = |dG + w*dH| / |denom + dH| <= (1 + |w|) * atol / (denom - atol).
    (No bound when atol reaches denom: then the other side's H + lambda may be anywhere near zero.)"""
    if atol == 0.0:
        return 0.0
    return (1.0 + abs(w)) * atol / (denom - atol) if denom > atol else np.inf


def _gain_atol(sides, G, H, lam, rtol, atol):
    """How far a reported gain may lie from the oracle's gain of the same candidate when every sum behind it
    (GL, HL, GR, HR, G, H) carries a relative error of rtol and an absolute one of atol.  A term T = S^2 / D
    with D = Hs + lambda moves by at most (2|w| + w^2) * dS for w = S / D, and by 3 * rtol * T; the gain is
    two terms minus a third, so the three allowances add up."""
    tol = 0.0
    for S, Hs in ((sides[0], sides[1]), (sides[2], sides[3]), (G, H)):
        D = Hs + lam
        if D > 0.0:
            w = abs(S) / D
            tol += 3.0 * rtol * S * S / D + (2.0 * w + w * w) * atol
    return tol


def replay_tree(other, sym, nb, missing_sym, gpair, *, max_depth, max_bins, lam=1.0, gamma=0.0,
                min_child_weight=1.0, tie_rtol=1e-6, sum_rtol=1e-5, sum_atol_per_row=0.0,
                nodes=None):
    """Judge a tree grown elsewhere (dict with the fields of ``new_tree``).

    Walks ``other`` from the root with the oracle's OWN row lists.  For every
    node it checks the row count exactly, the (G, H) totals and the leaf weight
    to ``sum_rtol`` (plus ``sum_atol_per_row`` * rows, the other side's stated
    per-row quantisation bound), the gain the other side reports for its split
    (against the oracle's fp64 gain of that same candidate, within what those
    allowances on the sums can move it), and the split decision: identical to
    the oracle's exhaustive best, or its fp64 gain within ``tie_rtol``
    (relative) of the best one.  Children are then formed with the OTHER side's split, so one
    legal tie does not make the rest incomparable.

    ``nodes``: optional set of node ids whose split is searched exhaustively
    (the partition and the totals are always checked for every node).
    Returns a report dict; ``report['ok']`` is the outcome.
    """
    n, F = sym.shape
    B = max_bins
    rows = np.arange(n, dtype=np.uint32)
    leaf_of_row = np.zeros(n, np.int32)
    rep = dict(ok=True, identical=True, n_nodes=int(other["n_nodes"]), ties=[], errors=[],
               checked_splits=0)

    def err(msg):
        rep["ok"] = False
        rep["errors"].append(msg)

    queue = [(0, 0, n, 0)]
    head = 0
    seen = 0
    while head < len(queue):
        node, lo, hi, depth = queue[head]
        head += 1
        seen += 1
        r = rows[lo:hi]
        is_split = other["feature"][node] >= 0
        full = nodes is None or node in nodes
        if int(other["n_rows"][node]) != hi - lo:
            err(f"node {node}: n_rows {int(other['n_rows'][node])} != {hi - lo}")
        if is_split or (full and depth < max_depth):
            h_, cnt, G, H = hist(sym, B, missing_sym, r, gpair)
        else:
            gp = np.asarray(gpair, np.float32)[r].astype(np.float64)
            G, H = float(gp[:, 0].sum()), float(gp[:, 1].sum())
        atol = sum_atol_per_row * (hi - lo)
        for nm, ref, got in (("sumG", G, other["sumG"][node]), ("sumH", H, other["sumH"][node])):
            if abs(got - ref) > sum_rtol * abs(ref) + atol + 1e-300:
                err(f"node {node}: {nm} {got!r} vs {ref!r}")
        w = leaf_weight(G, H, lam)
        w_tol = sum_rtol * abs(w) + _weight_atol(w, H + lam, atol)
        if abs(other["weight"][node] - w) > w_tol + 1e-300:
            err(f"node {node}: weight {other['weight'][node]!r} vs {w!r}")
        thr = max(gamma, GAIN_FLOOR)
        if full:
            rep["checked_splits"] += 1
            best = eval_split(h_, cnt, nb, G, H, hi - lo, lam, min_child_weight) \
                if depth < max_depth else dict(valid=0, gain=-np.inf, feature=-1, bin=0, default_left=0)
            want_split = bool(best["valid"]) and best["gain"] > thr
        if is_split:
            f, b, dl = int(other["feature"][node]), int(other["bin"][node]), int(other["default_left"][node])
            if depth >= max_depth:
                err(f"node {node}: split at depth {depth} >= max_depth")
            if not (0 <= f < F and 0 <= b < nb[f]):
                err(f"node {node}: split ({f},{b}) out of range")
                continue
            g_other, sides = candidate_gain(h_, f, b, dl, G, H, lam, min_child_weight, cnt=cnt, n_rows=hi - lo)
            if not np.isfinite(g_other):
                err(f"node {node}: chosen split ({f},{b},{dl}) is not a valid candidate")
            elif abs(other["gain"][node] - g_other) > _gain_atol(sides, G, H, lam, sum_rtol, atol) + 1e-300:
                err(f"node {node}: reported gain {other['gain'][node]!r} vs {g_other!r} for its own split")
            if np.isfinite(g_other) and full:
                same = (f, b, dl) == (best["feature"], best["bin"], best["default_left"])
                if not same:
                    rep["identical"] = False
                    close = abs(g_other - best["gain"]) <= tie_rtol * abs(best["gain"])
                    rep["ties"].append((node, (f, b, dl), (best["feature"], best["bin"], best["default_left"]),
                                        g_other, best["gain"]))
                    if not close:
                        err(f"node {node}: split ({f},{b},{dl}) gain {g_other!r} vs best "
                            f"({best['feature']},{best['bin']},{best['default_left']}) gain {best['gain']!r}")
                if not want_split and not abs(best["gain"] - thr) <= tie_rtol * max(abs(thr), abs(best["gain"])):
                    err(f"node {node}: split although the best gain {best['gain']!r} is below {thr}")
            out, nl = partition(sym, r, f, b, dl, missing_sym)
            rows[lo:hi] = out
            queue.append((int(other["left"][node]), lo, lo + nl, depth + 1))
            queue.append((int(other["right"][node]), lo + nl, hi, depth + 1))
        else:
            leaf_of_row[r] = node
            if full and want_split:
                rep["identical"] = False
                if not abs(best["gain"] - thr) <= tie_rtol * max(abs(thr), abs(best["gain"])):
                    err(f"node {node}: leaf although best gain {best['gain']!r} > {thr}")
    if seen != int(other["n_nodes"]):
        err(f"reached {seen} nodes, tree says {int(other['n_nodes'])}")
    rep["row_idx"] = rows
    rep["leaf_of_row"] = leaf_of_row
    return rep


def replay_tree_lossguide(other, sym, nb, missing_sym, gpair, *, max_leaves, max_depth, max_bins, lam=1.0,
                          gamma=0.0, min_child_weight=1.0, tie_rtol=1e-6, sum_rtol=1e-5, sum_atol_per_row=0.0):
    """Judge a loss-guided tree grown elsewhere.  The k-th expansion of ``other`` is the node
    whose children are 2k+1 and 2k+2.  Replays the expansions in that order on the oracle's
    own row lists and checks, besides everything ``replay_tree`` checks per node, the policy:
    the expanded node was an open leaf whose chosen split's fp64 gain is within ``tie_rtol``
    (relative) of the largest best gain over the leaves open at that moment, and growth
    stopped only at max_leaves leaves or with no open leaf left (ties at the threshold aside)."""
    n, F = sym.shape
    B = max_bins
    rows = np.arange(n, dtype=np.uint32)
    leaf_of_row = np.zeros(n, np.int32)
    rep = dict(ok=True, identical=True, n_nodes=int(other["n_nodes"]), ties=[], errors=[], checked_splits=0)
    thr = max(gamma, GAIN_FLOOR)

    def err(msg):
        rep["ok"] = False
        rep["errors"].append(msg)

    seg, info = {}, {}   # node -> (lo, hi, depth); node -> (hist, cnt, G, H, best)

    def settle(node, lo, hi, depth):
        r = rows[lo:hi]
        if int(other["n_rows"][node]) != hi - lo:
            err(f"node {node}: n_rows {int(other['n_rows'][node])} != {hi - lo}")
        h_, cnt, G, H = hist(sym, B, missing_sym, r, gpair)
        atol = sum_atol_per_row * (hi - lo)
        for nm, ref, got in (("sumG", G, other["sumG"][node]), ("sumH", H, other["sumH"][node])):
            if abs(got - ref) > sum_rtol * abs(ref) + atol + 1e-300:
                err(f"node {node}: {nm} {got!r} vs {ref!r}")
        w = leaf_weight(G, H, lam)
        if abs(other["weight"][node] - w) > sum_rtol * abs(w) + _weight_atol(w, H + lam, atol) + 1e-300:
            err(f"node {node}: weight {other['weight'][node]!r} vs {w!r}")
        rep["checked_splits"] += 1
        best = eval_split(h_, cnt, nb, G, H, hi - lo, lam, min_child_weight) \
            if depth < max_depth else dict(valid=0, gain=-np.inf, feature=-1, bin=0, default_left=0)
        seg[node] = (lo, hi, depth)
        info[node] = (h_, cnt, G, H, best)

    def open_gain(node):
        best = info[node][4]
        return best["gain"] if bool(best["valid"]) and best["gain"] > thr else -np.inf

    nn = int(other["n_nodes"])
    if nn % 2 != 1 or nn > 2 * max_leaves - 1:
        err(f"n_nodes {nn} is not an odd number <= {2 * max_leaves - 1}")
        return rep
    parent_of = {}
    for node in range(nn):
        if other["feature"][node] >= 0:
            parent_of[int(other["left"][node])] = node
    settle(0, 0, n, 0)
    leaves = {0}
    for k in range((nn - 1) // 2):
        li, ri = 2 * k + 1, 2 * k + 2
        node = parent_of.get(li)
        if node is None or int(other["right"][node]) != ri or node not in leaves:
            err(f"expansion {k}: children {li},{ri} do not hang under one current leaf")
            return rep
        lo, hi, depth = seg[node]
        h_, cnt, G, H, best = info[node]
        f, b, dl = int(other["feature"][node]), int(other["bin"][node]), int(other["default_left"][node])
        if not (0 <= f < F and 0 <= b < nb[f]) or depth >= max_depth:
            err(f"node {node}: split ({f},{b}) out of range or too deep")
            return rep
        g_other, sides = candidate_gain(h_, f, b, dl, G, H, lam, min_child_weight, cnt=cnt, n_rows=hi - lo)
        if not np.isfinite(g_other):
            err(f"node {node}: chosen split ({f},{b},{dl}) is not a valid candidate")
            return rep
        if abs(other["gain"][node] - g_other) > _gain_atol(sides, G, H, lam, sum_rtol, sum_atol_per_row * (hi - lo)) + 1e-300:
            err(f"node {node}: reported gain {other['gain'][node]!r} vs {g_other!r} for its own split")
        if (f, b, dl) != (best["feature"], best["bin"], best["default_left"]):
            rep["identical"] = False
            rep["ties"].append((node, (f, b, dl), (best["feature"], best["bin"], best["default_left"]),
                                g_other, best["gain"]))
            if not abs(g_other - best["gain"]) <= tie_rtol * abs(best["gain"]):
                err(f"node {node}: split ({f},{b},{dl}) gain {g_other!r} vs best gain {best['gain']!r}")
        top = max(open_gain(x) for x in leaves)
        if not g_other >= top - tie_rtol * abs(top):
            err(f"expansion {k}: node {node} (gain {g_other!r}) expanded while a leaf with gain {top!r} was open")
        elif node != min(leaves, key=lambda x: (-open_gain(x), x)):
            rep["identical"] = False
        if not g_other > thr - tie_rtol * max(abs(thr), abs(g_other)):
            err(f"node {node}: split although its gain {g_other!r} is below {thr}")
        out, nl = partition(sym, rows[lo:hi], f, b, dl, missing_sym)
        rows[lo:hi] = out
        leaves.remove(node)
        settle(li, lo, lo + nl, depth + 1)
        settle(ri, lo + nl, hi, depth + 1)
        leaves |= {li, ri}
    if len(leaves) < max_leaves:
        top = max(open_gain(x) for x in leaves)
        if np.isfinite(top) and not abs(top - thr) <= tie_rtol * max(abs(thr), abs(top)):
            rep["identical"] = False
            err(f"stopped at {len(leaves)} leaves although a leaf with gain {top!r} was open")
    for node in leaves:
        if other["feature"][node] >= 0:
            err(f"node {node} is marked as split but has no children among the {nn} nodes")
        lo, hi, _ = seg[node]
        leaf_of_row[rows[lo:hi]] = node
    rep["row_idx"] = rows
    rep["leaf_of_row"] = leaf_of_row
    return rep
