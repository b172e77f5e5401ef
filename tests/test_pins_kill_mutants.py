"""Do the oracle's pins notice a mistake?  Each case below plants ONE plausible mistake (a wrong sign, a
dropped term, an off-by-one index, a transposed operand, a swapped branch) into a COPY of the oracle, on
the CPU, and runs the oracle's pin tests (tests/test_oracle_*.py) against that copy in a child process:
at least one pin has to fail.  A mistake that no pin sees fails THIS test, naming the mistake.

The copies live in a temporary directory; the oracle under ``oracle/`` is never changed, and nothing here
touches the GPU library.
"""
import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor


ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PIN_FILES = ["test_oracle_quantise.py", "test_oracle_steps.py", "test_oracle_tree.py", "test_oracle_lossguide.py"]

C, PY = "gbt_oracle.c", "__init__.py"

# (name, file, which occurrence of `old` (1-based; 0 = every occurrence), old, new)
MUTANTS = [
    # Sec. 2.1: quantile cuts and binning
    ("cut index one too low", C, 1, "v[(int64_t)(((__int128)k * m) / B)]", "v[(int64_t)(((__int128)k * m) / B) - 1]"),
    ("cut rank rounded to the next multiple", C, 1, "((__int128)k * m) / B)]", "((__int128)k * (m - 1)) / B)]"),
    ("repeated cuts kept", C, 1, "if (nc > 0 && cuts_out[nc - 1] == c) continue;", ""),
    ("a value equal to a cut goes below it", C, 1, "if (c[mid] <= x) lo = mid + 1; else hi = mid;",
     "if (c[mid] < x) lo = mid + 1; else hi = mid;"),
    ("few distinct values: first value becomes a cut", C, 1,
     "for (int64_t i = 1; i < m; ++i) if (v[i] != v[i - 1]) cuts_out[nc++] = v[i];",
     "cuts_out[nc++] = v[0]; for (int64_t i = 1; i < m && nc < B - 1; ++i) if (v[i] != v[i - 1]) cuts_out[nc++] = v[i];"),
    ("a cut equal to the smallest value kept (bin 0 empty)", C, 1, "if (c == v[0]) continue;", ""),
    ("a missing value gets symbol 0", C, 1, "s = missing_sym;", "s = 0;"),
    # Sec. 2.2: bit width and packing
    ("one bit too few", C, 1, "(max_value >> bits) != 0", "(max_value >> bits) > 1"),
    ("bits of a word filled from the top", C, 1, "(uint32_t)1 << (p & 31)", "(uint32_t)1 << (31 - (p & 31))"),
    ("element bits reversed on unpack", C, 1, "& 1u) << j;", "& 1u) << (bits - 1 - j);"),
    ("no pad word after the stream", C, 1, "return (n_elems * bits + 31) / 32 + 1;", "return (n_elems * bits + 31) / 32;"),
    # Sec. 2.5: gradients
    ("sign of the logistic gradient", C, 1, "g = p - y;", "g = y - p;"),
    ("logistic hessian p(1+p)", C, 1, "h = p * (1.0 - p);", "h = p * (1.0 + p);"),
    ("sigmoid of the wrong sign", C, 1, "1.0 / (1.0 + exp(-m))", "1.0 / (1.0 + exp(m))"),
    ("squared error gradient reversed", C, 1, "g = m - y;", "g = y - m;"),
    # Alg. 1: histogram
    ("h summed from g", C, 1, "hf[2 * s + 1] += (double)gpair[2 * r + 1];", "hf[2 * s + 1] += (double)gpair[2 * r];"),
    ("row list ignored in the bins", C, 1, "int64_t r = rows ? (int64_t)rows[i] : i;", "int64_t r = i;"),
    ("row list ignored in the totals", C, 2, "int64_t r = rows ? (int64_t)rows[i] : i;", "int64_t r = i;"),
    ("symbols read with the wrong stride", C, 1, "uint32_t s = sym[r * F + f];", "uint32_t s = sym[f * F + r % F];"),
    # Alg. 1 / Sec. 2.3: split evaluation
    ("parent term added", C, 1, "return (a + b) - c;", "return (a + b) + c;"),
    ("lambda dropped from the parent term", C, 1, "double c = term(G, H, lambda);", "double c = term(G, H, 0.0);"),
    ("terms not squared", C, 1, "return d > 0.0 ? G * G / d : 0.0;", "return d > 0.0 ? G / d : 0.0;"),
    ("a side without curvature prices as infinite", C, 1, "return d > 0.0 ? G * G / d : 0.0;", "return G * G / d;"),
    ("right term over the left hessian", C, 1, "double b = term(GR, HR, lambda);", "double b = term(GR, HL, lambda);"),
    ("a side without rows may win", C, 1, "if (n_left == 0 || n_left == n_rows) continue;",
     "if (b == nb[f] - 1 && (dir == 1 || !has_missing)) continue;"),
    ("a named candidate with a side without rows is priced", C, 1, "if (n_left == 0 || n_left == n_rows) return NAN; /* a side without rows is no split */", ""),
    ("a named candidate forgets the rows of the missing side", C, 1, "if (default_left) { GL += Gm; HL += Hm; n_left += n_rows - present; }",
     "if (default_left) { GL += Gm; HL += Hm; }"),
    ("rows of the missing side not counted", C, 1, "int64_t n_left = pc + (dir == 1 ? n_rows - present : 0);", "int64_t n_left = pc;"),
    ("later candidate wins ties", C, 1, "if (gain > best.gain) {", "if (gain >= best.gain) {"),
    ("missing mass on the wrong side", C, 1, "if (dir == 1) { GL += Gm; HL += Hm; }", "if (dir == 0) { GL += Gm; HL += Hm; }"),
    ("missing mass with the wrong sign", C, 2, "double Gm = G - sg, Hm = H - sh;", "double Gm = sg - G, Hm = sh - H;"),
    ("right child's weight not checked", C, 1, "if (!(HL >= min_child_weight) || !(HR >= min_child_weight)) continue;",
     "if (!(HL >= min_child_weight)) continue;"),
    ("prefix sum skips the split bin", C, 1, "for (int32_t b = 0; b < nb[f]; ++b) {\n            pg += hf[2 * b];\n            ph += hf[2 * b + 1];",
     "for (int32_t b = 0; b < nb[f]; ++b) {\n            if (b) { pg += hf[2 * b - 2]; ph += hf[2 * b - 1]; }"),
    ("named candidate: prefix excludes its bin", C, 1, "for (int32_t k = 0; k <= b; ++k) { GL += hf[2 * k]; HL += hf[2 * k + 1]; n_left += cf[k]; }",
     "for (int32_t k = 0; k < b; ++k) { GL += hf[2 * k]; HL += hf[2 * k + 1]; n_left += cf[k]; }"),
    ("named candidate: default side ignored", C, 1, "if (default_left) { GL += Gm; HL += Hm; n_left += n_rows - present; }", ""),
    ("named candidate: child weights not checked", C, 1,
     "if (!(HL >= min_child_weight) || !(HR >= min_child_weight)) return NAN;", ""),
    # Alg. 1: repartition
    ("boundary bin goes right", C, 0, "int left = (s == missing_sym) ? default_left : (s <= bin);",
     "int left = (s == missing_sym) ? default_left : (s < bin);"),
    ("missing rows ignore the default side", C, 0, "int left = (s == missing_sym) ? default_left : (s <= bin);",
     "int left = (s <= bin);"),
    ("right part written backwards", C, 1, "if (!left) rows_out[k++] = rows[i];", "if (!left) rows_out[n_rows - 1 - (k++ - nl)] = rows[i];"),
    # Sec. 2.4: prediction
    ("prediction: boundary bin goes right", C, 1, "(s <= bin[node])", "(s < bin[node])"),
    ("prediction on floats: value equal to the threshold goes left", C, 1, "(x < threshold[node])", "(x <= threshold[node])"),
    ("prediction: children swapped", C, 1, "node = go_left ? left[node] : right[node];", "node = go_left ? right[node] : left[node];"),
    ("prediction: learning rate ignored", C, 1, "(double)margin_inout[r] + eta * weight[node]", "(double)margin_inout[r] + weight[node]"),
    ("prediction: missing value takes the other side", C, 1, "(s == missing_sym) ? default_left[node]", "(s == missing_sym) ? !default_left[node]"),
    ("prediction on floats: NaN takes the other side", C, 1, "isnan(x) ? default_left[node]", "isnan(x) ? !default_left[node]"),
    # the tree drivers
    ("leaf weight sign", PY, 1, "return -G / (H + lam) if H + lam > 0.0 else 0.0", "return G / (H + lam) if H + lam > 0.0 else 0.0"),
    ("leaf weight without lambda", PY, 1, "return -G / (H + lam) if H + lam > 0.0 else 0.0", "return -G / H if H > 0.0 else 0.0"),
    ("leaf weight without curvature is not 0", PY, 1, "return -G / (H + lam) if H + lam > 0.0 else 0.0",
     "return -G / (H + lam) if H + lam > 0.0 else -np.sign(G) * np.inf"),
    ("children recorded the other way round", PY, 1, 't["left"][node], t["right"][node], t["gain"][node] = li, ri, sp["gain"]',
     't["left"][node], t["right"][node], t["gain"][node] = ri, li, sp["gain"]'),
    ("threshold is the cut below", PY, 1, "return np.float32(cuts_[f, b]) if b < nb[f] - 1", "return np.float32(cuts_[f, b - 1]) if b < nb[f] - 1"),
    ("gamma ignored", PY, 1, 'bool(sp["valid"]) and sp["gain"] > gamma and sp["gain"] > GAIN_FLOOR', 'bool(sp["valid"]) and sp["gain"] > GAIN_FLOOR'),
    ("grows one level too deep", PY, 1, "if depth < max_depth:", "if depth <= max_depth:"),
    ("children's row ranges swapped", PY, 1, "queue.append((li, lo, lo + nl, depth + 1))\n        queue.append((ri, lo + nl, hi, depth + 1))",
     "queue.append((ri, lo, lo + nl, depth + 1))\n        queue.append((li, lo + nl, hi, depth + 1))"),
    ("loss-guided: smallest gain first", PY, 1, 'key=lambda k: (-open_[k]["gain"], k)', 'key=lambda k: (open_[k]["gain"], k)'),
    ("loss-guided: larger id first on equal gains", PY, 1, 'key=lambda k: (-open_[k]["gain"], k)', 'key=lambda k: (-open_[k]["gain"], -k)'),
    ("loss-guided: one leaf too many", PY, 1, "while n_leaves < max_leaves and open_:", "while n_leaves <= max_leaves and open_:"),
    ("loss-guided: leaf weight sign", PY, 2, 't["weight"][node] = leaf_weight(G, H, lam)', 't["weight"][node] = -leaf_weight(G, H, lam)'),
    ("boosting: margin not carried over", PY, 1, "margin = predict_sym(t, sym, missing_sym, eta, margin)",
     "margin = predict_sym(t, sym, missing_sym, eta, np.full(n, base_margin, np.float32))"),
    ("judge: accepts any gain", PY, 1, "close = abs(g_other - best[\"gain\"]) <= tie_rtol * abs(best[\"gain\"])", "close = True"),
    ("judge: reported gains not compared", PY, 1, "elif abs(other[\"gain\"][node] - g_other) > _gain_atol(sides, G, H, lam, sum_rtol, atol) + 1e-300:", "elif False:"),
    ("loss-guided judge: reported gains not compared", PY, 1,
     "if abs(other[\"gain\"][node] - g_other) > _gain_atol(sides, G, H, lam, sum_rtol, sum_atol_per_row * (hi - lo)) + 1e-300:", "if False:"),
    ("judge: row counts not compared", PY, 1, 'if int(other["n_rows"][node]) != hi - lo:', "if False:"),
    ("judge: leaf weights not compared", PY, 1, 'if abs(other["weight"][node] - w) > w_tol + 1e-300:', "if False:"),
    ("judge: weight tolerance without the hessian's share", PY, 1, "    return (1.0 + abs(w)) * atol / (denom - atol) if denom > atol else np.inf",
     "    return atol / (denom - atol) if denom > atol else np.inf"),
    ("judge: totals not compared", PY, 1, "if abs(got - ref) > sum_rtol * abs(ref) + atol + 1e-300:", "if False:"),
    ("judge: a split below the threshold is accepted", PY, 1,
     'err(f"node {node}: split although the best gain {best[\'gain\']!r} is below {thr}")', "pass"),
    ("judge: a split below the depth limit is accepted", PY, 1, 'err(f"node {node}: split at depth {depth} >= max_depth")', "pass"),
    ("judge: an invalid candidate is accepted", PY, 1, 'err(f"node {node}: chosen split ({f},{b},{dl}) is not a valid candidate")', "pass"),
    ("loss-guided judge: totals not compared", PY, 2, "if abs(got - ref) > sum_rtol * abs(ref) + atol + 1e-300:", "if False:"),
    ("judge: a leaf that should split is accepted", PY, 1, 'err(f"node {node}: leaf although best gain {best[\'gain\']!r} > {thr}")', "pass"),
    ("loss-guided judge: order of expansions not checked", PY, 1, "if not g_other >= top - tie_rtol * abs(top):", "if False:"),
    ("loss-guided judge: early stop accepted", PY, 1, 'err(f"stopped at {len(leaves)} leaves although a leaf with gain {top!r} was open")', "pass"),
]


def _replace_nth(text, old, new, nth):
    if nth == 0:
        return text.replace(old, new) if old in text else None
    pos = -1
    for _ in range(nth):
        pos = text.find(old, pos + 1)
        if pos < 0:
            return None
    return text[:pos] + new + text[pos + len(old):]


def _plant(tmp, idx, mutant):
    name, fname, nth, old, new = mutant
    root = os.path.join(tmp, f"m{idx:02d}")
    os.makedirs(os.path.join(root, "oracle"))
    os.makedirs(os.path.join(root, "tests"))
    for f in (C, PY):
        shutil.copy(os.path.join(ROOT, "oracle", f), os.path.join(root, "oracle", f))
    shutil.copytree(os.path.join(ROOT, "synth"), os.path.join(root, "synth"), ignore=shutil.ignore_patterns("__pycache__"))
    shutil.copytree(os.path.join(ROOT, "tests", "golden"), os.path.join(root, "tests", "golden"))
    for f in PIN_FILES + ["conftest.py"]:
        shutil.copy(os.path.join(ROOT, "tests", f), os.path.join(root, "tests", f))
    path = os.path.join(root, "oracle", fname)
    text = _replace_nth(open(path).read(), old, new, nth)
    if text is None:
        return root, f"{name}: the text to replace was not found in oracle/{fname} (update the list)"
    open(path, "w").write(text)
    return root, None


def _run(root):
    env = dict(os.environ, PYTHONDONTWRITEBYTECODE="1", OMP_NUM_THREADS="2")
    env.pop("PYTHONPATH", None)
    try:
        p = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "--no-header",
                            *[os.path.join("tests", f) for f in PIN_FILES]],
                           cwd=root, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, timeout=300)
        return p.returncode, p.stdout.decode(errors="replace")
    except subprocess.TimeoutExpired:
        return 124, "timeout"


def test_unchanged_copy_passes_and_every_planted_mistake_is_caught(tmp_path):
    tmp = str(tmp_path)
    # the harness itself: an unchanged copy must pass, or "fails" below would mean nothing
    root, _ = _plant(tmp, 99, ("none", PY, 1, '"""CPU oracle', '"""CPU oracle'))
    code, out = _run(root)
    assert code == 0, out[-3000:]
    assert os.path.exists(os.path.join(root, "oracle", "libgbt_oracle.so"))   # it was the copy that was built and run

    planted = [_plant(tmp, i, m) for i, m in enumerate(MUTANTS)]
    stale = [msg for _, msg in planted if msg]
    assert not stale, stale
    with ThreadPoolExecutor(max_workers=4) as pool:
        results = list(pool.map(lambda pr: _run(pr[0]), planted))
    survivors = [m[0] for m, (code, _) in zip(MUTANTS, results) if code == 0]
    assert not survivors, f"no pin notices: {survivors}"
    # "caught" has to mean that a pin ran and failed (pytest's exit code 1 with a test named), not that the
    # copy did not compile, import or collect, or that it crashed
    unclear = [(m[0], code, out[-300:]) for m, (code, out) in zip(MUTANTS, results)
               if code != 1 or not any(l.startswith(("FAILED tests/", "ERROR tests/")) for l in out.splitlines())]
    assert not unclear, unclear
