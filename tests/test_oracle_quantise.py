"""Pins for the oracle's quantile cuts, binning and bit packing (paper Sec. 2.1, 2.2)."""
import numpy as np
import pytest


def test_cuts_permutation_closed_form(oracle):
    # x = a permutation of 0..n-1 with n = k*B: cut j is the order statistic
    # v[floor(j*n/B)] = j*k, and every bin then holds exactly k rows.
    B, k = 16, 25
    n = B * k
    rng = np.random.default_rng(1)
    X = rng.permutation(n).astype(np.float32).reshape(n, 1)
    cuts, nb = oracle.cuts(X, B)
    assert nb[0] == B
    assert np.array_equal(cuts[0], np.arange(1, B) * k)
    sym, missing, mx = oracle.bin_matrix(X, cuts, nb)
    assert mx == B - 1 and missing == B
    assert np.array_equal(np.bincount(sym[:, 0], minlength=B), np.full(B, k))


def test_cuts_few_distinct_is_rank_identity(oracle):
    # d <= B distinct values: each gets its own bin, symbol = rank of the value.
    rng = np.random.default_rng(2)
    vals = np.array([-3.5, -1.0, 0.0, 0.25, 7.0, 1e6], np.float32)
    x = rng.choice(vals, 500).astype(np.float32)
    cuts, nb = oracle.cuts(x.reshape(-1, 1), 8)
    assert nb[0] == 6
    assert np.array_equal(cuts[0][:5], vals[1:])
    assert np.all(np.isinf(cuts[0][5:]))
    sym, _, _ = oracle.bin_matrix(x.reshape(-1, 1), cuts, nb)
    assert np.array_equal(sym[:, 0], np.searchsorted(vals, x))


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_cuts_against_numpy_sort(oracle, seed):
    # the rule re-derived with the library sort: candidates v[(k*m)//B], unique,
    # any candidate equal to the minimum dropped
    rng = np.random.default_rng(seed)
    n, F, B = 3001, 5, 32
    X = rng.standard_normal((n, F)).astype(np.float32)
    X[:, 1] = np.round(X[:, 1] * 2)                     # heavy ties, > B? no: few distinct
    X[:, 2] = np.where(rng.random(n) < 0.7, 0.0, X[:, 2])   # one huge tie at the minimum side
    X[:, 2] = np.abs(X[:, 2])
    X[:, 3] = np.where(rng.random(n) < 0.5, 0.125, X[:, 3])   # many distinct values, half the rows on one of
                                                             # them: several quantile ranks land on it
    X[rng.random((n, F)) < 0.1] = np.nan
    X[:, 4] = np.nan                                     # nothing present
    cuts, nb = oracle.cuts(X, B)
    for f in range(F):
        v = np.sort(X[~np.isnan(X[:, f]), f])
        m = len(v)
        if m == 0:
            assert nb[f] == 1 and np.all(np.isinf(cuts[f]))
            continue
        u = np.unique(v)
        if len(u) <= B:
            want = u[1:]
        else:
            cand = v[(np.arange(1, B) * m) // B]
            if f == 3:
                assert np.count_nonzero(cand == np.float32(0.125)) > 3
            cand = np.unique(cand)
            want = cand[cand != v[0]]
        assert nb[f] == len(want) + 1 <= B
        assert np.array_equal(cuts[f][: len(want)], want)
        assert np.all(np.isinf(cuts[f][len(want):]))
        assert np.all(np.diff(want) > 0)
        assert (v < (want[0] if len(want) else np.inf)).sum() > 0   # bin 0 is not empty


def test_binning_is_searchsorted_right(oracle):
    rng = np.random.default_rng(5)
    n, F, B = 2000, 4, 64
    X = rng.lognormal(0, 1, (n, F)).astype(np.float32)
    X[rng.random((n, F)) < 0.2] = np.nan
    cuts, nb = oracle.cuts(X, B)
    sym, missing, mx = oracle.bin_matrix(X, cuts, nb)
    assert missing == nb.max()
    for f in range(F):
        pres = ~np.isnan(X[:, f])
        ref = np.searchsorted(cuts[f][: nb[f] - 1], X[pres, f], side="right")
        assert np.array_equal(sym[pres, f], ref)
        assert np.all(sym[~pres, f] == missing)
        # definition by counting, on a few rows
        for r in np.flatnonzero(pres)[:20]:
            assert sym[r, f] == sum(1 for c in cuts[f][: nb[f] - 1] if c <= X[r, f])
        # a value equal to a cut falls in the bin to the right of the cut
        for k in range(nb[f] - 1):
            s, _, _ = oracle.bin_matrix(np.full((1, F), cuts[f][k], np.float32), cuts, nb)
            assert s[0, f] == k + 1
        # monotone
        order = np.argsort(X[pres, f], kind="stable")
        assert np.all(np.diff(sym[pres, f][order].astype(int)) >= 0)
    assert mx == sym.max()


def test_bits(oracle):
    # smallest width that holds max_value: 255 -> 8, 256 -> 9, 63 -> 6, 15 -> 4
    table = {0: 1, 1: 1, 2: 2, 3: 2, 4: 3, 15: 4, 16: 5, 63: 6, 64: 7, 255: 8, 256: 9, 511: 9,
             512: 10, 65535: 16}
    for mv, b in table.items():
        assert oracle.bits_for(mv) == b
    for mv in range(1, 2000):
        assert oracle.bits_for(mv) == int(mv).bit_length()


@pytest.mark.parametrize("bits", list(range(1, 17)))
def test_pack_roundtrip_and_packbits(oracle, bits):
    rng = np.random.default_rng(bits)
    n, F = 37, 13
    sym = rng.integers(0, 1 << bits, (n, F)).astype(np.uint16)
    words = oracle.pack(sym, bits)
    assert words.dtype == np.uint32
    assert len(words) == (n * F * bits + 31) // 32 + 1 and words[-1] == 0
    assert np.array_equal(oracle.unpack(words, n * F, bits), sym.reshape(-1))
    # library statement: the little-endian bit matrix, flattened, packed little-endian
    bitmat = ((sym.reshape(-1, 1).astype(np.uint32) >> np.arange(bits)) & 1).astype(np.uint8)
    by = np.packbits(bitmat.reshape(-1), bitorder="little")
    by = np.concatenate([by, np.zeros(len(words) * 4 - len(by), np.uint8)])
    assert np.array_equal(by.view("<u4"), words)


def test_pack_reduces_to_reinterpretation(oracle):
    rng = np.random.default_rng(9)
    s8 = rng.integers(0, 256, (101, 13)).astype(np.uint16)
    w = oracle.pack(s8, 8)
    assert np.array_equal(w.view(np.uint8)[: s8.size], s8.astype(np.uint8).reshape(-1))
    s16 = rng.integers(0, 65536, (55, 3)).astype(np.uint16)
    w = oracle.pack(s16, 16)
    assert np.array_equal(w.view(np.uint16)[: s16.size], s16.reshape(-1))
    # the smallest workload: 10,000 x 8 symbols at 4 bits = 40,000 bytes (+ pad word)
    assert oracle.packed_words(10_000 * 8, 4) * 4 == 40_000 + 4
