"""gbt_partition_static: the stable partition over the library's static scratch array, for callers that
cannot allocate (-m gpu).  It must give exactly what gbt_partition gives (and what the oracle's stable
filter gives), on two calls in a row, the second on a smaller input than the first, so that whatever the
first call left in the array is still there when the second runs."""
import numpy as np
import pytest
import torch

import synth
from gpu_util import dev, host_u32, oracle_prep

pytestmark = pytest.mark.gpu


def _case(ctx, oracle, cfg, n, seed):
    d = synth.make(cfg, n)
    X = d["X"]
    n, F = X.shape
    o = oracle_prep(oracle, X, d["params"]["max_bins"])
    packed = dev(o["words"].view(np.int32))
    rng = np.random.default_rng(seed)
    rows = np.sort(rng.choice(n, max(1, (2 * n) // 3), replace=False)).astype(np.uint32)
    f = int(rng.integers(0, F))
    b = int(rng.integers(0, max(1, o["nb"][f] - 1)))
    dl = int(rng.integers(0, 2))
    begin, end = len(rows) // 7, len(rows) - len(rows) // 11      # a segment strictly inside the list
    print(f"partition_static C{cfg} n={n} F={F} bits={o['bits']} segment [{begin}, {end}) split ({f},{b},{dl})", flush=True)
    a = dev(rows.view(np.int32))
    s = a.clone()
    nl_a = ctx.partition(packed, o["bits"], n, F, a, begin, end, f, b, dl, o["missing"])
    nl_s = ctx.partition_static(packed, o["bits"], n, F, s, begin, end, f, b, dl, o["missing"])
    ref, nl = oracle.partition(o["sym"], rows[begin:end], f, b, dl, o["missing"])
    assert nl_s == nl_a == nl
    assert torch.equal(s, a)                                           # bit for bit what the existing call gives
    got = host_u32(s)
    assert np.array_equal(got[begin:end], ref)                         # and the oracle's stable filter
    assert np.array_equal(got[:begin], rows[:begin]) and np.array_equal(got[end:], rows[end:])   # the rest untouched


def test_partition_static_matches_partition_twice_in_a_row(oracle):
    import paper_1806_11248_amd as g
    ctx = g.Context(0)
    try:
        _case(ctx, oracle, 3, 300_000, 1)     # 9-bit symbols with missing values, several hundred tiles, a ragged tail
        _case(ctx, oracle, 4, 41_003, 2)      # then a smaller input over the same scratch array
        _case(ctx, oracle, 1, 777, 3)         # and a segment shorter than one tile
        # an empty segment, and the size limit
        d = synth.make(1, 100)
        o = oracle_prep(oracle, d["X"], 16)
        packed = dev(o["words"].view(np.int32))
        idx = dev(np.arange(100, dtype=np.int32))
        assert ctx.partition_static(packed, o["bits"], 100, 8, idx, 5, 5, 0, 0, 0, o["missing"]) == 0
        big = g.binding.PARTITION_STATIC_MAX_ROWS + 1
        with pytest.raises(g.GbtError) as e:
            ctx.partition_static(packed, o["bits"], big, 8, idx, 0, big, 0, 0, 0, o["missing"])
        assert e.value.code == g.binding.EUNSUPPORTED and "static scratch" in str(e.value)
    finally:
        ctx.close()
