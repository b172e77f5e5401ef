"""The fixed-point grid that the GPU library declares for its sums (include/gbt.h, gbt_gpair_fixed),
restated on the TEST side.  Not part of the oracle and not from the paper: it lets a decision that
rounding could tip (is this child heavy enough? which of two close gains is larger?) be judged in the
library's own precision, in addition to the plain fp64 judgement.  Pinned by tests/test_grid.py on the
CPU and compared bit for bit with gbt_gpair_fixed on the GPU."""
import numpy as np

G_TOP, H_TOP = 26, 22


def fixed_point(gpair: np.ndarray):
    """The library rounds every g to an integer multiple of 1/scale_g and every h to one of 1/scale_h,
    ties to even, with power-of-two scales: for a largest magnitude m * 2^e (0.5 <= m < 1) the scale is
    2^(26 - e) for g and 2^(22 - e) for h, 1 when all are zero.
    Returns (q int32 [n][2], (scale_g, scale_h))."""
    gp = np.ascontiguousarray(gpair, np.float32).astype(np.float64)
    scale = []
    for col, top in ((0, G_TOP), (1, H_TOP)):
        vmax = float(np.abs(gp[:, col]).max()) if len(gp) else 0.0
        scale.append(2.0 ** (top - np.frexp(vmax)[1]) if vmax > 0.0 else 1.0)
    q = np.rint(gp * np.array(scale)).astype(np.int32)
    return q, (scale[0], scale[1])


def on_grid(gpair: np.ndarray) -> np.ndarray:
    """The pairs moved onto that grid, as fp32 (exact: an fp32 value scaled by a power of two and rounded
    to an integer still fits 24 bits).  Sums of these in fp64 are exact, so a tree judged on them is judged
    in the GPU library's own precision."""
    q, scale = fixed_point(gpair)
    out = (q.astype(np.float64) / np.array(scale)).astype(np.float32)
    assert np.array_equal(out.astype(np.float64) * np.array(scale), q)
    return out
