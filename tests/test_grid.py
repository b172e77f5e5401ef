"""Pins of tests/grid.py, the test-side restatement of the GPU library's fixed-point grid (CPU only)."""
import numpy as np

import grid


def test_fixed_point_grid():
    # the scale: the power of two that puts the largest magnitude into [2^25, 2^26) (g) or [2^21, 2^22) (h)
    gp = np.array([[0.75, 0.25], [-3.0, 0.0], [1e-3, 1.0]], np.float32)
    q, scale = grid.fixed_point(gp)
    assert scale == (2.0 ** 24, 2.0 ** 21)
    assert q.tolist() == [[3 * 2 ** 22, 2 ** 19], [-3 * 2 ** 24, 0], [16777, 2 ** 21]]   # 1e-3 * 2^24 = 16777.216
    assert grid.fixed_point(np.array([[0.99, 0.49]], np.float32))[1] == (2.0 ** 26, 2.0 ** 23)
    assert grid.fixed_point(np.zeros((4, 2), np.float32))[1] == (1.0, 1.0)
    assert grid.fixed_point(np.zeros((0, 2), np.float32))[1] == (1.0, 1.0)
    # ties go to the even integer: 2.5 and 3.5 quanta (the 1.0 fixes the quantum at 2^-25)
    q, scale = grid.fixed_point(np.array([[1.0, 1.0], [2.5 * 2.0 ** -25, 3.5 * 2.0 ** -21]], np.float32))
    assert scale == (2.0 ** 25, 2.0 ** 21) and q[1].tolist() == [2, 4]
    rng = np.random.default_rng(4)
    for sg, sh in ((1.0, 1.0), (1e-6, 3e4), (7e5, 1e-3)):
        gp = np.stack([rng.standard_normal(5000) * sg, rng.uniform(0, 1, 5000) * sh], 1).astype(np.float32)
        q, scale = grid.fixed_point(gp)
        for c, top in ((0, 26), (1, 22)):
            m = np.abs(q[:, c].astype(np.int64)).max()
            assert 2 ** (top - 1) <= m <= 2 ** top and np.log2(scale[c]) == np.round(np.log2(scale[c]))
        assert np.all(np.abs(q / np.array(scale) - gp.astype(np.float64)) <= 0.5 / np.array(scale))   # one rounding
        og = grid.on_grid(gp)
        assert og.dtype == np.float32 and np.array_equal(og.astype(np.float64) * np.array(scale), q)
        q2, scale2 = grid.fixed_point(og)                                # already on the grid: nothing moves
        assert scale2 == scale and np.array_equal(q2, q)
        # sums of on-grid values are exact in fp64 whatever the order
        assert og[:, 0].astype(np.float64).sum() == og[::-1, 0].astype(np.float64).sum() == q[:, 0].astype(np.int64).sum() / scale[0]
