"""Pins for the cost-model oracle: exact recovery of planted constants, a 3-sample system solved
by hand, the normal equations (residual orthogonal to every regressor), rejection of degenerate
samples."""

import numpy as np
import pytest

from oracle import cost_model as cm


def test_three_samples_by_hand():
    # t = 2*b + 5*i + 7 at (b, i) = (1, 1), (3, 1), (1, 2): 14, 18, 19 -> exact fit, zero residual
    a, c, t0, rms = cm.fit([1, 3, 1], [1, 1, 2], [14.0, 18.0, 19.0])
    assert abs(a - 2) < 1e-12 and abs(c - 5) < 1e-12 and abs(t0 - 7) < 1e-12 and rms < 1e-12


def test_planted_constants_are_recovered():
    rng = np.random.default_rng(0)
    b = rng.integers(2000, 4000, 256)
    i = rng.integers(20, 60, 256)
    t = 3.25 * b + 41.0 * i + 900.0
    a, c, t0, rms = cm.fit(b, i, t)
    assert abs(a - 3.25) < 1e-9 and abs(c - 41.0) < 1e-7 and abs(t0 - 900.0) < 1e-5 and rms < 1e-7
    assert np.allclose(cm.predict(b[:5], i[:5], a, c, t0), t[:5])


def test_residual_is_orthogonal_to_the_regressors():
    rng = np.random.default_rng(1)
    b = rng.integers(100, 900, 64).astype(np.float64)
    i = rng.integers(1, 30, 64).astype(np.float64)
    t = 2.0 * b + 10.0 * i + 50.0 + rng.normal(0, 25.0, 64)
    a, c, t0, rms = cm.fit(b, i, t)
    r = t - np.array(cm.predict(b, i, a, c, t0))
    scale = np.abs(t).sum()
    assert abs(r @ b) < 1e-9 * scale * b.max() and abs(r @ i) < 1e-9 * scale * i.max() and abs(r.sum()) < 1e-9 * scale
    assert abs(rms - np.sqrt(np.mean(r * r))) < 1e-9
    # least squares: any other constants fit worse
    for da, dc, d0 in ((0.01, 0, 0), (0, 0.5, 0), (0, 0, 5.0), (-0.01, -0.5, 3.0)):
        r2 = t - np.array(cm.predict(b, i, a + da, c + dc, t0 + d0))
        assert (r2 * r2).sum() > (r * r).sum()


def test_degenerate_samples_are_rejected():
    with pytest.raises(ValueError):
        cm.fit([1, 2], [1, 2], [1.0, 2.0])
    with pytest.raises(ValueError):
        cm.fit([2, 4, 6, 8], [1, 2, 3, 4], [1.0, 2.0, 3.0, 4.0])       # items proportional to blocks
    with pytest.raises(ValueError):
        cm.fit([5, 5, 5], [1, 2, 3], [1.0, 2.0, 3.0])                  # blocks constant = the intercept column
