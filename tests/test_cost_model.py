"""The alpha-beta computation-cost fit (paper Eq. 12): recovers known coefficients, minimises the
relative error, and rejects degenerate input."""
import numpy as np
import pytest

from paper_2412_01523_amd import cost_model as cm


def _batches(rng, n):
    out = []
    for i in range(n):
        k = int(rng.integers(1, 40))
        out.append([int(x) for x in rng.integers(64, 20000, size=k)])
    return out


def test_features_are_sum_of_squares_sum_and_one():
    assert cm.features([3, 4]).tolist() == [25.0, 7.0, 1.0]
    assert cm.features([]).tolist() == [0.0, 0.0, 1.0]


def test_fit_recovers_exact_coefficients():
    rng = np.random.default_rng(3)
    b = _batches(rng, 12)
    true = (3.1e-9, 4.7e-6, 0.02)
    t = [cm.predict(true, x) for x in b]
    got = cm.fit(b, t)
    assert np.allclose(got, true, rtol=1e-8)
    assert np.abs(cm.relative_errors(got, b, t)).max() < 1e-10


def test_fit_is_closed_form_weighted_least_squares():
    # independent formulation: normal equations of the 1/t-weighted problem
    rng = np.random.default_rng(5)
    b = _batches(rng, 20)
    t = np.array([cm.predict((2e-9, 1e-6, 0.05), x) for x in b]) * (1 + 0.03 * rng.standard_normal(20))
    X = np.stack([cm.features(x) for x in b]) / t[:, None]
    want = np.linalg.solve(X.T @ X, X.T @ np.ones(20))
    assert np.allclose(cm.fit(b, t), want, rtol=1e-6)
    # 3 % noise on the measurements leaves the fit within a few per cent
    assert np.abs(cm.relative_errors(cm.fit(b, t), b, t)).max() < 0.12


def test_fit_rejects_degenerate_input():
    with pytest.raises(ValueError):
        cm.fit([[1], [2]], [1.0, 2.0])
    with pytest.raises(ValueError):
        cm.fit([[1], [2], [3]], [1.0, 0.0, 2.0])
