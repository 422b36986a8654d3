"""alpha selection (Section V-C): polynomial fit + smallest feasible alpha,
checked against closed forms."""
import numpy as np
import pytest

from paper_2508_18983_amd.alpha_select import fit_tpot, select_alpha


def test_fit_recovers_a_polynomial_exactly():
    a = np.linspace(0, 0.6, 7)
    t = 120.0 - 80.0 * a + 15.0 * a ** 2
    np.testing.assert_allclose(fit_tpot(a, t, 2), [15.0, -80.0, 120.0], rtol=1e-9)


def test_linear_tpot_gives_the_closed_form_threshold():
    # T(alpha) = 100 - 50 alpha <= R  <=>  alpha >= (100 - R) / 50   (TPOT falls linearly with alpha)
    a = [0.0, 0.1, 0.2, 0.3, 0.4, 0.5, 0.6]
    t = [100 - 50 * v for v in a]
    for budget in (95.0, 90.0, 81.3, 70.0):
        got, _ = select_alpha(a, t, budget, degree=1, resolution=6001)
        assert got == pytest.approx((100 - budget) / 50, abs=1.1e-4)
    assert select_alpha(a, t, 100.0, degree=1)[0] == 0.0          # already within budget: no substitution
    assert select_alpha(a, t, 60.0, degree=1)[0] is None          # unreachable inside the sampled range


def test_quadratic_takes_the_smaller_root_and_noise_is_smoothed():
    a = np.linspace(0, 0.6, 13)
    t = 100 - 90 * a + 60 * a ** 2
    got, coef = select_alpha(a, t, 80.0, degree=2, resolution=60001)
    roots = np.roots([60.0, -90.0, 20.0])
    assert got == pytest.approx(min(roots), abs=2e-5)
    rng = np.random.default_rng(0)
    got_noisy, _ = select_alpha(a, t + rng.normal(0, 0.3, a.size), 80.0, degree=2)
    assert abs(got_noisy - min(roots)) < 0.02


def test_needs_enough_samples():
    with pytest.raises(ValueError):
        fit_tpot([0.0, 0.1], [1.0, 0.9], degree=2)
