"""alpha selection (Section V-C, Eq. 5).  The oracle's select_alpha is pinned by
closed forms and a brute-force scan; the library's (C, reached through the CPU
test shim here and through the C ABI in the GPU tests) must agree with it."""
import ctypes as C
import os

import numpy as np
import pytest

from oracle import smoe_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SHIM = os.path.join(ROOT, "paper_2508_18983_amd", "libsmoe_hostlogic.so")


def lib_select(alphas, tpots, budget, degree=2, resolution=2001):
    lib = C.CDLL(SHIM)
    lib.smoe_hl_select_alpha.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_double, C.c_int, C.c_int,
                                         C.POINTER(C.c_double), C.c_void_p]
    a = np.ascontiguousarray(alphas, np.float64)
    t = np.ascontiguousarray(tpots, np.float64)
    coef = np.zeros(degree + 1)
    out = C.c_double()
    rc = lib.smoe_hl_select_alpha(a.ctypes.data, t.ctypes.data, a.size, budget, degree, resolution,
                                  C.byref(out), coef.ctypes.data)
    assert rc in (0, 1), rc
    return (out.value if rc == 0 else None), coef


# ---------------------------------------------------------------- pins of the oracle
def test_oracle_fit_recovers_a_polynomial_and_matches_the_library_fit():
    a = np.linspace(0, 0.6, 7)
    t = 120.0 - 80.0 * a + 15.0 * a ** 2
    _, coef = O.select_alpha(a, t, 0.0, degree=2)
    np.testing.assert_allclose(coef, [120.0, -80.0, 15.0], rtol=1e-9)
    np.testing.assert_allclose(coef[::-1], np.polyfit(a, t, 2), rtol=1e-9)


def test_oracle_linear_tpot_gives_the_closed_form_threshold():
    # T(alpha) = 100 - 50 alpha <= R  <=>  alpha >= (100 - R) / 50   (TPOT falls linearly with alpha)
    a = [0.0, 0.1, 0.2, 0.3, 0.4, 0.5, 0.6]
    t = [100 - 50 * v for v in a]
    for budget in (95.0, 90.0, 81.3, 70.0):
        got, _ = O.select_alpha(a, t, budget, degree=1, resolution=6001)
        assert got == pytest.approx((100 - budget) / 50, abs=1.1e-4)
        assert got >= (100 - budget) / 50 - 1e-12                  # feasible, and the first feasible point
    assert O.select_alpha(a, t, 100.0, degree=1)[0] == 0.0         # already within budget: no substitution
    assert O.select_alpha(a, t, 60.0, degree=1)[0] is None         # unreachable inside the sampled range


def test_oracle_quadratic_takes_the_smaller_root_and_noise_is_smoothed():
    a = np.linspace(0, 0.6, 13)
    t = 100 - 90 * a + 60 * a ** 2
    got, _ = O.select_alpha(a, t, 80.0, degree=2, resolution=60001)
    roots = np.roots([60.0, -90.0, 20.0])
    assert got == pytest.approx(min(roots), abs=2e-5)
    rng = np.random.default_rng(0)
    got_noisy, _ = O.select_alpha(a, t + rng.normal(0, 0.3, a.size), 80.0, degree=2)
    assert abs(got_noisy - min(roots)) < 0.02


def test_oracle_is_the_first_feasible_grid_point_bruteforce():
    """Independent evaluation: fit with the library polynomial routine, evaluate
    it on the whole grid at once, take the first index under the budget -- also
    for non-monotone fits, where 'smallest feasible' is not 'the root'."""
    rng = np.random.default_rng(4)
    for trial in range(60):
        n = int(rng.integers(4, 10))
        a = np.sort(rng.uniform(0, 0.7, n))
        t = 100 - 60 * a + rng.normal(0, 4.0, n) + 40 * np.sin(5 * a)
        degree = int(rng.integers(1, 4))
        res = 501
        budget = float(np.quantile(t, rng.uniform(0.1, 0.9)))
        got, _ = O.select_alpha(a, t, budget, degree=degree, resolution=res)
        grid = a.min() + (a.max() - a.min()) * np.arange(res) / (res - 1)
        pred = np.polyval(np.polyfit(a, t, degree), grid)
        ok = np.nonzero(pred <= budget)[0]
        # (a point within rounding of the budget may fall either way: skip those draws)
        if np.min(np.abs(pred - budget)) < 1e-7:
            continue
        assert got == (None if ok.size == 0 else pytest.approx(grid[ok[0]], abs=1e-12))


# ---------------------------------------------------------------- the library's host code against the oracle
def test_library_select_alpha_matches_the_oracle():
    rng = np.random.default_rng(9)
    checked = 0
    for trial in range(200):
        n = int(rng.integers(3, 12))
        a = np.sort(rng.uniform(0, 0.6, n))
        if np.min(np.diff(a)) < 1e-3:
            continue
        t = 130 - 95 * a + 30 * a ** 2 + rng.normal(0, 1.5, n)
        degree = int(rng.integers(0, min(4, n - 1) + 1))
        budget = float(rng.uniform(t.min() - 5, t.max() + 5))
        want, wcoef = O.select_alpha(a, t, budget, degree=degree, resolution=1001)
        got, gcoef = lib_select(a, t, budget, degree=degree, resolution=1001)
        np.testing.assert_allclose(gcoef, wcoef, rtol=1e-6, atol=1e-6)
        step = (a.max() - a.min()) / 1000
        if want is None or got is None:
            pred_min = min(sum(wcoef[p] * x ** p for p in range(degree + 1))
                           for x in np.linspace(a.min(), a.max(), 1001))
            assert (want is None and got is None) or abs(pred_min - budget) < 1e-6
        else:
            assert abs(got - want) <= step * 1.0000001           # same grid point, or its neighbour when the
        checked += 1                                              # prediction equals the budget to rounding
    assert checked > 150


def test_library_select_alpha_rejects_bad_input():
    lib = C.CDLL(SHIM)
    lib.smoe_hl_select_alpha.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_double, C.c_int, C.c_int,
                                         C.POINTER(C.c_double), C.c_void_p]
    a = np.array([0.0, 0.1]); t = np.array([1.0, 0.9]); coef = np.zeros(8); out = C.c_double()
    args = (a.ctypes.data, t.ctypes.data)
    assert lib.smoe_hl_select_alpha(*args, 2, 1.0, 2, 100, C.byref(out), coef.ctypes.data) == -1   # n <= degree
    assert lib.smoe_hl_select_alpha(*args, 2, 1.0, 1, 1, C.byref(out), coef.ctypes.data) == -1     # resolution
    same = np.array([0.2, 0.2, 0.2]); t3 = np.array([1.0, 2.0, 3.0])
    assert lib.smoe_hl_select_alpha(same.ctypes.data, t3.ctypes.data, 3, 1.0, 1, 100, C.byref(out),
                                    coef.ctypes.data) == -1                                        # singular
