"""CPU checks of the closed forms the second orthonormalisation round of the HIP path relies on
(Newton-Schulz corrections of a nearly orthonormal basis).  Pure numpy; no kernel is called: the
coefficients and acceptance levels written here are the ones the kernels use, and the parity tests
on the GPU exercise the kernels themselves.

With E = Q1^T Q1 - I symmetric and ||E||_2 < 1, Q = Q1 (I + E)^(-1/2) is orthonormal and
  (I + E)^(-1/2) = I - E/2 + 3 E^2/8 - 5 E^3/16 + 35 E^4/128 - 63 E^5/256 + ...
"""
import numpy as np
import pytest


def _near_orthonormal(m, k, e_norm2, seed):
    rng = np.random.default_rng(seed)
    q, _ = np.linalg.qr(rng.standard_normal((m, k)))
    s = rng.standard_normal((k, k))
    s = (s + s.T) / 2
    s *= e_norm2 / np.linalg.norm(s, 2)
    # Q1 = Q (I + S)^(1/2)  =>  Q1^T Q1 = I + S exactly
    w, v = np.linalg.eigh(np.eye(k) + s)
    return q @ (v * np.sqrt(w)) @ v.T


@pytest.mark.parametrize("e_norm2", [1e-3, 0.015, 0.1, 0.2])
def test_first_order_correction_leaves_three_quarters_of_e_squared(e_norm2):
    q1 = _near_orthonormal(400, 24, e_norm2, seed=1)
    e = q1.T @ q1 - np.eye(24)
    q = q1 @ (np.eye(24) - e / 2)
    defect = np.linalg.norm(q.T @ q - np.eye(24), 2)
    # (I - E/2)(I + E)(I - E/2) - I = -3E^2/4 + E^3/4
    assert defect <= 0.75 * e_norm2 ** 2 + 0.25 * e_norm2 ** 3 + 1e-14
    assert defect >= 0.5 * e_norm2 ** 2 or e_norm2 < 1e-6


@pytest.mark.parametrize("e_norm2", [0.05, 0.12, 0.2])
def test_degree_four_series_defect_is_below_its_first_dropped_term(e_norm2):
    k = 32
    q1 = _near_orthonormal(600, k, e_norm2, seed=2)
    e = q1.T @ q1 - np.eye(k)
    e2 = e @ e
    t = -0.5 * e + 0.375 * e2 - 0.3125 * e2 @ e + 0.2734375 * e2 @ e2      # the four coefficients
    q = q1 @ (np.eye(k) + t)
    defect = np.linalg.norm(q.T @ q - np.eye(k), 2)
    # the polynomial misses (I + E)^(-1/2) by 63/256 E^5 (1 + O(E)); squared against I + E that is
    # twice as much to first order
    bound = 2 * (63 / 256) * e_norm2 ** 5 / (1 - e_norm2) ** 2
    assert defect <= bound, (defect, bound)
    # at the acceptance level ||E||_2 <= 0.2 this is far inside the 1e-3 orthogonality tolerance
    assert 2 * (63 / 256) * 0.2 ** 5 / 0.8 ** 2 < 3e-4


def test_frobenius_norm_of_the_fourth_power_bounds_the_spectral_norm():
    # the kernels accept the series on ||E^4||_F^(1/4) <= 0.2, a computable upper bound of ||E||_2
    rng = np.random.default_rng(3)
    for k in (8, 64):
        s = rng.standard_normal((k, k))
        e = (s + s.T) * 0.01
        e4 = np.linalg.matrix_power(e, 4)
        assert np.linalg.norm(e, 2) <= np.linalg.norm(e4, "fro") ** 0.25 + 1e-15
        assert np.linalg.norm(e4, "fro") ** 0.25 <= k ** 0.125 * np.linalg.norm(e, 2) + 1e-15


def test_a_wrong_series_coefficient_is_caught():
    k = 16
    q1 = _near_orthonormal(300, k, 0.2, seed=4)
    e = q1.T @ q1 - np.eye(k)
    e2 = e @ e
    t_bad = -0.5 * e + 0.375 * e2 - 0.25 * e2 @ e + 0.2734375 * e2 @ e2    # planted: 5/16 -> 4/16
    q = q1 @ (np.eye(k) + t_bad)
    defect = np.linalg.norm(q.T @ q - np.eye(k), 2)
    assert defect > 2 * (63 / 256) * 0.2 ** 5 / 0.8 ** 2
