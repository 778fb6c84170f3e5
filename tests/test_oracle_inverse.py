"""Pins for the oracle's damped inverse: closed forms and invariants, none of which
re-run the oracle's own Cholesky path."""
import numpy as np
import pytest

import oracle


def spd(d, seed, cond=100.0):
    rng = np.random.default_rng(seed)
    Q, _ = np.linalg.qr(rng.standard_normal((d, d)))
    lam = np.geomspace(1.0, cond, d)
    return (Q * lam) @ Q.T


@pytest.mark.parametrize("d", [1, 2, 3, 17, 64, 129, 300])
def test_residual_symmetry_definiteness(d):
    F, gamma = spd(d, d), 0.03
    X = oracle.damped_inverse(F, gamma)
    M = F + gamma * np.eye(d)
    assert np.linalg.norm(M @ X - np.eye(d)) / np.sqrt(d) < 1e-12
    assert np.linalg.norm(X @ M - np.eye(d)) / np.sqrt(d) < 1e-12
    np.testing.assert_array_equal(X, X.T)
    ev = np.linalg.eigvalsh(X)
    lam = np.linalg.eigvalsh(F)
    assert ev.min() >= 1 / (lam.max() + gamma) * (1 - 1e-10)
    assert ev.max() <= 1 / (lam.min() + gamma) * (1 + 1e-10)


def test_identity_and_diagonal():
    np.testing.assert_allclose(oracle.damped_inverse(np.eye(9), 0.03), np.eye(9) / 1.03, rtol=1e-15)
    dg = np.arange(1.0, 8.0)
    np.testing.assert_allclose(oracle.damped_inverse(np.diag(dg), 0.5), np.diag(1 / (dg + 0.5)), rtol=1e-15, atol=0)


def test_two_by_two_closed_form():
    a, b, c, g = 2.0, 0.7, 1.5, 0.1
    X = oracle.damped_inverse(np.array([[a, b], [b, c]]), g)
    det = (a + g) * (c + g) - b * b
    np.testing.assert_allclose(X, np.array([[c + g, -b], [-b, a + g]]) / det, rtol=1e-14)


@pytest.mark.parametrize("d", [5, 257, 1500])
def test_rank_one_sherman_morrison(d):
    u = np.random.default_rng(d).standard_normal(d)
    g = 0.03
    X = oracle.damped_inverse(np.outer(u, u), g)
    want = (np.eye(d) - np.outer(u, u) / (g + u @ u)) / g
    np.testing.assert_allclose(X, want, rtol=1e-9, atol=1e-9)


def test_against_lu_inverse():
    """numpy.linalg.inv is LU with partial pivoting: a different factorisation."""
    F = spd(200, 11, cond=1e3)
    np.testing.assert_allclose(oracle.damped_inverse(F, 0.01), np.linalg.inv(F + 0.01 * np.eye(200)), rtol=1e-9, atol=1e-11)


def test_gamma_is_added_not_scaled():
    F = spd(6, 12)
    X0 = oracle.damped_inverse(F, 0.0)
    np.testing.assert_allclose(X0 @ F, np.eye(6), atol=1e-12)
    lam, Q = np.linalg.eigh(F)
    np.testing.assert_allclose(oracle.damped_inverse(F, 0.3), (Q / (lam + 0.3)) @ Q.T, rtol=1e-10)


def test_not_positive_definite_info():
    M = np.diag([1.0, 2.0, -1.0, 3.0])
    with pytest.raises(oracle.NotPositiveDefinite) as e:
        oracle.damped_inverse(M, 0.5)
    assert e.value.info == 3
    M = np.array([[1.0, 2.0], [2.0, 1.0]])      # second leading minor = -3
    with pytest.raises(oracle.NotPositiveDefinite) as e:
        oracle.damped_inverse(M, 0.0)
    assert e.value.info == 2
