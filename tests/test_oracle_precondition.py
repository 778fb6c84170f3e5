"""Pins for the oracle's preconditioning and for a whole step on the small FC workload."""
import numpy as np
import pytest

import oracle
from synth import shapes, inputs


def test_bruteforce_kronecker_solve():
    """(A+gI) (x) (G+gI) applied to the column-stacked P must give back the column-stacked V."""
    rng = np.random.default_rng(0)
    dA, dG, g = 7, 4, 0.03
    ra, rg = rng.standard_normal((20, dA)), rng.standard_normal((20, dG))
    A, G = ra.T @ ra / 20, rg.T @ rg / 20
    V = rng.standard_normal((dG, dA))
    P = oracle.precondition(oracle.damped_inverse(G, g), oracle.damped_inverse(A, g), V)
    K = np.kron(A + g * np.eye(dA), G + g * np.eye(dG))          # acts on vec_col of a [dG, dA] matrix
    p = np.linalg.solve(K, V.flatten(order="F"))
    np.testing.assert_allclose(P.flatten(order="F"), p, rtol=1e-10, atol=1e-12)
    # element-wise definition of the two-sided product with plain loops
    XG, XA = oracle.damped_inverse(G, g), oracle.damped_inverse(A, g)
    for i in range(dG):
        for j in range(dA):
            s = sum(XG[i, k] * V[k, l] * XA[l, j] for k in range(dG) for l in range(dA))
            assert P[i, j] == pytest.approx(s, rel=1e-10, abs=1e-13)


def test_sides_are_not_swapped():
    """Distinct diagonal inverses: rows are scaled by X_G and columns by X_A."""
    XG, XA = np.diag([1.0, 2.0]), np.diag([3.0, 5.0, 7.0])
    V = np.ones((2, 3))
    np.testing.assert_array_equal(oracle.precondition(XG, XA, V), np.outer([1.0, 2.0], [3.0, 5.0, 7.0]))


def test_identity_linearity_roundtrip():
    rng = np.random.default_rng(1)
    V, W = rng.standard_normal((5, 9)), rng.standard_normal((5, 9))
    np.testing.assert_array_equal(oracle.precondition(np.eye(5), np.eye(9), V), V)
    ra, rg = rng.standard_normal((30, 9)), rng.standard_normal((30, 5))
    A, G, g = ra.T @ ra / 30, rg.T @ rg / 30, 0.03
    XA, XG = oracle.damped_inverse(A, g), oracle.damped_inverse(G, g)
    np.testing.assert_allclose(oracle.precondition(XG, XA, 2 * V - 3 * W),
                               2 * oracle.precondition(XG, XA, V) - 3 * oracle.precondition(XG, XA, W), rtol=1e-11, atol=1e-12)
    P = oracle.precondition(XG, XA, V)
    np.testing.assert_allclose((G + g * np.eye(5)) @ P @ (A + g * np.eye(9)), V, rtol=1e-10, atol=1e-12)


def test_fc_config_three_steps():
    """The small FC workload, all three steps at full size, against closed forms that hold per step."""
    hp = shapes.config_hparams("fc")
    layer = shapes.config_layers("fc")[0]
    A, G = [np.eye(65)], [np.eye(32)]
    A_manual, G_manual = np.eye(65), np.eye(32)
    for step in range(3):
        a, g, v = inputs.layer_inputs(layer, hp["cid"], step, 0, hp["relu"])
        assert a.dtype == np.float32 and a.min() >= 0 and g.std() == pytest.approx(1e-3, rel=0.1)
        A, G, XA, XG, P = oracle.kfac_step([layer], [a], [g], [v], A, G, hp["xi"], hp["gamma"])
        ab = np.concatenate([a.astype(np.float64), np.ones((32, 1))], 1)
        A_manual = 0.95 * A_manual + 0.05 * sum(np.outer(r, r) for r in ab) / 32
        G_manual = 0.95 * G_manual + 0.05 * sum(np.outer(r, r) for r in g.astype(np.float64)) / 32
        np.testing.assert_allclose(A[0], A_manual, rtol=1e-12, atol=1e-15)
        np.testing.assert_allclose(G[0], G_manual, rtol=1e-12, atol=1e-18)
        assert A[0][-1, -1] == pytest.approx(1.0, abs=1e-14)
        assert np.linalg.eigvalsh(A[0]).min() >= 0.95 ** (step + 1) - 1e-12
        for F, X in ((A[0], XA[0]), (G[0], XG[0])):
            d = F.shape[0]
            assert np.linalg.norm((F + 0.03 * np.eye(d)) @ X - np.eye(d)) / np.sqrt(d) < 1e-12
            assert np.linalg.eigvalsh(X).max() <= 1 / (0.95 ** (step + 1) + 0.03) + 1e-12
        np.testing.assert_allclose((G[0] + 0.03 * np.eye(32)) @ P[0] @ (A[0] + 0.03 * np.eye(65)), v, rtol=1e-9, atol=1e-12)
