"""Pins for the oracle's FIM and inverse-FIM-vector product (Sec. 2.1 cache stage, damping of App. B):
explicit loops, closed forms (diagonal, rank one / Sherman-Morrison, Woodbury), the eigen-decomposition
form and limits."""
import numpy as np
import pytest

from oracle import grass_oracle as orc


def _rows(n, k, seed):
    return np.random.default_rng(seed).standard_normal((n, k))


def test_fim_is_the_average_outer_product():
    G = _rows(7, 5, 0)
    F = orc.fim(G)
    want = np.zeros((5, 5))
    for i in range(7):
        for a in range(5):
            for b in range(5):
                want[a, b] += G[i, a] * G[i, b] / 7
    assert np.allclose(F, want, rtol=1e-13, atol=1e-15)
    assert np.array_equal(F, F.T)
    assert np.isclose(np.trace(F), np.mean(np.sum(G ** 2, axis=1)))
    assert np.linalg.eigvalsh(F).min() > -1e-12


def test_fim_has_rank_at_most_n():
    G = _rows(3, 9, 1)
    ev = np.linalg.eigvalsh(orc.fim(G))
    assert np.sum(ev > 1e-10) == 3


def test_ifvp_solves_the_damped_system():
    G = _rows(6, 8, 2)
    F = orc.fim(_rows(20, 8, 3))
    lam = 0.3
    X = orc.ifvp(G, F, lam)
    for i in range(6):
        for a in range(8):
            lhs = lam * X[i, a] + sum(F[a, b] * X[i, b] for b in range(8))
            assert np.isclose(lhs, G[i, a], rtol=1e-10, atol=1e-12)


def test_ifvp_diagonal_fim_is_an_elementwise_division():
    f = np.array([0.5, 2.0, 0.0, 7.0])
    G = _rows(3, 4, 4)
    assert np.allclose(orc.ifvp(G, np.diag(f), 0.25), G / (f + 0.25)[None, :], rtol=1e-13)


def test_ifvp_rank_one_fim_sherman_morrison():
    """F = u u^T: (lam I + u u^T)^{-1} g = (g - u <u, g> / (lam + |u|^2)) / lam."""
    u = _rows(1, 6, 5)
    F = orc.fim(u)                      # n = 1
    G = _rows(4, 6, 6)
    lam = 0.7
    want = (G - (G @ u.T) * u / (lam + float((u @ u.T)[0, 0]))) / lam
    assert np.allclose(orc.ifvp(G, F, lam), want, rtol=1e-12)
    # the FIM's own row: (lam I + u u^T)^{-1} u = u / (lam + |u|^2)
    assert np.allclose(orc.ifvp(u, F, lam), u / (lam + float((u @ u.T)[0, 0])), rtol=1e-12)


def test_ifvp_woodbury_when_fewer_rows_than_columns():
    """(lam I_k + A^T A / n)^{-1} = (I_k - A^T (n lam I_n + A A^T)^{-1} A) / lam: an n x n system instead of k x k."""
    n, k, lam = 4, 11, 0.05
    A = _rows(n, k, 7)
    G = _rows(5, k, 8)
    small = np.linalg.inv(n * lam * np.eye(n) + A @ A.T)
    want = (G - G @ A.T @ small @ A) / lam
    assert np.allclose(orc.ifvp(G, orc.fim(A), lam), want, rtol=1e-9)


def test_ifvp_eigen_form_and_limits():
    A = _rows(30, 7, 9)
    F = orc.fim(A)
    G = _rows(3, 7, 10)
    w, V = np.linalg.eigh(F)
    lam = 1e-2
    assert np.allclose(orc.ifvp(G, F, lam), (G @ V / (w + lam)) @ V.T, rtol=1e-10)
    big = 1e9
    assert np.allclose(orc.ifvp(G, F, big) * big, G, rtol=1e-6)                 # lam -> infinity: g / lam
    assert np.allclose(orc.ifvp(G, F, 0.0), G @ np.linalg.inv(F), rtol=1e-8)     # no damping: F^{-1} g


def test_influence_definition_and_symmetry():
    train, test = _rows(12, 5, 11), _rows(4, 5, 12)
    lam = 0.1
    I = orc.influence(train, test, lam)
    W = np.linalg.inv(orc.fim(train) + lam * np.eye(5))
    for m in range(4):
        for i in range(12):
            assert np.isclose(I[m, i], test[m] @ W @ train[i], rtol=1e-10)
    S = orc.influence(train, train, lam)
    assert np.allclose(S, S.T, rtol=1e-10, atol=1e-12)
    # self-influence through the hat-matrix identity: g_i^T (lam I + G^T G / n)^{-1} g_i  < n  for every row
    assert np.all(np.diag(S) < 12) and np.all(np.diag(S) > 0)
