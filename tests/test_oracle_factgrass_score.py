"""Pins for the oracle's FactGraSS, score and dense-projection baseline (CPU only).

Eq. (2): vec(DW) = sum_t x_t (x) g_t for the layer gradient DW = sum_t g_t x_t^T
(d_out x d_in).  Eq. (3): a Kronecker-factorised map applied to vec(DW) equals
the token sum of Kronecker products of the separately mapped factors; with
selection matrices as the factors this is FactGraSS's stages 1 and 2
(Sec. 3.3.2).  App. B.4.2: <a (x) b, c (x) d> = <a, c><b, d>.
"""
import numpy as np
import pytest

from oracle import grass_oracle as orc


def _factors(rng, n, T, d_in, d_out):
    return rng.standard_normal((n, T, d_in)), rng.standard_normal((n, T, d_out))


def test_layer_streams():
    assert orc.layer_streams(0) == (16, 17, 18)
    assert orc.layer_streams(3) == (28, 29, 30)


def test_factgrass_equals_materialise_mask_sjlt():
    """Form the full layer gradient, vectorise it column-major (Eq. (2)), keep
    the Kronecker index set, SJLT with the same stream: identical."""
    rng = np.random.default_rng(0)
    n, T, d_in, d_out, ka, kb, k, s = 3, 7, 12, 9, 5, 4, 8, 2
    x, g = _factors(rng, n, T, d_in, d_out)
    idx_in = orc.mask_indices(1, 16, d_in, ka)
    idx_out = orc.mask_indices(1, 17, d_out, kb)
    got = orc.factgrass_linear(x, g, idx_in, idx_out, k, s, seed=1, stream=18)
    for i in range(n):
        DW = np.zeros((d_out, d_in))
        for t in range(T):
            DW += np.outer(g[i, t], x[i, t])               # dl/dW = (dl/dz_out) z_in^T
        vec = DW.flatten(order="F")                         # column-major: index a*d_out + b
        keep = np.array([a * d_out + b for a in idx_in for b in idx_out])
        assert np.all(np.diff(keep) > 0)
        want = orc.sjlt(vec[keep], k, s, seed=1, stream=18)
        assert np.allclose(got[i], want, rtol=0, atol=1e-12)


def test_vec_identity_of_eq2():
    rng = np.random.default_rng(1)
    T, d_in, d_out = 5, 6, 4
    x, g = _factors(rng, 1, T, d_in, d_out)
    full = orc.factgrass_sparsified_gradient(x, g, np.arange(d_in), np.arange(d_out))[0]
    DW = sum(np.outer(g[0, t], x[0, t]) for t in range(T))
    assert np.allclose(full, DW.flatten(order="F"), rtol=0, atol=1e-13)
    assert np.allclose(full.reshape(d_in, d_out), DW.T, rtol=0, atol=1e-13)


def test_factored_selection_equals_kronecker_of_selection_matrices():
    """Eq. (3) with P_in, P_out binary selection matrices."""
    rng = np.random.default_rng(2)
    T, d_in, d_out, ka, kb = 4, 7, 6, 3, 2
    x, g = _factors(rng, 1, T, d_in, d_out)
    idx_in = orc.mask_indices(0, 16, d_in, ka)
    idx_out = orc.mask_indices(0, 17, d_out, kb)
    Min = np.zeros((ka, d_in)); Min[np.arange(ka), idx_in] = 1
    Mout = np.zeros((kb, d_out)); Mout[np.arange(kb), idx_out] = 1
    vec = sum(np.kron(x[0, t], g[0, t]) for t in range(T))
    want = np.kron(Min, Mout) @ vec
    got = orc.factgrass_sparsified_gradient(x, g, idx_in, idx_out)[0]
    assert np.allclose(got, want, rtol=0, atol=1e-13)


def test_single_token_is_outer_product():
    rng = np.random.default_rng(3)
    x, g = _factors(rng, 2, 1, 10, 8)
    idx_in = np.array([1, 4, 9]); idx_out = np.array([0, 7])
    v = orc.factgrass_sparsified_gradient(x, g, idx_in, idx_out)
    for i in range(2):
        assert np.array_equal(v[i].reshape(3, 2), np.outer(x[i, 0, idx_in], g[i, 0, idx_out]))


def test_full_masks_reduce_to_sjlt_of_layer_gradient():
    rng = np.random.default_rng(4)
    T, d_in, d_out, k = 6, 8, 5, 10
    x, g = _factors(rng, 1, T, d_in, d_out)
    got = orc.factgrass_linear(x, g, np.arange(d_in), np.arange(d_out), k, 1, seed=0, stream=18)[0]
    DW = sum(np.outer(g[0, t], x[0, t]) for t in range(T))
    want = orc.sjlt(DW.flatten(order="F"), k, 1, seed=0, stream=18)
    assert np.allclose(got, want, rtol=0, atol=1e-12)


def test_bilinear_in_the_factors():
    rng = np.random.default_rng(5)
    n, T, d_in, d_out = 1, 5, 9, 7
    x1, g1 = _factors(rng, n, T, d_in, d_out)
    x2, g2 = _factors(rng, n, T, d_in, d_out)
    ii, io = np.array([0, 3, 8]), np.array([1, 2, 6])
    f = lambda x, g: orc.factgrass_linear(x, g, ii, io, 6, 2, seed=3, stream=22)
    assert np.allclose(f(2 * x1 - x2, g1), 2 * f(x1, g1) - f(x2, g1), rtol=0, atol=1e-12)
    assert np.allclose(f(x1, g1 + 3 * g2), f(x1, g1) + 3 * f(x1, g2), rtol=0, atol=1e-12)


def test_kronecker_inner_product_identity():
    rng = np.random.default_rng(6)
    x1, g1 = _factors(rng, 1, 1, 11, 6)
    x2, g2 = _factors(rng, 1, 1, 11, 6)
    ii, io = np.array([2, 5, 10]), np.array([0, 3, 4, 5])
    v1 = orc.factgrass_sparsified_gradient(x1, g1, ii, io)[0]
    v2 = orc.factgrass_sparsified_gradient(x2, g2, ii, io)[0]
    want = (x1[0, 0, ii] @ x2[0, 0, ii]) * (g1[0, 0, io] @ g2[0, 0, io])
    assert np.isclose(v1 @ v2, want, rtol=1e-12)


def test_swapping_factors_changes_the_order():
    """Guards the flat order a'*k_out' + b' (x index major)."""
    x = np.zeros((1, 1, 4)); g = np.zeros((1, 1, 3))
    x[0, 0, 2] = 1.0; g[0, 0, 1] = 1.0
    v = orc.factgrass_sparsified_gradient(x, g, np.arange(4), np.arange(3))[0]
    assert np.flatnonzero(v).tolist() == [2 * 3 + 1]


# ------------------------------------------------------------------- LoGra
def test_logra_equals_kronecker_projection_of_the_layer_gradient():
    """Eq. (3): (P_in (x) P_out) vec(DW) with vec(DW) = sum_t x_t (x) g_t (column-major vec of g x^T)."""
    rng = np.random.default_rng(20)
    n, T, d_in, d_out, ki, ko = 2, 5, 7, 6, 3, 4
    x, g = _factors(rng, n, T, d_in, d_out)
    Pi = rng.standard_normal((ki, d_in)); Po = rng.standard_normal((ko, d_out))
    got = orc.logra_linear(x, g, Pi, Po)
    for i in range(n):
        DW = sum(np.outer(g[i, t], x[i, t]) for t in range(T))
        want = np.kron(Pi, Po) @ DW.flatten(order="F")
        assert np.allclose(got[i], want, rtol=0, atol=1e-11)


def test_logra_with_selection_matrices_is_factorised_masking():
    """Swapping the Gaussian factors for selection matrices gives Mask_{k_in (x) k_out},
    i.e. FactGraSS's stages 1 and 2 (Sec. 3.3.2, 'Bottlenecks of integrating GraSS with LoGra')."""
    rng = np.random.default_rng(21)
    x, g = _factors(rng, 2, 4, 9, 8)
    ii, io = np.array([1, 5, 8]), np.array([0, 2, 3, 7])
    Mi = np.zeros((3, 9)); Mi[np.arange(3), ii] = 1
    Mo = np.zeros((4, 8)); Mo[np.arange(4), io] = 1
    assert np.allclose(orc.logra_linear(x, g, Mi, Mo), orc.factgrass_sparsified_gradient(x, g, ii, io),
                       rtol=0, atol=1e-13)


def test_logra_is_bilinear_and_token_additive():
    rng = np.random.default_rng(22)
    x, g = _factors(rng, 1, 6, 5, 4)
    Pi = rng.standard_normal((2, 5)); Po = rng.standard_normal((3, 4))
    whole = orc.logra_linear(x, g, Pi, Po)
    parts = orc.logra_linear(x[:, :2], g[:, :2], Pi, Po) + orc.logra_linear(x[:, 2:], g[:, 2:], Pi, Po)
    assert np.allclose(whole, parts, rtol=0, atol=1e-12)
    assert np.allclose(orc.logra_linear(3 * x, g, Pi, Po), 3 * whole, rtol=0, atol=1e-12)


# ------------------------------------------------------------------- score
def test_score_definition_and_symmetry():
    rng = np.random.default_rng(7)
    train = rng.standard_normal((9, 13)); test = rng.standard_normal((4, 13))
    sc = orc.score(train, test)
    assert sc.shape == (4, 9)
    for m in range(4):
        for i in range(9):
            assert np.isclose(sc[m, i], sum(test[m, c] * train[i, c] for c in range(13)), rtol=1e-12)
    self_sc = orc.score(train, train)
    assert np.allclose(self_sc, self_sc.T, rtol=0, atol=1e-13)
    assert np.allclose(np.diag(self_sc), (train ** 2).sum(axis=1))


def test_score_of_compressed_gradients_estimates_graddot():
    rng = np.random.default_rng(8)
    d, k, trials = 64, 16, 2000
    u, v = rng.standard_normal((2, d))
    vals = []
    for seed in range(trials):
        c = orc.sjlt(np.stack([u, v]), k, 1, seed)
        vals.append(orc.score(c[:1], c[1:])[0, 0])
    vals = np.array(vals)
    assert abs(vals.mean() - u @ v) < 4.5 * vals.std() / np.sqrt(trials)


def test_gauss_project_definition():
    rng = np.random.default_rng(9)
    g = rng.standard_normal((3, 20)); P = rng.standard_normal((5, 20)) / np.sqrt(5)
    out = orc.gauss_project(g, P)
    for i in range(3):
        for a in range(5):
            assert np.isclose(out[i, a], sum(P[a, j] * g[i, j] for j in range(20)), rtol=1e-12)


def test_gauss_matrix_is_standard_normal_scaled():
    """Sec. 2.2: P_ab ~ N(0, 1/k) i.i.d.  Checked against scipy's normal CDF and the closed-form moments."""
    from scipy import stats
    p, k = 4000, 50
    P = orc.gauss_matrix(5, 2, p, k)
    z = P.ravel() * np.sqrt(k)
    nz = z.size
    assert stats.kstest(z, "norm").pvalue > 1e-3
    assert abs(z.mean()) < 4 / np.sqrt(nz)
    assert abs(z.var() - 1) < 4 * np.sqrt(2 / nz)
    assert abs((z ** 3).mean()) < 4 * np.sqrt(15 / nz)
    assert abs((z ** 4).mean() - 3) < 4 * np.sqrt(96 / nz)
    # independence along both axes and between the two uniform fields
    assert abs(np.corrcoef(P[:, :-1].ravel(), P[:, 1:].ravel())[0, 1]) < 4 / np.sqrt(nz)
    assert abs(np.corrcoef(P[:-1].ravel(), P[1:].ravel())[0, 1]) < 4 / np.sqrt(nz)
    assert abs(np.corrcoef(np.abs(P[:, :-1]).ravel(), np.abs(P[:, 1:]).ravel())[0, 1]) < 4 / np.sqrt(nz)


def test_gauss_matrix_windows_seeds_and_streams():
    p, k = 300, 7
    P = orc.gauss_matrix(1, 2, p, k)
    assert np.array_equal(orc.gauss_matrix(1, 2, p, k, 100, 50), P[:, 100:150])    # a window is a slice
    assert np.array_equal(orc.gauss_matrix(1, 2, p, k, rows=[6, 0]), P[[6, 0]])
    assert not np.allclose(orc.gauss_matrix(2, 2, p, k), P)
    assert not np.allclose(orc.gauss_matrix(1, 3, p, k), P)
    # entry (a, b) depends on the flat index a*p + b: with p' = 2p row a of the narrow matrix is not row a of the wide
    assert not np.allclose(orc.gauss_matrix(1, 2, 2 * p, k)[1:, :p], P[1:])
    assert np.array_equal(orc.gauss_matrix(1, 2, 2 * p, k)[0, :p], P[0] )


def test_gauss_projection_preserves_norms_in_expectation():
    """Sec. 2.2 (Johnson-Lindenstrauss): E||P g||^2 = ||g||^2 and Var = 2||g||^4/k for Gaussian P."""
    rng = np.random.default_rng(3)
    p, k, trials = 60, 16, 1500
    g = rng.standard_normal((1, p))
    vals = np.array([np.sum(orc.gauss_project(g, orc.gauss_matrix(seed, 2, p, k)) ** 2) for seed in range(trials)])
    n2 = float(np.sum(g ** 2))
    assert abs(vals.mean() - n2) < 4.5 * np.sqrt(2 * n2 ** 2 / k / trials)
    assert abs(vals.var() / (2 * n2 ** 2 / k) - 1) < 0.25


def test_projection_matrix_is_the_compressor():
    """Sec. 3.1 / 3.3.1: the dense matrix applied to g equals the scan; s non-zeros per kept column, none elsewhere."""
    rng = np.random.default_rng(21)
    p, k, s = 90, 12, 3
    g = rng.standard_normal((4, p))
    P = orc.projection_matrix(6, 1, p, k, s)
    assert np.allclose(g @ P.T, orc.sjlt(g, k, s, 6, 1), rtol=1e-12, atol=1e-14)
    assert np.all((P != 0).sum(axis=0) == s) and np.allclose(np.abs(P[P != 0]), 1 / np.sqrt(s))
    idx = orc.mask_indices(6, 0, p, 20)
    Pm = orc.projection_matrix(6, 1, p, k, s, idx)
    assert np.allclose(g @ Pm.T, orc.grass(g, idx, k, s, 6, 1), rtol=1e-12, atol=1e-14)
    kept = np.zeros(p, bool); kept[idx] = True
    assert np.all((Pm != 0).sum(axis=0)[kept] == s) and not Pm[:, ~kept].any()


def test_factorised_sjlt_baseline_is_per_token_sjlt_then_kronecker():
    """SJLT_{k_in x k_out} of Sec. 3.3.2 = Eq. (3) with SJLT matrices: sum_t SJLT(x_t) (x) SJLT(g_t)."""
    rng = np.random.default_rng(22)
    n, T, d_in, d_out, k_in, k_out = 2, 5, 30, 24, 4, 6
    x, g = rng.standard_normal((n, T, d_in)), rng.standard_normal((n, T, d_out))
    P_in, P_out = orc.projection_matrix(3, 40, d_in, k_in, 1), orc.projection_matrix(3, 41, d_out, k_out, 1)
    got = orc.logra_linear(x, g, P_in, P_out)
    for i in range(n):
        want = sum(np.kron(orc.sjlt(x[i, t:t + 1], k_in, 1, 3, 40)[0], orc.sjlt(g[i, t:t + 1], k_out, 1, 3, 41)[0])
                   for t in range(T))
        assert np.allclose(got[i], want, rtol=1e-12, atol=1e-14)


def test_factorised_mask_baseline_is_logra_with_selection_matrices():
    """Mask_{k_in x k_out} = Eq. (3) with binary selection matrices = the sparsified gradient of FactGraSS."""
    rng = np.random.default_rng(23)
    n, T, d_in, d_out = 2, 4, 20, 16
    x, g = rng.standard_normal((n, T, d_in)), rng.standard_normal((n, T, d_out))
    ii, io = orc.mask_indices(1, 16, d_in, 5), orc.mask_indices(1, 17, d_out, 3)
    M_in = np.zeros((5, d_in)); M_in[np.arange(5), ii] = 1
    M_out = np.zeros((3, d_out)); M_out[np.arange(3), io] = 1
    assert np.allclose(orc.factgrass_sparsified_gradient(x, g, ii, io), orc.logra_linear(x, g, M_in, M_out), rtol=1e-13)
