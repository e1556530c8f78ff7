"""Pins for the oracle's Selective Mask objective, gradient and index extraction (Sec. 3.2 Eq. (1), App. B.4)."""
import numpy as np
import pytest
from scipy import stats

from oracle import grass_oracle as orc


def _problem(n=9, m=3, p=7, seed=0):
    rng = np.random.default_rng(seed)
    return rng.standard_normal(p), rng.standard_normal((n, p)), rng.standard_normal((m, p))


def test_objective_matches_scipy_pearson_written_out():
    S, G, Gt = _problem()
    lam = 0.03
    sig = 1 / (1 + np.exp(-S))
    want = 0.0
    for t in range(Gt.shape[0]):
        exact = [sum(G[i, j] * Gt[t, j] for j in range(7)) for i in range(9)]
        masked = [sum(sig[j] * G[i, j] * sig[j] * Gt[t, j] for j in range(7)) for i in range(9)]
        want += stats.pearsonr(exact, masked)[0]
    want = want / Gt.shape[0] - lam * sum(sig)
    assert np.isclose(orc.selective_mask_objective(S, G, Gt, lam), want, rtol=1e-12)


def test_constant_logits_give_perfect_correlation():
    """sigma constant: the masked scores are a positive multiple of the exact ones, corr = 1 for every test point."""
    _, G, Gt = _problem(seed=1)
    for s0 in (-2.0, 0.0, 3.0):
        S = np.full(7, s0)
        sig = 1 / (1 + np.exp(-s0))
        assert np.isclose(orc.selective_mask_objective(S, G, Gt, 0.1), 1.0 - 0.1 * 7 * sig, rtol=1e-12)


def test_objective_invariances():
    S, G, Gt = _problem(seed=2)
    base = orc.selective_mask_objective(S, G, Gt, 0.05)
    # correlation ignores positive rescaling of a test gradient and of all training gradients
    Gt2 = Gt * np.array([[2.0], [0.5], [7.0]])
    assert np.isclose(orc.selective_mask_objective(S, G, Gt2, 0.05), base, rtol=1e-12)
    assert np.isclose(orc.selective_mask_objective(S, 3.0 * G, Gt, 0.05), base, rtol=1e-12)
    # temperature: S / T with T = 2 equals logits S / 2 at T = 1
    assert np.isclose(orc.selective_mask_objective(S, G, Gt, 0.05, temperature=2.0),
                      orc.selective_mask_objective(S / 2.0, G, Gt, 0.05), rtol=1e-12)
    # a coordinate that is zero in every gradient only pays the penalty
    G0, Gt0 = np.hstack([G, np.zeros((9, 1))]), np.hstack([Gt, np.zeros((3, 1))])
    S0 = np.append(S, 1.3)
    assert np.isclose(orc.selective_mask_objective(S0, G0, Gt0, 0.05), base - 0.05 / (1 + np.exp(-1.3)), rtol=1e-12)


@pytest.mark.parametrize("temperature,lam,seed", [(1.0, 0.0, 3), (1.0, 0.07, 4), (0.5, 0.02, 5), (3.0, 0.3, 6)])
def test_gradient_matches_central_differences(temperature, lam, seed):
    S, G, Gt = _problem(n=11, m=4, p=9, seed=seed)
    g = orc.selective_mask_gradient(S, G, Gt, lam, temperature)
    h = 1e-6
    for j in range(S.size):
        e = np.zeros_like(S); e[j] = h
        fd = (orc.selective_mask_objective(S + e, G, Gt, lam, temperature)
              - orc.selective_mask_objective(S - e, G, Gt, lam, temperature)) / (2 * h)
        assert np.isclose(g[j], fd, rtol=2e-6, atol=1e-9)


def test_gradient_of_the_penalty_alone_at_perfect_correlation():
    """At constant logits the correlation term is flat along the all-ones direction (scale invariance):
    the directional derivative there is the penalty's alone."""
    _, G, Gt = _problem(seed=7)
    S = np.full(7, 0.4)
    sig = 1 / (1 + np.exp(-0.4))
    g = orc.selective_mask_gradient(S, G, Gt, 0.2)
    assert np.isclose(g.sum(), -0.2 * 7 * sig * (1 - sig), rtol=1e-9)


def test_gradient_ascent_increases_the_objective():
    S, G, Gt = _problem(n=20, m=5, p=12, seed=8)
    f0 = orc.selective_mask_objective(S, G, Gt, 0.01)
    S1 = S + 0.05 * orc.selective_mask_gradient(S, G, Gt, 0.01)
    assert orc.selective_mask_objective(S1, G, Gt, 0.01) > f0


def test_index_extraction():
    S = np.array([0.3, -0.1, 0.0, 2.0, -5.0, 0.3])
    assert orc.selective_mask_indices(S).tolist() == [0, 2, 3, 5]            # sigma(S) >= 1/2  <=>  S >= 0
    assert orc.selective_mask_indices(S, k=2).tolist() == [0, 3]             # 2.0, then the first of the two 0.3
    assert orc.selective_mask_indices(S, k=3).tolist() == [0, 3, 5]
    assert orc.selective_mask_indices(S, k=6).tolist() == [0, 1, 2, 3, 4, 5]
    assert orc.selective_mask_indices(S, k=1).dtype == np.int32
    # brute force
    rng = np.random.default_rng(9)
    S = rng.standard_normal(50)
    want = sorted(sorted(range(50), key=lambda j: (-S[j], j))[:13])
    assert orc.selective_mask_indices(S, k=13).tolist() == want


def _fact_problem(seed=0, n=8, m=3, d_in=5, d_out=4):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal(d_in), rng.standard_normal(d_out), rng.standard_normal((n, d_in)),
            rng.standard_normal((n, d_out)), rng.standard_normal((m, d_in)), rng.standard_normal((m, d_out)))


def test_factorized_objective_equals_the_plain_one_on_kronecker_gradients():
    """App. B.4: with g_i = z_in (x) z_out and mask sigma_in (x) sigma_out the correlation term is Eq. (1) itself."""
    S_in, S_out, Z_in, Z_out, Zt_in, Zt_out = _fact_problem(1)
    G = np.stack([np.kron(Z_in[i], Z_out[i]) for i in range(Z_in.shape[0])])
    Gt = np.stack([np.kron(Zt_in[t], Zt_out[t]) for t in range(Zt_in.shape[0])])
    sig = np.kron(1 / (1 + np.exp(-S_in)), 1 / (1 + np.exp(-S_out)))
    S_full = np.log(sig / (1 - sig))                         # logits whose sigmoid is the Kronecker mask
    plain = orc.selective_mask_objective(S_full, G, Gt, 0.0)
    obj, _, _ = orc.selective_mask_factorized(S_in, S_out, Z_in, Z_out, Zt_in, Zt_out, 0.0)
    assert np.isclose(obj, plain, rtol=1e-11)
    lam = 0.07
    pen = lam * ((1 / (1 + np.exp(-S_in))).sum() + (1 / (1 + np.exp(-S_out))).sum())
    assert np.isclose(orc.selective_mask_factorized(S_in, S_out, Z_in, Z_out, Zt_in, Zt_out, lam)[0], plain - pen, rtol=1e-11)


@pytest.mark.parametrize("temperature,lam,seed", [(1.0, 0.0, 2), (0.7, 0.05, 3), (2.0, 0.2, 4)])
def test_factorized_gradients_match_central_differences(temperature, lam, seed):
    S_in, S_out, Z_in, Z_out, Zt_in, Zt_out = _fact_problem(seed, n=10, m=4, d_in=6, d_out=5)
    _, gi, go = orc.selective_mask_factorized(S_in, S_out, Z_in, Z_out, Zt_in, Zt_out, lam, temperature)
    f = lambda a, b: orc.selective_mask_factorized(a, b, Z_in, Z_out, Zt_in, Zt_out, lam, temperature)[0]
    h = 1e-6
    for j in range(S_in.size):
        e = np.zeros_like(S_in); e[j] = h
        assert np.isclose(gi[j], (f(S_in + e, S_out) - f(S_in - e, S_out)) / (2 * h), rtol=2e-6, atol=1e-9)
    for j in range(S_out.size):
        e = np.zeros_like(S_out); e[j] = h
        assert np.isclose(go[j], (f(S_in, S_out + e) - f(S_in, S_out - e)) / (2 * h), rtol=2e-6, atol=1e-9)


# ------------------------------------------------------------------ factorised form on sequences of tokens
def _seq_problem(n=7, m=3, T=4, Tt=3, d_in=5, d_out=4, seed=0):
    rng = np.random.default_rng(seed)
    return (0.4 * rng.standard_normal(d_in), 0.4 * rng.standard_normal(d_out), rng.standard_normal((n, T, d_in)),
            rng.standard_normal((n, T, d_out)), rng.standard_normal((m, Tt, d_in)), rng.standard_normal((m, Tt, d_out)))


def _layer_gradients(X_in, X_out):
    """Materialised per-sample layer gradients sum_t x_t (x) g_t (Eq. (2)), flattened input index major."""
    return np.einsum("nta,ntb->nab", X_in, X_out).reshape(X_in.shape[0], -1)


def test_sequence_graddot_equals_inner_products_of_materialised_layer_gradients():
    _, _, X_in, X_out, Xt_in, Xt_out = _seq_problem(seed=1)
    G, Gt = _layer_gradients(X_in, X_out), _layer_gradients(Xt_in, Xt_out)
    assert np.allclose(orc.graddot_factorized_seq(X_in, X_out, Xt_in, Xt_out), Gt @ G.T, rtol=1e-12, atol=1e-12)


def test_sequence_factorized_objective_equals_the_plain_one_on_materialised_gradients():
    """With logits whose sigmoid is sigma(S_in) (x) sigma(S_out), the plain objective of Eq. (1) on the materialised
    layer gradients is the factorised one (no penalty: the two forms penalise different sums)."""
    S_in, S_out, X_in, X_out, Xt_in, Xt_out = _seq_problem(seed=2)
    for T in (1.0, 0.6):
        sig = np.kron(1 / (1 + np.exp(-S_in / T)), 1 / (1 + np.exp(-S_out / T)))
        S_flat = T * np.log(sig / (1 - sig))
        plain = orc.selective_mask_objective(S_flat, _layer_gradients(X_in, X_out), _layer_gradients(Xt_in, Xt_out), 0.0, T)
        obj, _, _ = orc.selective_mask_factorized_seq(S_in, S_out, X_in, X_out, Xt_in, Xt_out, 0.0, T)
        assert np.isclose(obj, plain, rtol=1e-10)
    lam = 0.07
    pen = lam * ((1 / (1 + np.exp(-S_in))).sum() + (1 / (1 + np.exp(-S_out))).sum())
    assert np.isclose(orc.selective_mask_factorized_seq(S_in, S_out, X_in, X_out, Xt_in, Xt_out, lam)[0],
                      orc.selective_mask_factorized_seq(S_in, S_out, X_in, X_out, Xt_in, Xt_out, 0.0)[0] - pen, rtol=1e-12)


@pytest.mark.parametrize("temperature,lam,seed", [(1.0, 0.0, 3), (0.7, 0.05, 4)])
def test_sequence_factorized_gradients_match_central_differences(temperature, lam, seed):
    S_in, S_out, X_in, X_out, Xt_in, Xt_out = _seq_problem(seed=seed)
    _, gi, go = orc.selective_mask_factorized_seq(S_in, S_out, X_in, X_out, Xt_in, Xt_out, lam, temperature)
    f = lambda a, b: orc.selective_mask_factorized_seq(a, b, X_in, X_out, Xt_in, Xt_out, lam, temperature)[0]
    h = 1e-6
    for j in range(S_in.size):
        e = np.zeros_like(S_in); e[j] = h
        assert np.isclose(gi[j], (f(S_in + e, S_out) - f(S_in - e, S_out)) / (2 * h), rtol=1e-5, atol=1e-9)
    for j in range(S_out.size):
        e = np.zeros_like(S_out); e[j] = h
        assert np.isclose(go[j], (f(S_in, S_out + e) - f(S_in, S_out - e)) / (2 * h), rtol=1e-5, atol=1e-9)


def test_sequence_form_with_one_token_is_the_single_token_form():
    S_in, S_out, X_in, X_out, Xt_in, Xt_out = _seq_problem(T=1, Tt=1, seed=5)
    a = orc.selective_mask_factorized_seq(S_in, S_out, X_in, X_out, Xt_in, Xt_out, 0.03, 0.8)
    b = orc.selective_mask_factorized(S_in, S_out, X_in[:, 0], X_out[:, 0], Xt_in[:, 0], Xt_out[:, 0], 0.03, 0.8)
    assert np.isclose(a[0], b[0], rtol=1e-12) and np.allclose(a[1], b[1], rtol=1e-11, atol=1e-14)
    assert np.allclose(a[2], b[2], rtol=1e-11, atol=1e-14)


def test_sequence_form_ignores_token_order_and_all_zero_tokens():
    """The layer gradient is a sum over tokens: permuting the tokens of a sample (both factors alike) or appending a
    token whose factors are zero changes nothing."""
    S_in, S_out, X_in, X_out, Xt_in, Xt_out = _seq_problem(seed=6)
    base = orc.selective_mask_factorized_seq(S_in, S_out, X_in, X_out, Xt_in, Xt_out, 0.02, 1.0)
    perm = np.array([2, 0, 3, 1])
    X_in2, X_out2 = X_in.copy(), X_out.copy()
    X_in2[1], X_out2[1] = X_in[1][perm], X_out[1][perm]
    pad = lambda a: np.concatenate([a, np.zeros_like(a[:, :1])], axis=1)
    other = orc.selective_mask_factorized_seq(S_in, S_out, pad(X_in2), pad(X_out2), pad(Xt_in), pad(Xt_out), 0.02, 1.0)
    assert np.isclose(base[0], other[0], rtol=1e-12)
    assert np.allclose(base[1], other[1], rtol=1e-10, atol=1e-14) and np.allclose(base[2], other[2], rtol=1e-10, atol=1e-14)
    # permuting the tokens of one factor only is a different gradient
    X_in3 = X_in.copy(); X_in3[1] = X_in[1][perm]
    assert not np.isclose(orc.selective_mask_factorized_seq(S_in, S_out, X_in3, X_out, Xt_in, Xt_out, 0.02, 1.0)[0], base[0])
