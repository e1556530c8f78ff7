"""Pins for the oracle's training loop of the factorised Selective Mask (App. B.4 "Linear Layer": masks
sigma(S_in) (x) sigma(S_out) on gradients z_in (x) z_out).  The factorised objective and its derivatives are pinned in
test_oracle_selective_mask.py (against the plain objective on materialised Kronecker gradients and against central
differences); the plain training loop in test_oracle_selective_mask_train.py.  Here: what the two-vector loop must do."""
import numpy as np

import synth
from oracle import grass_oracle as orc


def _problem(n=12, m=4, d_in=6, d_out=5, seed=0):
    rng = np.random.default_rng(seed)
    return (0.3 * rng.standard_normal(d_in), 0.3 * rng.standard_normal(d_out), rng.standard_normal((n, d_in)),
            rng.standard_normal((n, d_out)), rng.standard_normal((m, d_in)), rng.standard_normal((m, d_out)))


def _objective(S_in, S_out, Z, lam, T):
    return orc.selective_mask_factorized(S_in, S_out, *Z, lam, T)[0]


def test_no_steps_and_zero_step_size_leave_the_logits_alone():
    S_in, S_out, *Z = _problem()
    a, b, hist = orc.selective_mask_train_factorized(S_in, S_out, *Z, 0.01, 0.5, [])
    assert np.array_equal(a, S_in) and np.array_equal(b, S_out) and hist.size == 0 and a is not S_in and b is not S_out
    a, b, hist = orc.selective_mask_train_factorized(S_in, S_out, *Z, 0.01, 0.0, [1.0, 0.5])
    assert np.array_equal(a, S_in) and np.array_equal(b, S_out)
    assert hist[0] == _objective(S_in, S_out, Z, 0.01, 1.0) and hist[1] == _objective(S_in, S_out, Z, 0.01, 0.5)


def test_first_step_moves_both_vectors_along_the_finite_difference_gradient():
    S_in, S_out, *Z = _problem(seed=1)
    lam, lr, T, h = 0.02, 0.7, 0.8, 1e-6
    a, b, hist = orc.selective_mask_train_factorized(S_in, S_out, *Z, lam, lr, [T])
    fd_in, fd_out = np.empty_like(S_in), np.empty_like(S_out)
    for j in range(S_in.size):
        e = np.zeros_like(S_in); e[j] = h
        fd_in[j] = (_objective(S_in + e, S_out, Z, lam, T) - _objective(S_in - e, S_out, Z, lam, T)) / (2 * h)
    for j in range(S_out.size):
        e = np.zeros_like(S_out); e[j] = h
        fd_out[j] = (_objective(S_in, S_out + e, Z, lam, T) - _objective(S_in, S_out - e, Z, lam, T)) / (2 * h)
    assert np.allclose(a - S_in, lr * fd_in, rtol=1e-5, atol=1e-9)
    assert np.allclose(b - S_out, lr * fd_out, rtol=1e-5, atol=1e-9)
    assert hist.shape == (1,) and hist[0] == _objective(S_in, S_out, Z, lam, T)


def test_a_trivial_output_factor_reduces_it_to_the_plain_training_loop():
    """d_out = 1 with z_out = 1 everywhere and a saturated output logit (sigma = 1, zero slope): gradients are z_in,
    the mask is sigma(S_in), and the input logits must follow the plain loop on G = Z_in step for step; the history
    differs by the constant penalty lam * 1 of the output coordinate."""
    rng = np.random.default_rng(2)
    n, m, d = 14, 3, 8
    Z_in, Zt_in = rng.standard_normal((n, d)), rng.standard_normal((m, d))
    ones_n, ones_m = np.ones((n, 1)), np.ones((m, 1))
    S0 = 0.3 * rng.standard_normal(d)
    temps = [1.0, 0.9, 0.8, 0.7]
    lam, lr = 0.02, 0.6
    a, b, hist = orc.selective_mask_train_factorized(S0, [60.0], Z_in, ones_n, Zt_in, ones_m, lam, lr, temps)
    want, want_hist = orc.selective_mask_train(S0, Z_in, Zt_in, lam, lr, temps)
    assert np.allclose(a, want, rtol=1e-12, atol=1e-14)
    assert np.allclose(hist, want_hist - lam, rtol=1e-12, atol=1e-14)
    assert abs(b[0] - 60.0) < 1e-12                                    # the saturated logit does not move


def test_swapping_the_two_factors_swaps_the_two_results():
    """<a (x) b, c (x) d> = <a, c> <b, d> is symmetric in the factors, so is the penalty: training with the roles of
    the input and output factors exchanged gives the exchanged logits and the same history."""
    S_in, S_out, Z_in, Z_out, Zt_in, Zt_out = _problem(seed=3)
    temps = [1.0, 0.8, 0.6]
    a, b, hist = orc.selective_mask_train_factorized(S_in, S_out, Z_in, Z_out, Zt_in, Zt_out, 0.03, 0.5, temps)
    b2, a2, hist2 = orc.selective_mask_train_factorized(S_out, S_in, Z_out, Z_in, Zt_out, Zt_in, 0.03, 0.5, temps)
    assert np.allclose(a, a2, rtol=1e-12, atol=1e-14) and np.allclose(b, b2, rtol=1e-12, atol=1e-14)
    assert np.allclose(hist, hist2, rtol=1e-12, atol=1e-14)
    assert not np.allclose(a, S_in) and not np.allclose(b, S_out)      # both vectors did move


def test_dead_coordinates_of_either_factor_follow_the_penalty_in_closed_form():
    S_in, S_out, Z_in, Z_out, Zt_in, Zt_out = _problem(seed=4)
    Z_in[:, 2] = 0.0; Zt_in[:, 2] = 0.0
    Z_out[:, 4] = 0.0; Zt_out[:, 4] = 0.0
    lam, lr, T = 0.2, 1.5, 0.5
    a, b, _ = orc.selective_mask_train_factorized(S_in, S_out, Z_in, Z_out, Zt_in, Zt_out, lam, lr, [T])
    for got, s in ((a[2], S_in[2]), (b[4], S_out[4])):
        sig = 1.0 / (1.0 + np.exp(-s / T))
        assert np.isclose(got, s - lr * lam * sig * (1.0 - sig) / T, rtol=1e-12)


def test_training_is_a_composition_of_its_steps_each_at_its_own_temperature():
    S_in, S_out, *Z = _problem(seed=5)
    temps = [2.0, 0.25, 1.0]
    a, b, hist = orc.selective_mask_train_factorized(S_in, S_out, *Z, 0.03, 0.4, temps)
    a1, b1, h1 = orc.selective_mask_train_factorized(S_in, S_out, *Z, 0.03, 0.4, temps[:1])
    a2, b2, h2 = orc.selective_mask_train_factorized(a1, b1, *Z, 0.03, 0.4, temps[1:])
    assert np.array_equal(a, a2) and np.array_equal(b, b2) and np.array_equal(hist, np.concatenate([h1, h2]))
    sa, sb, _ = orc.selective_mask_train_factorized(S_in, S_out, *Z, 0.03, 0.4, temps[::-1])
    assert not np.allclose(sa, a) and not np.allclose(sb, b)


def test_small_steps_never_decrease_the_objective():
    S_in, S_out, *Z = _problem(n=20, m=5, d_in=7, d_out=6, seed=6)
    a, b, hist = orc.selective_mask_train_factorized(S_in, S_out, *Z, 0.01, 0.05, [1.0] * 60)
    final = _objective(a, b, Z, 0.01, 1.0)
    assert np.all(np.diff(hist) >= 0.0) and final >= hist[-1] and final > hist[0] + 1e-4


def test_trained_factor_masks_find_the_planted_coordinates_of_both_factors():
    """Both factors carry a few planted coordinates that dominate the inner products; training raises exactly those
    logits in both vectors, and the Kronecker mask built from the extracted indices preserves the layer's GradDot
    scores better than random factor masks of the same sizes (Sec. 3.2; App. B.4)."""
    n, m, d_in, d_out, k_in, k_out = 64, 8, 40, 30, 6, 5
    Z_in, Zt_in, p_in = (t.numpy() for t in synth.planted_gradients(n, m, d_in, k_in, seed=11))
    Z_out, Zt_out, p_out = (t.numpy() for t in synth.planted_gradients(n, m, d_out, k_out, seed=12))
    rng = np.random.default_rng(0)
    S_in0, S_out0 = 0.1 * rng.standard_normal(d_in), 0.1 * rng.standard_normal(d_out)
    temps = np.geomspace(1.0, 0.3, 150)
    a, b, hist = orc.selective_mask_train_factorized(S_in0, S_out0, Z_in, Z_out, Zt_in, Zt_out, 3e-3, 5.0, temps)
    assert np.array_equal(orc.selective_mask_indices(a, k_in), p_in.astype(np.int32))
    assert np.array_equal(orc.selective_mask_indices(b, k_out), p_out.astype(np.int32))
    assert a[p_in].min() > np.delete(a, p_in).max() + 1.0 and b[p_out].min() > np.delete(b, p_out).max() + 1.0
    assert hist[-1] > hist[0]

    def corr(ii, io):           # GradDot correlation of the layer gradients z_in (x) z_out under the mask ii (x) io
        G = np.einsum("na,nb->nab", Z_in, Z_out).reshape(n, -1)
        Gt = np.einsum("na,nb->nab", Zt_in, Zt_out).reshape(m, -1)
        flat = (np.asarray(ii)[:, None] * d_out + np.asarray(io)[None, :]).ravel()
        return orc.graddot_correlation(G, Gt, flat)
    c_sel = corr(orc.selective_mask_indices(a, k_in), orc.selective_mask_indices(b, k_out))
    c_rand = np.mean([corr(orc.mask_indices(sd, 0, d_in, k_in), orc.mask_indices(sd, 1, d_out, k_out)) for sd in range(20)])
    assert c_sel > 0.9 and c_sel > c_rand + 0.2


# ------------------------------------------------------------------ the same loop on sequences of tokens
def _seq_problem(n=7, m=3, T=4, Tt=3, d_in=5, d_out=4, seed=0):
    rng = np.random.default_rng(seed)
    return (0.4 * rng.standard_normal(d_in), 0.4 * rng.standard_normal(d_out), rng.standard_normal((n, T, d_in)),
            rng.standard_normal((n, T, d_out)), rng.standard_normal((m, Tt, d_in)), rng.standard_normal((m, Tt, d_out)))


def _seq_objective(S_in, S_out, X, lam, T):
    return orc.selective_mask_factorized_seq(S_in, S_out, *X, lam, T)[0]


def test_sequence_training_with_one_token_is_the_single_token_loop():
    S_in, S_out, *X = _seq_problem(T=1, Tt=1, seed=20)
    temps = [1.0, 0.7, 0.5]
    a, b, hist = orc.selective_mask_train_factorized_seq(S_in, S_out, *X, 0.02, 0.6, temps)
    a1, b1, hist1 = orc.selective_mask_train_factorized(S_in, S_out, *(x[:, 0] for x in X), 0.02, 0.6, temps)
    assert np.allclose(a, a1, rtol=1e-12, atol=1e-14) and np.allclose(b, b1, rtol=1e-12, atol=1e-14)
    assert np.allclose(hist, hist1, rtol=1e-12, atol=1e-14)


def test_sequence_training_first_step_follows_the_finite_difference_gradient_of_the_sequence_objective():
    S_in, S_out, *X = _seq_problem(seed=21)
    lam, lr, T, h = 0.02, 0.7, 0.8, 1e-6
    a, b, hist = orc.selective_mask_train_factorized_seq(S_in, S_out, *X, lam, lr, [T])
    for got, S, which in ((a, S_in, 0), (b, S_out, 1)):
        fd = np.empty_like(S)
        for j in range(S.size):
            e = np.zeros_like(S); e[j] = h
            plus = _seq_objective(S_in + e, S_out, X, lam, T) if which == 0 else _seq_objective(S_in, S_out + e, X, lam, T)
            minus = _seq_objective(S_in - e, S_out, X, lam, T) if which == 0 else _seq_objective(S_in, S_out - e, X, lam, T)
            fd[j] = (plus - minus) / (2 * h)
        assert np.allclose(got - S, lr * fd, rtol=1e-5, atol=1e-9)
    assert hist.shape == (1,) and hist[0] == _seq_objective(S_in, S_out, X, lam, T)


def test_sequence_training_with_a_trivial_output_factor_is_the_plain_loop_on_token_sums():
    """Output factor of width one, equal to 1 on every token, logit saturated: the layer gradient of a sample is the
    sum of its input tokens (Eq. (2)), the mask is sigma(S_in), so the input logits must follow the plain loop on the
    token sums; the history differs by the penalty lam * 1 of the output coordinate."""
    rng = np.random.default_rng(22)
    n, m, T, Tt, d = 10, 3, 4, 2, 6
    X_in, Xt_in = rng.standard_normal((n, T, d)), rng.standard_normal((m, Tt, d))
    S0 = 0.3 * rng.standard_normal(d)
    temps, lam, lr = [1.0, 0.9, 0.8], 0.02, 0.6
    a, b, hist = orc.selective_mask_train_factorized_seq(S0, [60.0], X_in, np.ones((n, T, 1)), Xt_in, np.ones((m, Tt, 1)),
                                                         lam, lr, temps)
    want, want_hist = orc.selective_mask_train(S0, X_in.sum(1), Xt_in.sum(1), lam, lr, temps)
    assert np.allclose(a, want, rtol=1e-11, atol=1e-13) and np.allclose(hist, want_hist - lam, rtol=1e-11, atol=1e-13)
    assert abs(b[0] - 60.0) < 1e-12


def test_sequence_training_is_a_composition_of_its_steps_and_moves_both_vectors():
    S_in, S_out, *X = _seq_problem(seed=23)
    temps = [2.0, 0.25, 1.0]
    a, b, hist = orc.selective_mask_train_factorized_seq(S_in, S_out, *X, 0.03, 0.4, temps)
    a1, b1, h1 = orc.selective_mask_train_factorized_seq(S_in, S_out, *X, 0.03, 0.4, temps[:1])
    a2, b2, h2 = orc.selective_mask_train_factorized_seq(a1, b1, *X, 0.03, 0.4, temps[1:])
    assert np.array_equal(a, a2) and np.array_equal(b, b2) and np.array_equal(hist, np.concatenate([h1, h2]))
    sa, sb, _ = orc.selective_mask_train_factorized_seq(S_in, S_out, *X, 0.03, 0.4, temps[::-1])
    assert not np.allclose(sa, a) and not np.allclose(sb, b)
    assert not np.allclose(a, S_in) and not np.allclose(b, S_out)
    n0, _, h0 = orc.selective_mask_train_factorized_seq(S_in, S_out, *X, 0.03, 0.0, temps)
    assert np.array_equal(n0, S_in) and h0[1] == _seq_objective(S_in, S_out, X, 0.03, temps[1])


def test_sequence_training_small_steps_never_decrease_the_objective():
    S_in, S_out, *X = _seq_problem(n=12, m=4, seed=24)
    a, b, hist = orc.selective_mask_train_factorized_seq(S_in, S_out, *X, 0.01, 0.05, [1.0] * 40)
    final = _seq_objective(a, b, X, 0.01, 1.0)
    assert np.all(np.diff(hist) >= 0.0) and final >= hist[-1] and final > hist[0] + 1e-4
