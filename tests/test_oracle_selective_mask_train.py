"""Pins for the oracle's Selective Mask training loop (Sec. 3.2 Eq. (1) solved by first-order ascent; App. B.4
temperature annealing and top-k extraction).  The objective itself is pinned against scipy in
test_oracle_selective_mask.py; here the loop around it is pinned by what gradient ascent must do."""
import numpy as np
import pytest
from scipy import stats

import synth
from oracle import grass_oracle as orc


def _problem(n=12, m=4, p=10, seed=0):
    rng = np.random.default_rng(seed)
    return 0.3 * rng.standard_normal(p), rng.standard_normal((n, p)), rng.standard_normal((m, p))


def test_no_steps_and_zero_step_size_leave_the_logits_alone():
    S, G, Gt = _problem()
    out, hist = orc.selective_mask_train(S, G, Gt, 0.01, 0.5, [])
    assert np.array_equal(out, S) and hist.size == 0 and out is not S
    out, hist = orc.selective_mask_train(S, G, Gt, 0.01, 0.0, [1.0, 1.0, 0.5])
    assert np.array_equal(out, S)
    assert hist[0] == hist[1] == orc.selective_mask_objective(S, G, Gt, 0.01, 1.0)
    assert hist[2] == orc.selective_mask_objective(S, G, Gt, 0.01, 0.5)


def test_first_step_moves_along_the_finite_difference_gradient():
    """S_1 - S_0 = lr * dL/dS, with the derivative taken by central differences of the objective (not by the
    oracle's own gradient routine)."""
    S, G, Gt = _problem(seed=1)
    lam, lr, T, h = 0.02, 0.7, 0.8, 1e-6
    out, hist = orc.selective_mask_train(S, G, Gt, lam, lr, [T])
    fd = np.empty_like(S)
    for j in range(S.size):
        e = np.zeros_like(S); e[j] = h
        fd[j] = (orc.selective_mask_objective(S + e, G, Gt, lam, T) - orc.selective_mask_objective(S - e, G, Gt, lam, T)) / (2 * h)
    assert np.allclose(out - S, lr * fd, rtol=1e-5, atol=1e-9)
    assert hist.shape == (1,) and np.isclose(hist[0], orc.selective_mask_objective(S, G, Gt, lam, T), rtol=0, atol=0)


def test_training_is_a_composition_of_its_steps():
    S, G, Gt = _problem(seed=2)
    temps = [1.0, 0.9, 0.8, 0.7, 0.6]
    whole, hist = orc.selective_mask_train(S, G, Gt, 0.01, 0.3, temps)
    first, h1 = orc.selective_mask_train(S, G, Gt, 0.01, 0.3, temps[:2])
    second, h2 = orc.selective_mask_train(first, G, Gt, 0.01, 0.3, temps[2:])
    assert np.array_equal(whole, second) and np.array_equal(hist, np.concatenate([h1, h2]))


def test_small_steps_never_decrease_the_objective():
    """Gradient ascent with a small enough step on a smooth objective is monotone (constant temperature)."""
    S, G, Gt = _problem(n=20, m=5, p=12, seed=3)
    out, hist = orc.selective_mask_train(S, G, Gt, 0.01, 0.05, [1.0] * 60)
    final = orc.selective_mask_objective(out, G, Gt, 0.01, 1.0)
    assert np.all(np.diff(hist) >= 0.0) and final >= hist[-1] and final > hist[0] + 1e-4


def test_a_dead_coordinate_follows_the_penalty_in_closed_form():
    """A coordinate that is zero in every gradient feels only -lam * sigma(S/T): its logit after one step is
    S - lr * lam * sigma (1 - sigma) / T, whatever the other coordinates do."""
    S, G, Gt = _problem(seed=4)
    G[:, 3] = 0.0
    Gt[:, 3] = 0.0
    lam, lr, T = 0.2, 1.5, 0.5
    out, _ = orc.selective_mask_train(S, G, Gt, lam, lr, [T])
    sig = 1.0 / (1.0 + np.exp(-S[3] / T))
    assert np.isclose(out[3], S[3] - lr * lam * sig * (1.0 - sig) / T, rtol=1e-12)
    # and it keeps sinking step after step
    many, _ = orc.selective_mask_train(S, G, Gt, lam, lr, [T] * 10)
    assert many[3] < out[3] < S[3]


def test_annealing_uses_the_temperature_of_its_own_step():
    """Two steps at temperatures (T0, T1) equal a step at T0 followed by a fresh run of one step at T1."""
    S, G, Gt = _problem(seed=5)
    both, hist = orc.selective_mask_train(S, G, Gt, 0.03, 0.4, [2.0, 0.25])
    a, _ = orc.selective_mask_train(S, G, Gt, 0.03, 0.4, [2.0])
    b, hb = orc.selective_mask_train(a, G, Gt, 0.03, 0.4, [0.25])
    assert np.array_equal(both, b) and hist[1] == hb[0]
    swapped, _ = orc.selective_mask_train(S, G, Gt, 0.03, 0.4, [0.25, 2.0])
    assert not np.allclose(swapped, both)


def test_graddot_correlation_is_scipy_pearson_of_masked_scores():
    _, G, Gt = _problem(n=15, m=3, p=9, seed=6)
    idx = np.array([1, 4, 5, 8])
    want = 0.0
    for t in range(3):
        exact = [sum(G[i, j] * Gt[t, j] for j in range(9)) for i in range(15)]
        masked = [sum(G[i, j] * Gt[t, j] for j in idx) for i in range(15)]
        want += stats.pearsonr(exact, masked)[0] / 3
    assert np.isclose(orc.graddot_correlation(G, Gt, idx), want, rtol=1e-12)
    assert np.isclose(orc.graddot_correlation(G, Gt, np.arange(9)), 1.0, rtol=1e-12)       # the full mask changes nothing
    # the soft objective with saturated logits and no penalty is the hard-mask correlation
    S = np.full(9, -60.0); S[idx] = 60.0
    assert np.isclose(orc.selective_mask_objective(S, G, Gt, 0.0), orc.graddot_correlation(G, Gt, idx), rtol=1e-9)


def test_trained_mask_finds_planted_coordinates_and_beats_a_random_mask():
    """On gradients whose scores are dominated by a few planted coordinates, training raises their logits above the
    rest, the top-k extraction recovers them, and the resulting mask preserves GradDot scores better than a Random
    Mask of the same size (the claim of Sec. 3.2 and Table 1 that Selective Mask improves on Random Mask)."""
    n, m, p, kept = 64, 8, 200, 20
    G, Gt, planted = synth.planted_gradients(n, m, p, kept, seed=7)
    G, Gt, planted = G.numpy(), Gt.numpy(), planted.numpy()
    # constant logits are a stationary point of the correlation term (corr = 1 there): start from small random ones
    S0 = 0.1 * np.random.default_rng(0).standard_normal(p)
    temps = np.geomspace(1.0, 0.3, 150)
    S, hist = orc.selective_mask_train(S0, G, Gt, 3e-3, 20.0, temps)
    rest = np.setdiff1d(np.arange(p), planted)
    assert S[planted].min() > S[rest].max() + 1.0
    idx = orc.selective_mask_indices(S, kept)
    assert np.array_equal(idx, planted.astype(np.int32))
    # with the annealed temperature the plain threshold sigma >= 1/2 selects the same coordinates (App. B.4)
    assert np.array_equal(orc.selective_mask_indices(S), planted.astype(np.int32))
    assert hist[-1] > hist[0]
    c_sel = orc.graddot_correlation(G, Gt, idx)
    c_rand = np.mean([orc.graddot_correlation(G, Gt, orc.mask_indices(sd, 0, p, kept)) for sd in range(20)])
    assert c_sel > 0.9 and c_sel > c_rand + 0.2
