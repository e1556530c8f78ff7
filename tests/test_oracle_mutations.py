"""The pins bite: each plausible mistake planted in the oracle (CPU only) makes
at least one pin fail.  Mistakes are planted by monkeypatching the oracle, never
the GPU path."""
import importlib.util
import os

import numpy as np
import pytest

from oracle import grass_oracle as orc

HERE = os.path.dirname(os.path.abspath(__file__))


def _load(name):
    spec = importlib.util.spec_from_file_location(name, os.path.join(HERE, name + ".py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


pins_sjlt = _load("test_oracle_sjlt")
pins_mask = _load("test_oracle_hash_mask")
pins_fact = _load("test_oracle_factgrass_score")
pins_fim = _load("test_oracle_fim")
pins_sm = _load("test_oracle_selective_mask")
pins_train = _load("test_oracle_selective_mask_train")

_U64 = np.uint64


def _tables_variant(flip_sign=False, low_bits=False, no_block_offset=False, counter_transposed=False):
    def tables(seed, stream, d, k, s):
        m = k // s
        if counter_transposed:
            c = (np.arange(d, dtype=np.uint64)[:, None] + np.arange(s, dtype=np.uint64)[None, :] * _U64(d)).ravel()
        else:
            c = np.arange(d * s, dtype=np.uint64)
        h = orc.stream_hash(seed, stream, c).reshape(d, s)
        word = (h & _U64(0xFFFFFFFF)) if low_bits else (h >> _U64(32))
        within = (word * _U64(m)) >> _U64(32)
        off = np.zeros(s, dtype=np.uint64) if no_block_offset else np.arange(s, dtype=np.uint64) * _U64(m)
        bucket = (within + off[None, :]).astype(np.uint32)
        plus = (h & _U64(1)) == (1 if flip_sign else 0)
        return bucket, np.where(plus, 1, -1).astype(np.int8)
    return tables


@pytest.mark.parametrize("kwargs", [dict(flip_sign=True), dict(low_bits=True), dict(counter_transposed=True)])
def test_wrong_hash_use_is_caught_by_the_integer_brute_force(monkeypatch, kwargs):
    monkeypatch.setattr(orc, "sjlt_tables", _tables_variant(**kwargs))
    with pytest.raises(AssertionError):
        pins_sjlt.test_tables_brute_force_from_sequential_generator()


def test_missing_block_offset_is_caught_by_the_structure_pin(monkeypatch):
    monkeypatch.setattr(orc, "sjlt_tables", _tables_variant(no_block_offset=True))
    with pytest.raises(AssertionError):
        pins_sjlt.test_tables_structure(200, 12, 4)


def test_missing_scale_is_caught_by_the_norm_pin(monkeypatch):
    def sjlt_unscaled(g, k, s, seed, stream=orc.STREAM_SJLT):
        g = np.asarray(g, dtype=np.float64)
        if g.ndim == 1:
            return sjlt_unscaled(g[None, :], k, s, seed, stream)[0]
        bucket, sign = orc.sjlt_tables(seed, stream, g.shape[1], k, s)
        out = np.zeros((g.shape[0], k))
        for i in range(g.shape[0]):
            for r in range(s):
                np.add.at(out[i], bucket[:, r], sign[:, r] * g[i])
        return out
    monkeypatch.setattr(orc, "sjlt", sjlt_unscaled)
    with pytest.raises(AssertionError):
        pins_sjlt.test_sjlt_preserves_squared_norm_in_expectation(4)


def test_dropped_sign_is_caught_by_the_dense_matrix_pin(monkeypatch):
    real = orc.sjlt_tables

    def all_plus(seed, stream, d, k, s):
        b, sg = real(seed, stream, d, k, s)
        return b, np.ones_like(sg)
    # the dense matrix is built from the same tables, so that pin alone cannot see it ...
    monkeypatch.setattr(orc, "sjlt_tables", all_plus)
    pins_sjlt.test_sjlt_equals_dense_matrix_product(97, 16, 1)
    # ... the sign-balance and integer brute-force pins do
    with pytest.raises(AssertionError):
        pins_sjlt.test_bucket_histogram_uniform_and_signs_balanced()
    with pytest.raises(AssertionError):
        pins_sjlt.test_tables_brute_force_from_sequential_generator()


def test_swapped_kronecker_order_is_caught(monkeypatch):
    def swapped(x, gout, idx_in, idx_out):
        xs = np.asarray(x, dtype=np.float64)[..., np.asarray(idx_in, dtype=np.int64)]
        gs = np.asarray(gout, dtype=np.float64)[..., np.asarray(idx_out, dtype=np.int64)]
        return np.einsum("nta,ntb->nba", xs, gs).reshape(xs.shape[0], -1)      # g (x) x instead of x (x) g
    monkeypatch.setattr(orc, "factgrass_sparsified_gradient", swapped)
    with pytest.raises(AssertionError):
        pins_fact.test_factgrass_equals_materialise_mask_sjlt()
    with pytest.raises(AssertionError):
        pins_fact.test_swapping_factors_changes_the_order()


def test_dropped_token_is_caught(monkeypatch):
    real = orc.factgrass_sparsified_gradient
    monkeypatch.setattr(orc, "factgrass_sparsified_gradient",
                        lambda x, g, ii, io: real(np.asarray(x)[:, :-1], np.asarray(g)[:, :-1], ii, io))
    with pytest.raises(AssertionError):
        pins_fact.test_vec_identity_of_eq2()


def test_mask_taking_largest_keys_is_caught(monkeypatch):
    def largest(seed, stream, p, kprime):
        j = np.arange(p, dtype=np.uint64)
        key = orc.stream_hash(seed, stream, j)
        order = np.lexsort((j, key))[::-1]
        return np.sort(order[:kprime]).astype(np.int32)
    monkeypatch.setattr(orc, "mask_indices", largest)
    with pytest.raises(AssertionError):
        pins_mask.test_mask_indices_brute_force(100, 10, 3, 0)


def test_grass_keyed_by_original_coordinate_is_caught(monkeypatch):
    def grass_wrong_key(g, idx, k, s, seed, stream=orc.STREAM_SJLT):
        g = np.asarray(g, dtype=np.float64)
        p = g.shape[-1]
        bucket, sign = orc.sjlt_tables(seed, stream, p, k, s)          # tables over [p), not over [k')
        out = np.zeros((g.shape[0], k))
        for i in range(g.shape[0]):
            for r in range(s):
                np.add.at(out[i], bucket[idx, r], sign[idx, r] * g[i, idx] / np.sqrt(s))
        return out
    monkeypatch.setattr(orc, "grass", grass_wrong_key)
    with pytest.raises(AssertionError):
        pins_sjlt.test_grass_equals_masked_matrix_product()


def test_mask_with_rescaling_is_caught(monkeypatch):
    real = orc.mask
    monkeypatch.setattr(orc, "mask", lambda g, idx: real(g, idx) * np.sqrt(np.asarray(g).shape[-1] / len(idx)))
    with pytest.raises(AssertionError):
        pins_mask.test_mask_norm_expectation()


def test_fim_without_the_sample_average_is_caught(monkeypatch):
    monkeypatch.setattr(orc, "fim", lambda G: np.asarray(G, np.float64).T @ np.asarray(G, np.float64))
    with pytest.raises(AssertionError):
        pins_fim.test_fim_is_the_average_outer_product()
    with pytest.raises(AssertionError):
        pins_fim.test_ifvp_woodbury_when_fewer_rows_than_columns()


def test_fim_of_the_transposed_matrix_is_caught(monkeypatch):
    monkeypatch.setattr(orc, "fim", lambda G: np.asarray(G, np.float64) @ np.asarray(G, np.float64).T / G.shape[0])
    with pytest.raises((AssertionError, ValueError)):
        pins_fim.test_fim_is_the_average_outer_product()


def test_ifvp_with_damping_dropped_or_scaled_is_caught(monkeypatch):
    def no_damping(G, F, lam):
        return np.linalg.solve(np.asarray(F, np.float64) + 1e-300 * np.eye(F.shape[0]), np.asarray(G, np.float64).T).T
    monkeypatch.setattr(orc, "ifvp", no_damping)
    with pytest.raises(AssertionError):
        pins_fim.test_ifvp_diagonal_fim_is_an_elementwise_division()

    def damping_times_k(G, F, lam):
        k = F.shape[0]
        return np.linalg.solve(np.asarray(F, np.float64) + lam * k * np.eye(k), np.asarray(G, np.float64).T).T
    monkeypatch.setattr(orc, "ifvp", damping_times_k)
    with pytest.raises(AssertionError):
        pins_fim.test_ifvp_rank_one_fim_sherman_morrison()


def test_ifvp_multiplying_instead_of_solving_is_caught(monkeypatch):
    monkeypatch.setattr(orc, "ifvp", lambda G, F, lam: np.asarray(G, np.float64) @ (F + lam * np.eye(F.shape[0])))
    with pytest.raises(AssertionError):
        pins_fim.test_ifvp_solves_the_damped_system()


def _sm_objective_variant(single_sigma=False, plus_penalty=False, no_centering=False):
    def objective(S, G, Gt, lam, temperature=1.0):
        S = np.asarray(S, np.float64); G = np.asarray(G, np.float64); Gt = np.asarray(Gt, np.float64)
        sig = 1.0 / (1.0 + np.exp(-S / temperature))
        w = sig if single_sigma else sig * sig
        total = 0.0
        for t in range(Gt.shape[0]):
            a = G @ Gt[t]; b = (G * w) @ Gt[t]
            da, db = (a, b) if no_centering else (a - a.mean(), b - b.mean())
            total += (da @ db) / np.sqrt((da @ da) * (db @ db))
        pen = lam * sig.sum()
        return total / Gt.shape[0] + (pen if plus_penalty else -pen)
    return objective


@pytest.mark.parametrize("kwargs", [dict(single_sigma=True), dict(plus_penalty=True), dict(no_centering=True)])
def test_selective_mask_objective_mistakes_are_caught(monkeypatch, kwargs):
    monkeypatch.setattr(orc, "selective_mask_objective", _sm_objective_variant(**kwargs))
    failed = 0
    for pin in (pins_sm.test_objective_matches_scipy_pearson_written_out,
                pins_sm.test_constant_logits_give_perfect_correlation,
                lambda: pins_sm.test_gradient_matches_central_differences(1.0, 0.07, 4)):
        try:
            pin()
        except AssertionError:
            failed += 1
    assert failed >= 1


def test_selective_mask_gradient_mistakes_are_caught(monkeypatch):
    good = orc.selective_mask_gradient
    monkeypatch.setattr(orc, "selective_mask_gradient", lambda S, G, Gt, lam, temperature=1.0: good(S, G, Gt, lam, 1.0))
    with pytest.raises(AssertionError):                     # temperature ignored
        pins_sm.test_gradient_matches_central_differences(0.5, 0.02, 5)
    monkeypatch.setattr(orc, "selective_mask_gradient", lambda S, G, Gt, lam, temperature=1.0: good(S, G, Gt, 0.0, temperature))
    with pytest.raises(AssertionError):                     # penalty term dropped
        pins_sm.test_gradient_matches_central_differences(1.0, 0.07, 4)
    monkeypatch.setattr(orc, "selective_mask_gradient",
                        lambda S, G, Gt, lam, temperature=1.0: 0.5 * (good(S, G, Gt, lam, temperature) - lam * 0) )
    with pytest.raises(AssertionError):                     # factor 2 of d(sigma^2) lost
        pins_sm.test_gradient_matches_central_differences(1.0, 0.0, 3)


def test_selective_mask_threshold_mistake_is_caught(monkeypatch):
    monkeypatch.setattr(orc, "selective_mask_indices",
                        lambda S, k=None: np.nonzero(np.asarray(S) > 0.5)[0].astype(np.int32))   # thresholds S, not sigma(S)
    with pytest.raises(AssertionError):
        pins_sm.test_index_extraction()


def _train_variant(descent=False, stale_temperature=False, no_step_size=False, history_after=False):
    def train(S0, G, Gt, lam, lr, temperatures):
        S = np.array(S0, dtype=np.float64, copy=True)
        history = []
        for i, T in enumerate(temperatures):
            Tg = temperatures[0] if stale_temperature else T
            step = (1.0 if no_step_size else lr) * orc.selective_mask_gradient(S, G, Gt, lam, Tg)
            if not history_after:
                history.append(orc.selective_mask_objective(S, G, Gt, lam, T))
            S = S - step if descent else S + step
            if history_after:
                history.append(orc.selective_mask_objective(S, G, Gt, lam, T))
        return S, np.asarray(history, dtype=np.float64)
    return train


@pytest.mark.parametrize("kwargs,pin", [
    (dict(descent=True), "test_first_step_moves_along_the_finite_difference_gradient"),
    (dict(descent=True), "test_small_steps_never_decrease_the_objective"),
    (dict(stale_temperature=True), "test_annealing_uses_the_temperature_of_its_own_step"),
    (dict(no_step_size=True), "test_a_dead_coordinate_follows_the_penalty_in_closed_form"),
    (dict(no_step_size=True), "test_no_steps_and_zero_step_size_leave_the_logits_alone"),
    (dict(history_after=True), "test_first_step_moves_along_the_finite_difference_gradient"),
])
def test_selective_mask_training_mistakes_are_caught(monkeypatch, kwargs, pin):
    monkeypatch.setattr(orc, "selective_mask_train", _train_variant(**kwargs))
    with pytest.raises(AssertionError):
        getattr(pins_train, pin)()



pins_train_fact = _load("test_oracle_selective_mask_train_factorized")


def _train_factorized_variant(descent=False, stale_temperature=False, only_input=False, sequential=False,
                              no_step_size=False, step_fn="selective_mask_factorized"):
    def train(S_in0, S_out0, Z_in, Z_out, Zt_in, Zt_out, lam, lr, temperatures):
        S_in = np.array(S_in0, dtype=np.float64, copy=True)
        S_out = np.array(S_out0, dtype=np.float64, copy=True)
        history = []
        step = 1.0 if no_step_size else lr
        for T in temperatures:
            Tg = temperatures[0] if stale_temperature else T
            obj, g_in, g_out = getattr(orc, step_fn)(S_in, S_out, Z_in, Z_out, Zt_in, Zt_out, lam, Tg)
            history.append(getattr(orc, step_fn)(S_in, S_out, Z_in, Z_out, Zt_in, Zt_out, lam, T)[0])
            S_in = S_in - step * g_in if descent else S_in + step * g_in
            if sequential:          # output derivative taken after the input logits have already moved
                g_out = getattr(orc, step_fn)(S_in, S_out, Z_in, Z_out, Zt_in, Zt_out, lam, Tg)[2]
            if not only_input:
                S_out = S_out - step * g_out if descent else S_out + step * g_out
        return S_in, S_out, np.asarray(history, dtype=np.float64)
    return train


@pytest.mark.parametrize("kwargs,pin", [
    (dict(descent=True), "test_first_step_moves_both_vectors_along_the_finite_difference_gradient"),
    (dict(descent=True), "test_small_steps_never_decrease_the_objective"),
    (dict(stale_temperature=True), "test_training_is_a_composition_of_its_steps_each_at_its_own_temperature"),
    (dict(only_input=True), "test_swapping_the_two_factors_swaps_the_two_results"),
    (dict(only_input=True), "test_dead_coordinates_of_either_factor_follow_the_penalty_in_closed_form"),
    (dict(sequential=True), "test_first_step_moves_both_vectors_along_the_finite_difference_gradient"),
    (dict(sequential=True), "test_swapping_the_two_factors_swaps_the_two_results"),
    (dict(no_step_size=True), "test_a_trivial_output_factor_reduces_it_to_the_plain_training_loop"),
    (dict(no_step_size=True), "test_no_steps_and_zero_step_size_leave_the_logits_alone"),
])
def test_factorised_selective_mask_training_mistakes_are_caught(monkeypatch, kwargs, pin):
    monkeypatch.setattr(orc, "selective_mask_train_factorized", _train_factorized_variant(**kwargs))
    with pytest.raises(AssertionError):
        getattr(pins_train_fact, pin)()


def _seq_variant(diagonal_pairs=False, unsquared=False, wrong_factor_in_grad=False):
    """Planted mistakes in the sequence form: only matching token positions (t = t') instead of all pairs; weights
    sigma instead of sigma^2; the input gradient weighted by the input factor's own token products."""
    def f(S_in, S_out, X_in, X_out, Xt_in, Xt_out, lam, temperature=1.0):
        S_in, S_out = np.asarray(S_in, np.float64), np.asarray(S_out, np.float64)
        si, so = 1 / (1 + np.exp(-S_in / temperature)), 1 / (1 + np.exp(-S_out / temperature))
        dsi, dso = si * (1 - si) / temperature, so * (1 - so) / temperature
        wi, wo = (si, so) if unsquared else (si * si, so * so)
        m, n = Xt_in.shape[0], X_in.shape[0]
        total, gi, go = 0.0, np.zeros_like(S_in), np.zeros_like(S_out)
        for te in range(m):
            exact, masked, kin, kout = np.zeros(n), np.zeros(n), [], []
            for i in range(n):
                e_in, e_out = X_in[i] @ Xt_in[te].T, X_out[i] @ Xt_out[te].T
                a, b = (X_in[i] * wi) @ Xt_in[te].T, (X_out[i] * wo) @ Xt_out[te].T
                if diagonal_pairs:
                    q = min(a.shape)
                    keep = np.zeros_like(a); keep[np.arange(q), np.arange(q)] = 1
                    e_in, a = e_in * keep, a * keep
                exact[i], masked[i] = np.sum(e_in * e_out), np.sum(a * b)
                kin.append(a); kout.append(b)
            da, db = exact - exact.mean(), masked - masked.mean()
            na, nb = np.sqrt(da @ da), np.sqrt(db @ db)
            corr = (da @ db) / (na * nb)
            total += corr
            c = da / (na * nb) - corr * db / (nb * nb)
            for i in range(n):
                gi += c[i] * np.einsum("ab,aj,bj->j", kin[i] if wrong_factor_in_grad else kout[i], X_in[i], Xt_in[te])
                go += c[i] * np.einsum("ab,aj,bj->j", kin[i], X_out[i], Xt_out[te])
        obj = total / m - lam * (si.sum() + so.sum())
        return obj, gi / m * 2 * si * dsi - lam * dsi, go / m * 2 * so * dso - lam * dso
    return f


@pytest.mark.parametrize("kwargs,pin,args", [
    (dict(diagonal_pairs=True), "test_sequence_factorized_objective_equals_the_plain_one_on_materialised_gradients", ()),
    (dict(diagonal_pairs=True), "test_sequence_form_ignores_token_order_and_all_zero_tokens", ()),
    (dict(unsquared=True), "test_sequence_factorized_objective_equals_the_plain_one_on_materialised_gradients", ()),
    (dict(unsquared=True), "test_sequence_form_with_one_token_is_the_single_token_form", ()),
    (dict(wrong_factor_in_grad=True), "test_sequence_factorized_gradients_match_central_differences", (1.0, 0.0, 3)),
    (dict(wrong_factor_in_grad=True), "test_sequence_form_with_one_token_is_the_single_token_form", ()),
])
def test_sequence_factorised_selective_mask_mistakes_are_caught(monkeypatch, kwargs, pin, args):
    monkeypatch.setattr(orc, "selective_mask_factorized_seq", _seq_variant(**kwargs))
    with pytest.raises(AssertionError):
        getattr(pins_sm, pin)(*args)


def test_sequence_graddot_with_matching_positions_only_is_caught(monkeypatch):
    def diag_only(X_in, X_out, Xt_in, Xt_out):
        q = min(X_in.shape[1], Xt_in.shape[1])
        return np.einsum("ita,mta,itb,mtb->mi", X_in[:, :q], Xt_in[:, :q], X_out[:, :q], Xt_out[:, :q])
    monkeypatch.setattr(orc, "graddot_factorized_seq", diag_only)
    with pytest.raises(AssertionError):
        pins_sm.test_sequence_graddot_equals_inner_products_of_materialised_layer_gradients()


@pytest.mark.parametrize("kwargs,pin", [
    (dict(descent=True), "test_sequence_training_first_step_follows_the_finite_difference_gradient_of_the_sequence_objective"),
    (dict(descent=True), "test_sequence_training_small_steps_never_decrease_the_objective"),
    (dict(stale_temperature=True), "test_sequence_training_is_a_composition_of_its_steps_and_moves_both_vectors"),
    (dict(only_input=True), "test_sequence_training_is_a_composition_of_its_steps_and_moves_both_vectors"),
    (dict(sequential=True), "test_sequence_training_first_step_follows_the_finite_difference_gradient_of_the_sequence_objective"),
    (dict(sequential=True), "test_sequence_training_with_one_token_is_the_single_token_loop"),
    (dict(no_step_size=True), "test_sequence_training_with_a_trivial_output_factor_is_the_plain_loop_on_token_sums"),
    (dict(step_fn="_single_token_step"), "test_sequence_training_with_a_trivial_output_factor_is_the_plain_loop_on_token_sums"),
])
def test_sequence_factorised_training_mistakes_are_caught(monkeypatch, kwargs, pin):
    """The loop variants above around the sequence objective; the last one trains on the first token only."""
    def first_token(S_in, S_out, X_in, X_out, Xt_in, Xt_out, lam, temperature=1.0):
        return orc.selective_mask_factorized(S_in, S_out, X_in[:, 0], X_out[:, 0], Xt_in[:, 0], Xt_out[:, 0], lam, temperature)
    monkeypatch.setattr(orc, "_single_token_step", first_token, raising=False)
    kw = dict(step_fn="selective_mask_factorized_seq")
    kw.update(kwargs)
    monkeypatch.setattr(orc, "selective_mask_train_factorized_seq", _train_factorized_variant(**kw))
    with pytest.raises(AssertionError):
        getattr(pins_train_fact, pin)()
