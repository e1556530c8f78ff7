"""Pins for the oracle's random numbers and Random Mask (CPU only).

The generator is pinned to published splitmix64 outputs (tests/golden), the
counter form to the sequential generator, the mask to brute force and to the
properties Sec. 3.2 fixes (a binary selection matrix with one non-repeating
non-zero per row, a uniformly random subset).
"""
import os

import numpy as np
import pytest

from oracle import grass_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "splitmix64_vectors.txt")
MASK64 = (1 << 64) - 1


def _golden_vectors():
    rows = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            parts = line.split()
            rows.append((int(parts[0]), [int(x, 16) for x in parts[1:]]))
    return rows


def test_splitmix64_published_vectors():
    rows = _golden_vectors()
    assert len(rows) >= 2
    for seed, outs in rows:
        got = [int(v) for v in orc.splitmix64_sequence(seed, len(outs))]
        assert got == outs


def test_counter_form_equals_sequential_generator():
    for seed in (0, 1, 1234567, MASK64, 0xDEADBEEFCAFEF00D):
        seq = orc.splitmix64_sequence(seed, 10_000)
        ctr = orc.sm(seed, np.arange(10_000, dtype=np.uint64))
        assert np.array_equal(seq, ctr)


def test_stream_hash_is_generator_seeded_by_generator_output():
    seed, stream = 7, 18
    sub = int(orc.splitmix64_sequence(seed, stream + 1)[stream])
    want = orc.splitmix64_sequence(sub, 50)
    got = orc.stream_hash(seed, stream, np.arange(50, dtype=np.uint64))
    assert np.array_equal(want, got)
    # different streams are different sequences
    other = orc.stream_hash(seed, stream + 1, np.arange(50, dtype=np.uint64))
    assert not np.any(other == got)


def test_hash_bits_look_uniform():
    h = orc.stream_hash(0, 1, np.arange(1 << 16, dtype=np.uint64))
    for bit in (0, 1, 31, 32, 63):
        frac = float(((h >> np.uint64(bit)) & np.uint64(1)).mean())
        assert abs(frac - 0.5) < 4 * 0.5 / np.sqrt(1 << 16)


# ---------------------------------------------------------------- Random Mask
def _brute_force_mask(seed, stream, p, kprime):
    """Independent of the oracle's sort: Python integers and tuples."""
    sub = int(orc.splitmix64_sequence(seed, stream + 1)[stream])
    keys = [int(v) for v in orc.splitmix64_sequence(sub, p)]
    ranked = sorted(range(p), key=lambda j: (keys[j], j))
    return sorted(ranked[:kprime])


@pytest.mark.parametrize("p,kprime,seed,stream", [(1, 1, 0, 0), (17, 5, 0, 0), (100, 10, 3, 0),
                                                  (257, 256, 9, 16), (1000, 333, 0, 17)])
def test_mask_indices_brute_force(p, kprime, seed, stream):
    got = orc.mask_indices(seed, stream, p, kprime)
    assert got.dtype == np.int32
    assert got.tolist() == _brute_force_mask(seed, stream, p, kprime)


def test_mask_indices_structure():
    p, kp = 5000, 777
    idx = orc.mask_indices(0, 0, p, kp)
    assert idx.shape == (kp,)
    assert np.all(np.diff(idx) > 0)                  # ascending and distinct
    assert idx.min() >= 0 and idx.max() < p
    # nested: the k'-subset is the k'-smallest-key set, so it grows with k'
    bigger = orc.mask_indices(0, 0, p, kp + 100)
    assert set(idx.tolist()) <= set(bigger.tolist())


def test_mask_full_is_identity():
    for p in (1, 2, 63, 1000):
        assert orc.mask_indices(5, 0, p, p).tolist() == list(range(p))


def test_mask_rejects_bad_sizes():
    with pytest.raises(ValueError):
        orc.mask_indices(0, 0, 10, 11)
    with pytest.raises(ValueError):
        orc.mask_indices(0, 0, 10, 0)


def test_mask_inclusion_is_uniform_over_seeds():
    p, kp, trials = 64, 16, 4000
    hits = np.zeros(p)
    for seed in range(trials):
        hits[orc.mask_indices(seed, 0, p, kp)] += 1
    q = kp / p
    sd = np.sqrt(trials * q * (1 - q))
    assert np.all(np.abs(hits - trials * q) < 4.5 * sd)
    # pairs of coordinates: kept together with probability k'(k'-1)/(p(p-1))
    both = 0
    for seed in range(trials):
        s = set(orc.mask_indices(seed, 0, p, kp).tolist())
        both += (3 in s) and (40 in s)
    q2 = kp * (kp - 1) / (p * (p - 1))
    assert abs(both - trials * q2) < 4.5 * np.sqrt(trials * q2 * (1 - q2))


def test_mask_is_selection_matrix_product():
    rng = np.random.default_rng(0)
    p, kp, n = 300, 40, 5
    g = rng.standard_normal((n, p))
    idx = orc.mask_indices(1, 0, p, kp)
    M = np.zeros((kp, p))
    M[np.arange(kp), idx] = 1.0
    assert np.array_equal(M.sum(axis=1), np.ones(kp))     # one non-zero per row
    assert M.sum(axis=0).max() == 1.0                      # non-repeating
    assert np.array_equal(orc.mask(g, idx), g @ M.T)


def test_mask_norm_expectation():
    """M is binary (no rescaling), so E_seed ||M g||^2 = (k'/p) ||g||^2."""
    rng = np.random.default_rng(1)
    p, kp, trials = 128, 32, 3000
    g = rng.standard_normal(p) * rng.random(p)
    vals = np.array([np.sum(orc.mask(g, orc.mask_indices(s, 0, p, kp)) ** 2) for s in range(trials)])
    want = kp / p * np.sum(g ** 2)
    assert abs(vals.mean() - want) < 4.5 * vals.std() / np.sqrt(trials)
