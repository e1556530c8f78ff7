"""Pins for the oracle's SJLT and GraSS (CPU only).

Sec. 3.1 fixes: SJLT is the product with a k x p matrix that has s non-zero
+-1 entries per column; equivalently a scan in which each g(j) is added to or
subtracted from s output coordinates; cost scales with nnz(g) (zeros
contribute nothing).  Sec. 3.3.1 fixes GraSS = SJLT o Mask and its two limits.
The JL property gives E||SJLT g||^2 = ||g||^2; for s = 1 (a count sketch) the
variance has the closed form (2/k)(||g||_2^4 - ||g||_4^4).
"""
import numpy as np
import pytest

from oracle import grass_oracle as orc


def dense_matrix(seed, stream, d, k, s):
    """Materialise P (k x d) entry by entry from the tables."""
    bucket, sign = orc.sjlt_tables(seed, stream, d, k, s)
    P = np.zeros((k, d))
    for j in range(d):
        for r in range(s):
            P[bucket[j, r], j] += sign[j, r] / np.sqrt(s)
    return P


@pytest.mark.parametrize("d,k,s", [(1, 1, 1), (50, 8, 1), (333, 16, 2), (200, 12, 4), (64, 64, 64)])
def test_tables_structure(d, k, s):
    bucket, sign = orc.sjlt_tables(3, 1, d, k, s)
    assert bucket.shape == (d, s) and sign.shape == (d, s)
    assert bucket.dtype == np.uint32 and sign.dtype == np.int8
    m = k // s
    for r in range(s):                       # r-th non-zero lives in block r
        assert bucket[:, r].min() >= r * m and bucket[:, r].max() < (r + 1) * m
    assert set(np.unique(sign).tolist()) <= {-1, 1}
    P = dense_matrix(3, 1, d, k, s)
    assert np.all((P != 0).sum(axis=0) == s)               # exactly s non-zeros per column
    assert np.allclose(np.abs(P[P != 0]), 1 / np.sqrt(s))


def test_tables_brute_force_from_sequential_generator():
    """Bucket and sign recomputed with Python integers from the sequential
    generator (pinned to published vectors in test_oracle_hash_mask)."""
    seed, stream, d, k, s = 11, 1, 40, 12, 3
    sub = int(orc.splitmix64_sequence(seed, stream + 1)[stream])
    hs = [int(v) for v in orc.splitmix64_sequence(sub, d * s)]
    bucket, sign = orc.sjlt_tables(seed, stream, d, k, s)
    m = k // s
    for j in range(d):
        for r in range(s):
            h = hs[j * s + r]
            assert bucket[j, r] == r * m + (((h >> 32) * m) >> 32)
            assert sign[j, r] == (1 if h % 2 == 0 else -1)


def test_entries_are_the_table_rows_of_the_asked_positions():
    """Entries for a subset of positions (any order, beyond any table that fits in memory) are the rows of the full
    table; at a position near 2**31 the hash counter j*s + r is taken in 64 bits (checked with Python integers)."""
    d, k, s = 5000, 96, 3
    bucket, sign = orc.sjlt_tables(11, 1, d, k, s)
    pos = np.array([4999, 0, 17, 17, 2500], dtype=np.uint64)
    b, g = orc.sjlt_entries(11, 1, pos, k, s)
    assert np.array_equal(b, bucket[pos.astype(np.int64)]) and np.array_equal(g, sign[pos.astype(np.int64)])
    j, m = 2**31 - 2, k // s
    b, g = orc.sjlt_entries(11, 1, [j], k, s)
    for r in range(s):
        h = int(orc.stream_hash(11, 1, np.array([j * s + r], dtype=np.uint64))[0])
        assert int(b[0, r]) == r * m + (((h >> 32) * m) >> 32)
        assert int(g[0, r]) == (1 if h & 1 == 0 else -1)


def test_tables_reject_s_not_dividing_k():
    with pytest.raises(ValueError):
        orc.sjlt_tables(0, 1, 10, 10, 3)


def test_bucket_histogram_uniform_and_signs_balanced():
    d, k = 1 << 16, 64
    bucket, sign = orc.sjlt_tables(0, 1, d, k, 1)
    counts = np.bincount(bucket[:, 0], minlength=k)
    chi2 = ((counts - d / k) ** 2 / (d / k)).sum()
    assert chi2 < 63 + 5 * np.sqrt(2 * 63)                 # chi^2_{63}: mean 63, sd ~11.2
    assert abs(sign.astype(np.float64).mean()) < 4 / np.sqrt(d)
    # bucket and sign are uncorrelated
    assert abs(np.corrcoef(bucket[:, 0], sign[:, 0])[0, 1]) < 4 / np.sqrt(d)


@pytest.mark.parametrize("d,k,s", [(97, 16, 1), (300, 32, 4), (128, 8, 2)])
def test_sjlt_equals_dense_matrix_product(d, k, s):
    rng = np.random.default_rng(d)
    g = rng.standard_normal((6, d))
    P = dense_matrix(5, 1, d, k, s)
    got = orc.sjlt(g, k, s, seed=5, stream=1)
    assert np.allclose(got, g @ P.T, rtol=0, atol=1e-12)


def test_sjlt_vectorised_equals_python_scan():
    rng = np.random.default_rng(2)
    d, k, s = 211, 24, 3
    g = rng.standard_normal((3, d))
    bucket, sign = orc.sjlt_tables(9, 1, d, k, s)
    got = orc.sjlt(g, k, s, seed=9, stream=1)
    for i in range(3):
        assert np.allclose(got[i], orc.sjlt_scan(g[i], bucket, sign, k), rtol=0, atol=1e-13)


def test_sjlt_linearity():
    rng = np.random.default_rng(3)
    d, k, s = 500, 32, 2
    u, v = rng.standard_normal((2, d))
    a, b = 0.7, -2.25
    lhs = orc.sjlt(a * u + b * v, k, s, 1)
    rhs = a * orc.sjlt(u, k, s, 1) + b * orc.sjlt(v, k, s, 1)
    assert np.allclose(lhs, rhs, rtol=0, atol=1e-12)


def test_sjlt_basis_vector_gives_column():
    d, k, s = 37, 20, 4
    bucket, sign = orc.sjlt_tables(4, 1, d, k, s)
    for j in (0, 5, 36):
        e = np.zeros(d)
        e[j] = 1.0
        out = orc.sjlt(e, k, s, 4)
        want = np.zeros(k)
        want[bucket[j]] = sign[j] / 2.0                     # 1/sqrt(4)
        assert np.array_equal(out, want)


def test_sjlt_zero_input_and_zero_entries():
    d, k = 400, 16
    assert not orc.sjlt(np.zeros((2, d)), k, 1, 0).any()
    rng = np.random.default_rng(4)
    g = rng.standard_normal(d)
    g[rng.random(d) < 0.8] = 0.0
    nz = np.flatnonzero(g)
    bucket, sign = orc.sjlt_tables(0, 1, d, k, 1)
    want = np.zeros(k)
    np.add.at(want, bucket[nz, 0], sign[nz, 0] * g[nz])     # visit the non-zeros only
    assert np.allclose(orc.sjlt(g, k, 1, 0), want, rtol=0, atol=1e-13)


@pytest.mark.parametrize("s", [1, 4])
def test_sjlt_preserves_squared_norm_in_expectation(s):
    rng = np.random.default_rng(5)
    d, k, trials = 96, 16, 3000
    g = rng.standard_normal(d) * (rng.random(d) < 0.5)
    n2 = np.sum(g ** 2)
    vals = np.array([np.sum(orc.sjlt(g, k, s, seed) ** 2) for seed in range(trials)])
    assert abs(vals.mean() - n2) < 4.5 * vals.std() / np.sqrt(trials)
    if s == 1:
        var = 2.0 / k * (n2 ** 2 - np.sum(g ** 4))
        # sample variance of ~3000 draws: allow 15 %
        assert abs(vals.var() - var) < 0.15 * var


def test_sjlt_preserves_inner_products_in_expectation():
    rng = np.random.default_rng(6)
    d, k, trials = 80, 16, 3000
    u, v = rng.standard_normal((2, d))
    vals = np.array([orc.sjlt(u, k, 2, seed) @ orc.sjlt(v, k, 2, seed) for seed in range(trials)])
    assert abs(vals.mean() - u @ v) < 4.5 * vals.std() / np.sqrt(trials)


def test_sjlt_pairwise_distance_preserved_for_large_k():
    """JL: with k large the distortion of a pairwise distance is small."""
    rng = np.random.default_rng(7)
    d, k = 4096, 2048
    u, v = rng.standard_normal((2, d))
    su, sv = orc.sjlt(np.stack([u, v]), k, 1, 0)
    ratio = np.linalg.norm(su - sv) / np.linalg.norm(u - v)
    assert abs(ratio - 1) < 5 * np.sqrt(1.0 / k)


# ------------------------------------------------------------------- GraSS
def test_grass_equals_masked_matrix_product():
    """SJLT of the masked vector equals (P' M) g with both matrices explicit."""
    rng = np.random.default_rng(8)
    p, kp, k, s, n = 400, 60, 12, 2, 4
    g = rng.standard_normal((n, p))
    idx = orc.mask_indices(2, 0, p, kp)
    M = np.zeros((kp, p))
    M[np.arange(kp), idx] = 1
    Pp = dense_matrix(2, 1, kp, k, s)
    got = orc.grass(g, idx, k, s, seed=2)
    assert np.allclose(got, g @ (Pp @ M).T, rtol=0, atol=1e-12)
    # zero-filled p-vector through the masked SJLT: only kept coordinates matter
    g2 = g.copy()
    drop = np.setdiff1d(np.arange(p), idx)
    g2[:, drop] = rng.standard_normal((n, drop.size))
    assert np.array_equal(orc.grass(g2, idx, k, s, seed=2), got)


def test_grass_limit_full_mask_is_sjlt():
    rng = np.random.default_rng(9)
    p, k = 250, 10
    g = rng.standard_normal((3, p))
    idx = orc.mask_indices(0, 0, p, p)
    assert np.array_equal(orc.grass(g, idx, k, 1, seed=0), orc.sjlt(g, k, 1, seed=0))


def test_grass_limit_kprime_equals_k_is_signed_scatter_of_the_mask():
    rng = np.random.default_rng(10)
    p, k = 250, 16
    g = rng.standard_normal(p)
    idx = orc.mask_indices(0, 0, p, k)
    out = orc.grass(g, idx, k, 1, seed=0)
    # every kept value lands, with its sign, in the bucket of its compact position
    bucket, sign = orc.sjlt_tables(0, 1, k, k, 1)
    want = np.zeros(k)
    for jp in range(k):
        want[bucket[jp, 0]] += sign[jp, 0] * g[idx[jp]]
    assert np.allclose(out, want, rtol=0, atol=1e-13)


def test_max_rel_err_definition():
    want = np.array([[1.0, -4.0], [0.0, 0.0]])
    got = np.array([[1.0, -4.4], [0.5, 0.0]])
    assert np.isclose(orc.max_rel_err(got, want), 0.5)      # second row: zero oracle row -> absolute
    assert np.isclose(orc.max_rel_err(got[:1], want[:1]), 0.1)
