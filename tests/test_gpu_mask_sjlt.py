"""GPU parity: Random Mask indices, hash tables, mask gather, SJLT and fused
GraSS against the CPU oracle, through the C ABI.

Bars: bit-exact for indices, buckets and signs and for the gather (a copy);
max relative error (largest absolute difference in a row over the largest
absolute oracle value of that row) <= 1e-5 for fp32 SJLT / GraSS outputs.
"""
import numpy as np
import pytest
import torch

import synth
from oracle import grass_oracle as orc

pytestmark = pytest.mark.gpu

TOL_SJLT = 1e-5


@pytest.fixture(scope="module")
def grass():
    import paper_2505_18976_amd as g
    g.load_library()
    yield g


def _dev():
    return torch.device("cuda:0")


# ------------------------------------------------------------------ tables
@pytest.mark.parametrize("d,k,s,seed,stream", [(1, 1, 1, 0, 1), (1000, 1024, 1, 0, 1), (4099, 4096, 4, 7, 18),
                                               (65536, 1000, 2, 3, 1), (300, 64, 64, 1, 22), (70001, 8192, 1, 0, 1)])
def test_sjlt_tables_bit_exact(grass, d, k, s, seed, stream):
    bucket, sign = grass.grass_sjlt_tables(seed, stream, d, k, s, device=_dev())
    torch.cuda.synchronize()
    rb, rs = orc.sjlt_tables(seed, stream, d, k, s)
    assert np.array_equal(bucket.cpu().numpy().view(np.uint32), rb)
    assert np.array_equal(sign.cpu().numpy(), rs)


# ------------------------------------------------------------ mask indices
@pytest.mark.parametrize("p,kp,seed,stream", [(1, 1, 0, 0), (2, 1, 1, 0), (100, 10, 0, 0), (2048, 2048, 5, 0),
                                              (2049, 1, 2, 16), (4096, 64, 0, 16), (4096, 64, 0, 17),
                                              (65536, 8192, 0, 0), (100003, 99999, 4, 0),
                                              (1863690, 65536, 0, 0)])
def test_mask_indices_bit_exact(grass, p, kp, seed, stream):
    idx = grass.grass_mask_indices(seed, stream, p, kp, device=_dev())
    torch.cuda.synchronize()
    ref = orc.mask_indices(seed, stream, p, kp)
    assert np.array_equal(idx.cpu().numpy(), ref)
    assert grass.grass_check_indices(idx, p)


def test_mask_indices_resnet_scale(grass):
    p, kp = 11173962, 32768
    idx = grass.grass_mask_indices(0, 0, p, kp, device=_dev())
    torch.cuda.synchronize()
    assert np.array_equal(idx.cpu().numpy(), orc.mask_indices(0, 0, p, kp))


def test_check_indices_flags_bad_input(grass):
    good = torch.tensor([0, 3, 9], dtype=torch.int32, device=_dev())
    assert grass.grass_check_indices(good, 10)
    assert not grass.grass_check_indices(good, 9)                                   # out of range
    bad = torch.tensor([0, 3, 3], dtype=torch.int32, device=_dev())
    assert not grass.grass_check_indices(bad, 10)                                   # repeated
    bad2 = torch.tensor([4, 3, 9], dtype=torch.int32, device=_dev())
    assert not grass.grass_check_indices(bad2, 10)                                  # not ascending


# ------------------------------------------------------------------ gather
@pytest.mark.parametrize("n,p,kp,pad", [(1, 10, 10, 0), (5, 1000, 37, 3), (64, 65536, 8192, 0), (19, 5000, 4999, 1)])
def test_mask_gather_exact(grass, n, p, kp, pad):
    full = synth.bernoulli_sparse_normal(n, p + pad, 0.5, 1.0, seed=11, device=_dev())
    g = full[:, :p]
    idx = grass.grass_mask_indices(0, 0, p, kp, device=_dev())
    out = grass.grass_mask(g, idx)
    torch.cuda.synchronize()
    want = orc.mask(g.cpu().numpy(), idx.cpu().numpy())
    assert np.array_equal(out.cpu().numpy(), want)


# -------------------------------------------------------------------- SJLT
SJLT_CASES = [
    # n, d, k, s, row padding (changes alignment / vector width)
    (1, 1, 8, 1, 0),
    (3, 5, 8, 2, 0),
    (8, 1000, 1000, 1, 0),
    (13, 4099, 1024, 1, 1),
    (13, 4099, 1024, 4, 2),
    (5, 70001, 4096, 1, 3),
    (9, 70002, 4096, 2, 0),
    (6, 33000, 8192, 1, 0),
    (2, 20000, 32768, 1, 0),
    (64, 65536, 1024, 1, 0),
    (17, 8192, 16, 1, 0),
    (3, 100, 8, 8, 0),                   # s = k: every row of P is hit (dense Rademacher limit)
    (4, 9000, 3000, 3, 0),               # m not a power of two
]


@pytest.mark.parametrize("n,d,k,s,pad", SJLT_CASES)
def test_sjlt_parity(grass, n, d, k, s, pad):
    full = synth.bernoulli_sparse_normal(n, d + pad, 0.6, 1.0, seed=21, device=_dev())
    g = full[:, :d]
    out = grass.grass_sjlt(g, k, s, seed=0, stream_id=1)
    torch.cuda.synchronize()
    ref = orc.sjlt(g.cpu().numpy(), k, s, 0, 1)
    assert orc.max_rel_err(out.cpu().numpy(), ref) <= TOL_SJLT


# Unmasked rows are grouped so that all rows of a workgroup start at the same offset inside a 128-byte line
# (row period P = 32 / gcd(ld mod 32, 32)) and the vector loop starts on a line; the cases below walk through
# P = 32, 16, 8, 1, a ragged last block of rows, a misaligned base pointer and inputs shorter than the lead-in.
ALIGNED_CASES = [
    # n, d, pad (ld = off + d + pad), off (first column of the view), k, s
    (1100, 1001, 0, 0, 64, 1),           # ld mod 32 = 9: P = 32, 8 rows per group, last block ragged
    (520, 2050, 0, 0, 2048, 2),          # ld mod 32 = 2: P = 16
    (70, 4100, 0, 0, 8192, 1),           # ld mod 32 = 4: P = 8, 2 rows per group
    (40, 3000, 5, 3, 512, 4),            # ld = 3008: P = 1, base 12 bytes into a line (29 leading positions)
    (9, 64, 0, 0, 16, 1),                # one line per row
    (4, 10, 51, 3, 8, 1),                # fewer positions than the lead-in
    (5, 20, 12, 7, 8, 1),                # too few rows to group: consecutive rows, scalar loads
    (33, 70001, 31, 0, 1024, 1),         # ld = 70032 (mod 32 = 16): P = 2, several chunks
]


@pytest.mark.parametrize("n,d,pad,off,k,s", ALIGNED_CASES)
def test_sjlt_line_aligned_row_groups(grass, n, d, pad, off, k, s):
    full = synth.bernoulli_sparse_normal(n, off + d + pad, 0.5, 1.0, seed=23, device=_dev())
    g = full[:, off:off + d]
    out = grass.grass_sjlt(g, k, s, seed=3, stream_id=1)
    torch.cuda.synchronize()
    ref = orc.sjlt(g.cpu().numpy(), k, s, 3, 1)
    assert orc.max_rel_err(out.cpu().numpy(), ref) <= TOL_SJLT


# bf16 gradients: 64 elements per 128-byte line, 8 per 16-byte load; row periods 64 ... 1, consecutive-row fallbacks
BF16_CASES = [
    # n, d, pad, off, k, s, k' (0 = unmasked)
    (3, 5, 0, 0, 8, 2, 0),
    (2100, 1001, 0, 0, 64, 1, 0),         # ld mod 64 = 41: P = 64, 8 rows per group
    (600, 2050, 0, 0, 2048, 2, 0),        # ld mod 64 = 2: P = 32
    (70, 4104, 0, 0, 8192, 1, 0),         # ld mod 64 = 8: P = 8, 2 rows per group
    (40, 3000, 69, 3, 512, 4, 0),         # ld = 3072: P = 1, base 6 bytes into a line
    (9, 128, 0, 0, 16, 1, 0),
    (4, 10, 115, 3, 8, 1, 0),             # fewer positions than the lead-in
    (5, 24, 0, 0, 8, 1, 0),               # too few rows to group, rows 16-byte aligned: 8-element loads
    (5, 21, 0, 0, 8, 1, 0),               # ... and not aligned: scalar loads
    (33, 70001, 31, 0, 1024, 1, 0),
    (7, 3000, 0, 0, 64, 2, 500),          # fused mask
    (64, 65536, 0, 0, 1024, 1, 8192),
    (10, 100003, 0, 0, 4096, 4, 9973),
]


@pytest.mark.parametrize("n,d,pad,off,k,s,kp", BF16_CASES)
def test_sjlt_bf16_inputs(grass, n, d, pad, off, k, s, kp):
    full = synth.bernoulli_sparse_normal(n, off + d + pad, 0.5, 1.0, seed=24, device=_dev()).to(torch.bfloat16)
    g = full[:, off:off + d]
    exact = g.float().cpu().numpy()                              # bf16 values are exact in fp32
    if kp:
        idx = grass.grass_mask_indices(2, 0, d, kp, device=_dev())
        out = grass.grass_sjlt_bf16(g, k, s, seed=3, stream_id=1, idx=idx)
        ref = orc.grass(exact, orc.mask_indices(2, 0, d, kp), k, s, 3)
    else:
        out = grass.grass_sjlt_bf16(g, k, s, seed=3, stream_id=1)
        ref = orc.sjlt(exact, k, s, 3, 1)
    torch.cuda.synchronize()
    assert orc.max_rel_err(out.cpu().numpy(), ref) <= TOL_SJLT


# Long unmasked rows with s = 1 and at least 16 groups of rows read bucket and sign from a 16-bit table that the call
# builds in its workspace; the same call with a workspace that only holds the partial sums hashes per position.
# Both must match the oracle, and each other bit for bit (same values added in the same order).
TABLE_CASES = [
    # n, d, pad, off, k, bf16
    (130, 70001, 15, 0, 512, False),      # ld = 70016: P = 1, ragged tail of positions, 17 groups of 8 rows
    (140, 66001, 31, 0, 1000, False),     # m not a power of two
    (1100, 65537, 0, 0, 256, False),      # ld mod 32 = 1: P = 32
    (70, 70001, 15, 3, 8192, False),      # 4 rows per group, lead-in of 29 positions, k of the headline
    (40, 66000, 16, 0, 16384, False),     # 2 rows per group
    (130, 70001, 15, 0, 512, True),
    (150, 65600, 0, 5, 4096, True),       # bf16, lead-in of 59 positions
]


@pytest.mark.parametrize("n,d,pad,off,k,bf16", TABLE_CASES)
def test_sjlt_bucket_table_path(grass, n, d, pad, off, k, bf16):
    full = synth.bernoulli_sparse_normal(n, off + d + pad, 0.5, 1.0, seed=29, device=_dev())
    if bf16:
        full = full.to(torch.bfloat16)
    g = full[:, off:off + d]
    fn = grass.grass_sjlt_bf16 if bf16 else grass.grass_sjlt
    nbytes = grass.grass_sjlt_workspace_bytes(n, d, 0, k, 1)
    assert nbytes >= 2 * d                                        # the query reserves the table
    ws = torch.empty(nbytes, dtype=torch.uint8, device=_dev())
    out = fn(g, k, 1, seed=9, stream_id=1, ws=ws)
    small = ws[:max(256, nbytes - 2 * d)]                         # partial sums only: no room for the table
    plain = fn(g, k, 1, seed=9, stream_id=1, ws=small)
    torch.cuda.synchronize()
    ref = orc.sjlt(g.float().cpu().numpy(), k, 1, 9, 1)
    assert orc.max_rel_err(out.cpu().numpy(), ref) <= TOL_SJLT
    assert torch.equal(out, plain)


def test_sjlt_random_shapes_and_alignments(grass):
    """60 seeded random problems: shape, leading dimension, view offset, element type, mask, k and s all vary, so that
    every row period, lead-in length, vector width and chunk count of the planner is hit by something."""
    rng = np.random.default_rng(12345)
    for case in range(60):
        bf16 = bool(rng.integers(2))
        n = int(rng.choice([1, 2, 7, 33, 150, 700, 2200]))
        d = int(rng.integers(1, 6000)) if n > 100 else int(rng.integers(1, 90000))
        off, pad = int(rng.integers(0, 9)), int(rng.integers(0, 70))
        s = int(rng.choice([1, 1, 2, 4]))
        k = s * int(rng.choice([1, 3, 16, 250, 1024, 4096]))
        masked = bool(rng.integers(3) == 0)
        full = synth.bernoulli_sparse_normal(n, off + d + pad, float(rng.choice([0.0, 0.5, 0.95])), 1.0,
                                             seed=5000 + case, device=_dev())
        if bf16:
            full = full.to(torch.bfloat16)
        g = full[:, off:off + d]
        exact = g.float().cpu().numpy()
        fn = grass.grass_sjlt_bf16 if bf16 else grass.grass_sjlt
        if masked:
            kp = int(rng.integers(1, d + 1))
            idx = grass.grass_mask_indices(case, 0, d, kp, device=_dev())
            out = fn(g, k, s, seed=case, stream_id=1, idx=idx)
            ref = orc.grass(exact, orc.mask_indices(case, 0, d, kp), k, s, case)
        else:
            out = fn(g, k, s, seed=case, stream_id=1)
            ref = orc.sjlt(exact, k, s, case, 1)
        torch.cuda.synchronize()
        err = orc.max_rel_err(out.cpu().numpy(), ref)
        assert err <= TOL_SJLT, (case, bf16, n, d, off, pad, k, s, masked, err)


@pytest.mark.parametrize("rows,chunks,threads,acc", [(1, 1, 256, 0), (2, 3, 512, 1), (4, 7, 1024, 2), (8, 2, 256, 3),
                                                     (8, 1, 1024, 2), (4, 1, 512, 1), (2, 5, 1024, 3)])
def test_sjlt_parity_across_launch_shapes(grass, rows, chunks, threads, acc):
    n, d, k, s = 11, 50001, 2048, 2
    g = synth.bernoulli_sparse_normal(n, d, 0.3, 1.0, seed=22, device=_dev())
    ref = orc.sjlt(g.cpu().numpy(), k, s, 5, 1)
    tuning = dict(sjlt_rows_per_block=rows, sjlt_column_chunks=chunks, sjlt_threads=threads, sjlt_accumulator=acc)
    out = grass.grass_sjlt(g, k, s, seed=5, stream_id=1, tuning=tuning)
    torch.cuda.synchronize()
    assert orc.max_rel_err(out.cpu().numpy(), ref) <= TOL_SJLT


@pytest.mark.parametrize("masked", [False, True])
def test_sjlt_non_finite_values_stay_in_their_buckets(grass, masked):
    """A NaN or an infinity in a gradient reaches exactly the buckets its coordinate maps to (the zero test that skips
    exact zeros must not swallow it, and it must not leak into other buckets or rows); -0.0 counts as zero."""
    n, d, k, s = 6, 5000, 256, 2
    g = synth.bernoulli_sparse_normal(n, d, 0.5, 1.0, seed=31, device=_dev())
    g[1, 17] = float("nan")
    g[2, 4999] = float("inf")
    g[3, 0] = float("-inf")
    g[4, 123] = -0.0
    if masked:
        keep = np.unique(np.concatenate([[0, 17, 123, 4999], np.arange(5, 5000, 7)])).astype(np.int32)
        idx = torch.from_numpy(keep).to(_dev())
        out = grass.grass_sjlt(g, k, s, seed=4, stream_id=1, idx=idx)
        with np.errstate(invalid="ignore"):
            ref = orc.grass(g.cpu().numpy(), keep, k, s, 4, 1)
    else:
        out = grass.grass_sjlt(g, k, s, seed=4, stream_id=1)
        with np.errstate(invalid="ignore"):
            ref = orc.sjlt(g.cpu().numpy(), k, s, 4, 1)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert np.array_equal(np.isnan(got), np.isnan(ref))
    assert np.array_equal(np.isposinf(got), np.isposinf(ref)) and np.array_equal(np.isneginf(got), np.isneginf(ref))
    assert np.isnan(ref[1]).sum() == s and np.isinf(ref[2]).sum() == s and np.isinf(ref[3]).sum() == s
    fin = np.isfinite(ref)
    for i in range(n):
        scale = np.abs(ref[i][fin[i]]).max()
        assert np.abs(got[i][fin[i]] - ref[i][fin[i]]).max() <= TOL_SJLT * scale


def test_sjlt_dense_zero_and_offset_output(grass):
    n, d, k = 4, 3000, 256
    g = torch.zeros((n, d), dtype=torch.float32, device=_dev())
    wide = torch.full((n, 3 * k), 7.0, dtype=torch.float32, device=_dev())
    out = grass.grass_sjlt(g, k, 1, seed=0, out=wide[:, k:2 * k])                  # ldo = 3k
    torch.cuda.synchronize()
    w = wide.cpu().numpy()
    assert not w[:, k:2 * k].any()
    assert np.all(w[:, :k] == 7.0) and np.all(w[:, 2 * k:] == 7.0)                   # neighbours untouched
    assert out.data_ptr() == wide[:, k:2 * k].data_ptr()


# ------------------------------------------------------------------- GraSS
GRASS_CASES = [
    # n, p, k', k, s
    (1, 10, 10, 4, 1),
    (7, 3000, 500, 64, 2),
    (64, 65536, 8192, 1024, 1),          # the tiny config of the benchmark suite
    (10, 100003, 9973, 4096, 4),
    (5, 20000, 20000, 1000, 1),          # k' = p: plain SJLT
    (3, 50000, 128, 128, 1),             # k' = k: sparsification only (signed scatter)
]


@pytest.mark.parametrize("n,p,kp,k,s", GRASS_CASES)
def test_fused_grass_parity(grass, n, p, kp, k, s):
    g = synth.bernoulli_sparse_normal(n, p, 0.8, 1.0, seed=1001, device=_dev())
    idx = grass.grass_mask_indices(0, 0, p, kp, device=_dev())
    out = grass.grass_sjlt(g, k, s, seed=0, stream_id=1, idx=idx)
    torch.cuda.synchronize()
    ref = orc.grass(g.cpu().numpy(), idx.cpu().numpy(), k, s, 0, 1)
    assert orc.max_rel_err(out.cpu().numpy(), ref) <= TOL_SJLT
    # fused == two-step through the library's own gather
    two = grass.grass_sjlt(grass.grass_mask(g, idx), k, s, seed=0, stream_id=1)
    torch.cuda.synchronize()
    assert orc.max_rel_err(two.cpu().numpy(), ref) <= TOL_SJLT


def test_fused_grass_with_caller_supplied_indices(grass):
    """Selective Mask: the caller brings the indices (Sec. 3.2); any ascending set works."""
    n, p, k = 6, 40000, 512
    g = synth.bernoulli_sparse_normal(n, p, 0.5, 1.0, seed=31, device=_dev())
    idx_np = np.sort(np.random.default_rng(0).choice(p, size=3001, replace=False)).astype(np.int32)
    idx = torch.from_numpy(idx_np).to(_dev())
    out = grass.grass_sjlt(g, k, 1, seed=9, stream_id=1, idx=idx)
    torch.cuda.synchronize()
    ref = orc.grass(g.cpu().numpy(), idx_np, k, 1, 9, 1)
    assert orc.max_rel_err(out.cpu().numpy(), ref) <= TOL_SJLT


def test_runtime_argument_errors(grass):
    g = torch.zeros((4, 100), dtype=torch.float32, device=_dev())
    with pytest.raises(grass.GrassError) as e:
        grass.grass_sjlt(g, 48, 5, seed=0)                       # s does not divide k
    assert e.value.status == grass.GRASS_EINVAL
    with pytest.raises(grass.GrassError) as e:
        grass.grass_sjlt(g, 1 << 16, 1, seed=0)                  # k beyond the LDS-resident range
    assert e.value.status == grass.GRASS_EUNSUPPORTED
    empty = torch.zeros((0, 100), dtype=torch.float32, device=_dev())
    assert grass.grass_sjlt(empty, 16, 1, seed=0).shape == (0, 16)
