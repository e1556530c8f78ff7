"""GPU parity of the projected FIM, its damped inverse and the inverse-FIM-vector product against the CPU
oracle, through the C ABI.

Bars: the FIM is an fp32 MFMA product, 1e-5 of the largest magnitude of each row.  The damped inverse is
factorised in fp64 and rounded to fp32 once, so it matches the fp64 oracle inverse of the *same* fp32 F to
2^-24 relative plus cond * 1e-13.  The iFVP multiplies fp32 G by the fp32-rounded W with fp32 accumulation:
every output obeys |got - exact| <= 1e-5 * sum_c |g_c| |w_c| (2^-24 from rounding W, the rest accumulation).
"""
import numpy as np
import pytest
import torch

import synth
from oracle import grass_oracle as orc

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def grass():
    import paper_2505_18976_amd as g
    g.load_library()
    return g


def _dev():
    return torch.device("cuda:0")


@pytest.mark.parametrize("N,k", [(50, 7), (300, 130), (1000, 256), (9000, 300), (20000, 512), (17, 64), (8192, 128),
                                 (40000, 384), (2100, 640),
                                 # 16-byte aligned rows take G itself as both K-major operands: row counts that are not
                                 # whole slices or groups (zero-filled k-rows), a ragged column tile, a single row
                                 (33, 128), (1, 128), (4100, 132), (65, 260), (70001, 256)])
def test_fim_parity(grass, N, k):
    G = synth.compressed_gradients(N, k, seed=2000 + k, device=_dev())
    F = grass.grass_fim(G)
    torch.cuda.synchronize()
    assert torch.equal(F, F.T)
    ref = orc.fim(G.cpu().numpy())
    assert orc.max_rel_err(F.cpu().numpy(), ref) <= 1e-5


def test_fim_respects_leading_dimensions(grass):
    N, k = 700, 200
    big = synth.compressed_gradients(N, 260, seed=2100, device=_dev())
    G = big[:, 4:4 + k]                                   # ld 260, base 16-byte aligned
    out = torch.full((k, 300), 7.0, dtype=torch.float32, device=_dev())
    grass.grass_fim(G, out=out[:, :k])
    torch.cuda.synchronize()
    assert orc.max_rel_err(out[:, :k].cpu().numpy(), orc.fim(G.cpu().numpy())) <= 1e-5
    assert torch.all(out[:, k:] == 7.0)


@pytest.mark.parametrize("N,k,ld", [(1000, 576, 577), (1510, 576, 579), (1000, 300, 301), (2020, 1100, 1101), (16390, 576, 577)])
def test_fim_short_inputs_with_unaligned_rows(grass, N, k, ld):
    """Rows that are not 16-byte aligned go through transposed chunks; a first chunk too short for all the K ranges the
    workspace was laid out for must only sum the partial products it wrote (row counts just below a multiple of 512 are
    the case), and a short last chunk after a full one adds to a subset of them."""
    big = synth.compressed_gradients(N, ld, seed=2200 + k, device=_dev())
    G = big[:, :k]
    F = grass.grass_fim(G)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(F).all()) and torch.equal(F, F.T)
    assert orc.max_rel_err(F.cpu().numpy(), orc.fim(G.cpu().numpy())) <= 1e-5


def _inverse_case(k, lam, seed, N=None):
    N = N or 2 * k + 3
    G = synth.compressed_gradients(N, k, seed=seed, device="cpu").numpy().astype(np.float64)
    F32 = torch.from_numpy(orc.fim(G).astype(np.float32))
    F64 = F32.numpy().astype(np.float64)
    F64 = np.tril(F64) + np.tril(F64, -1).T               # the library reads the lower triangle
    A = F64 + lam * np.eye(k)
    return F32, A


@pytest.mark.parametrize("k,lam", [(5, 0.1), (64, 1e-3), (100, 0.1), (128, 10.0), (192, 1e-2), (320, 1e-3),
                                   (448, 0.1), (576, 1e-2), (1000, 1e-2), (1024, 1e-4), (1100, 1e-3), (2048, 1e-3)])
def test_fim_inverse_parity(grass, k, lam):
    F32, A = _inverse_case(k, lam, seed=2200 + k)
    info = torch.full((1,), -1, dtype=torch.int32, device=_dev())
    W = grass.grass_fim_inverse(F32.to(_dev()), lam, info=info)
    torch.cuda.synchronize()
    assert int(info.item()) == 0
    ref = np.linalg.inv(A)
    cond = np.linalg.cond(A)
    got = W.cpu().numpy().astype(np.float64)
    assert np.array_equal(got, got.T)
    assert orc.max_rel_err(got, ref) <= 2.0 ** -23 + cond * 1e-13
    # and it is an inverse: A W = I to fp32 rounding of W times the condition of the product
    resid = np.abs(A @ got - np.eye(k)).max()
    assert resid <= 2.0 ** -23 * (np.abs(A) @ np.abs(ref)).max()


def test_fim_inverse_rank_deficient_fim_needs_the_damping(grass):
    """N < k: F is singular, (F + lam I) is not; the Woodbury closed form is the reference."""
    N, k, lam = 40, 256, 0.05
    G = synth.compressed_gradients(N, k, seed=2300, device="cpu").numpy().astype(np.float64)
    F32 = torch.from_numpy(orc.fim(G).astype(np.float32))
    W = grass.grass_fim_inverse(F32.to(_dev()), lam)
    torch.cuda.synchronize()
    F64 = np.tril(F32.numpy().astype(np.float64)); F64 = F64 + np.tril(F64, -1).T
    ref = np.linalg.inv(F64 + lam * np.eye(k))
    assert orc.max_rel_err(W.cpu().numpy(), ref) <= 1e-6


def test_fim_inverse_reports_a_non_positive_pivot(grass):
    k = 130
    F = -torch.eye(k, dtype=torch.float32, device=_dev())
    F[:70, :70] = torch.eye(70, device=_dev())
    info = torch.zeros(1, dtype=torch.int32, device=_dev())
    grass.grass_fim_inverse(F, 0.5, info=info)            # 1.5 on the first 70 pivots, -0.5 from the 71st
    torch.cuda.synchronize()
    assert int(info.item()) == 71


@pytest.mark.parametrize("N,k,lam", [(33, 64, 0.1), (500, 200, 1e-2), (3000, 512, 1e-3), (300, 1000, 0.1)])
def test_ifvp_parity(grass, N, k, lam):
    G = synth.compressed_gradients(N, k, seed=2400 + k, device=_dev())
    F = grass.grass_fim(G)
    W = grass.grass_fim_inverse(F, lam)
    out = grass.grass_ifvp(G, W)
    torch.cuda.synchronize()
    Gh = G.cpu().numpy().astype(np.float64)
    Fh = F.cpu().numpy().astype(np.float64)
    ref = orc.ifvp(Gh, Fh, lam)                            # same fp32 F handed to the oracle as data
    Wref = np.linalg.inv(Fh + lam * np.eye(k))
    bound = 1e-5 * (np.abs(Gh) @ np.abs(Wref)) + 1e-30
    assert np.all(np.abs(out.cpu().numpy() - ref) <= bound)
    # end to end from the gradients alone (the FIM's own fp32 rounding enters, amplified by the conditioning)
    full = orc.ifvp(Gh, orc.fim(Gh), lam)
    cond = np.linalg.cond(orc.fim(Gh) + lam * np.eye(k))
    assert orc.max_rel_err(out.cpu().numpy(), full) <= 1e-5 + cond * 2e-7


def test_influence_scores_end_to_end(grass):
    """Sec. 2.1: I(z_i, z_test) = <g_test, (F + lam I)^{-1} g_i>, all four calls chained on the GPU."""
    N, M, k, lam = 2048, 64, 256, 1e-2
    train = synth.compressed_gradients(N, k, seed=2500, device=_dev())
    test = synth.compressed_gradients(M, k, seed=2501, device=_dev())
    F = grass.grass_fim(train)
    W = grass.grass_fim_inverse(F, lam)
    pre = grass.grass_ifvp(train, W)
    scores = grass.grass_score(pre, test, compute_mode=0)
    torch.cuda.synchronize()
    ref = orc.influence(train.cpu().numpy(), test.cpu().numpy(), lam)
    assert scores.shape == (M, N)
    assert orc.max_rel_err(scores.cpu().numpy(), ref) <= 1e-4


def test_attribution_pass_from_raw_gradients(grass):
    """The README pipeline: Random Mask + SJLT (fused), FIM, damped inverse, iFVP, scores -- against the oracle chain."""
    n, m, p, kp, k, lam = 300, 20, 20000, 4000, 128, 1e-2
    g_train = synth.bernoulli_sparse_normal(n, p, 0.5, 1.0, seed=2600, device=_dev())
    g_test = synth.bernoulli_sparse_normal(m, p, 0.5, 1.0, seed=2601, device=_dev())
    idx = grass.grass_mask_indices(seed=0, stream_id=0, p=p, kprime=kp, device=_dev())
    train = grass.grass_sjlt(g_train, k, 1, seed=0, stream_id=1, idx=idx)
    test = grass.grass_sjlt(g_test, k, 1, seed=0, stream_id=1, idx=idx)
    W = grass.grass_fim_inverse(grass.grass_fim(train), lam)
    score = grass.grass_score(grass.grass_ifvp(train, W), test)
    torch.cuda.synchronize()
    idx_h = orc.mask_indices(0, 0, p, kp)
    tr = orc.grass(g_train.cpu().numpy(), idx_h, k, 1, 0)
    te = orc.grass(g_test.cpu().numpy(), idx_h, k, 1, 0)
    ref = orc.influence(tr, te, lam)
    assert score.shape == (m, n)
    assert orc.max_rel_err(score.cpu().numpy(), ref) <= 1e-4


def test_fim_and_ifvp_argument_checks(grass):
    G = synth.compressed_gradients(8, 16, seed=1, device=_dev())
    F = grass.grass_fim(G)
    with pytest.raises(grass.GrassError):
        grass.grass_fim_inverse(F, -1.0)
    with pytest.raises(grass.GrassError):
        grass.grass_fim_inverse(F, float("nan"))
    with pytest.raises(grass.GrassError):
        grass.grass_fim(G, ws=torch.empty(256, dtype=torch.uint8, device=_dev()))
    with pytest.raises(grass.GrassError):
        grass.grass_fim_inverse(F, 0.1, ws=torch.empty(256, dtype=torch.uint8, device=_dev()))
