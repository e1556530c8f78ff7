"""GPU parity of the Selective Mask objective, gradient and index extraction against the CPU oracle.

Tolerance of the gradient: both contractions are fp32 MFMA products and the row c_t is a difference of two nearly
parallel vectors when the correlation is high (relative amplification about 1 / (1 - corr^2)); the test problems
keep the correlations away from 1 and the bar is 2e-4 of the largest gradient entry (observed up to 5e-6).  The objective
is a mean of correlations of order 1: absolute 1e-5.  Index extraction is bit-exact.
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


def _problem(n, m, p, seed, pad=0):
    G = synth.bernoulli_sparse_normal(n, p + pad, 0.4, 1.0, seed=seed, device=_dev())[:, :p]
    Gt = synth.bernoulli_sparse_normal(m, p + pad, 0.4, 1.0, seed=seed + 1, device=_dev())[:, :p]
    S = synth.dense_normal(1, p, seed=seed + 2, device=_dev(), std=1.5).reshape(-1).contiguous()
    return G, Gt, S


@pytest.mark.parametrize("n,m,p,lam,temp,pad", [(9, 3, 7, 0.03, 1.0, 0), (50, 5, 333, 0.01, 1.0, 1),
                                                (200, 130, 4096, 1e-3, 0.5, 0), (300, 140, 5002, 1e-4, 2.0, 2),
                                                (130, 129, 70000, 1e-5, 1.0, 0),
                                                # 16-byte aligned rows: the backward product reads G in place
                                                (131, 128, 70004, 1e-5, 1.0, 0), (77, 260, 4098, 1e-3, 1.0, 2),
                                                # 128 or 257..384 test rows: tiles of 128 rows in both products
                                                (160, 128, 4352, 1e-3, 1.0, 0), (90, 300, 8200, 1e-3, 0.7, 0)])
def test_selective_mask_grad_parity(grass, n, m, p, lam, temp, pad):
    G, Gt, S = _problem(n, m, p, seed=3000 + p, pad=pad)
    A = grass.grass_score(G, Gt, compute_mode=0)
    grad, obj = grass.grass_selective_mask_grad(G, Gt, A, S, lam, temp)
    torch.cuda.synchronize()
    Gh, Gth, Sh = G.cpu().numpy(), Gt.cpu().numpy(), S.cpu().numpy()
    want_obj = orc.selective_mask_objective(Sh, Gh, Gth, lam, temp)
    want_grad = orc.selective_mask_gradient(Sh, Gh, Gth, lam, temp)
    assert abs(float(obj.item()) - want_obj) <= 1e-5 * max(1.0, abs(want_obj))
    got = grad.cpu().numpy().astype(np.float64)
    assert np.abs(got - want_grad).max() <= 2e-4 * np.abs(want_grad).max()


def test_selective_mask_grad_column_chunks_aligned_and_unaligned_rows_agree(grass):
    """66,000 train rows make the backward product run over two column chunks.  The oracle would need minutes for this
    size, so the two GPU routes are held against each other instead: rows 16-byte aligned (G read in place as a
    K-major operand) and the same values stored with an odd row distance (transposed chunks, register-staged forward
    product), each route oracle-checked at smaller sizes above.  They differ only in fp32 summation order."""
    n, m, p, lam = 66000, 128, 5000, 1e-4
    G, Gt, S = _problem(n, m, p, seed=3900)                                   # row distance 5,000
    G2 = torch.empty((n, p + 1), dtype=torch.float32, device=_dev())[:, :p]
    G2.copy_(G)                                                               # row distance 5,001
    A = grass.grass_score(G, Gt, compute_mode=0)
    g1, o1 = grass.grass_selective_mask_grad(G, Gt, A, S, lam, 1.0)
    g2, o2 = grass.grass_selective_mask_grad(G2, Gt, A, S, lam, 1.0)
    torch.cuda.synchronize()
    assert abs(float(o1.item()) - float(o2.item())) <= 1e-6
    a, b = g1.cpu().numpy().astype(np.float64), g2.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(a)) and np.abs(a).max() > 0
    assert np.abs(a - b).max() <= 2e-5 * np.abs(b).max()


def test_selective_mask_grad_constant_logits_and_degenerate_rows(grass):
    """Constant logits: corr = 1 for every test row, the objective is 1 - lambda p sigma.  A test row of zeros has
    constant scores: it contributes nothing (the oracle would divide by zero, the library defines it as 0)."""
    n, m, p, lam = 40, 6, 500, 0.002
    G, Gt, _ = _problem(n, m, p, seed=3100)
    S = torch.full((p,), 0.7, dtype=torch.float32, device=_dev())
    A = grass.grass_score(G, Gt, compute_mode=0)
    _, obj = grass.grass_selective_mask_grad(G, Gt, A, S, lam)
    torch.cuda.synchronize()
    sig = 1 / (1 + np.exp(-0.7))
    assert abs(float(obj.item()) - (1.0 - lam * p * sig)) <= 1e-5
    Gt2 = Gt.clone(); Gt2[2] = 0.0
    S2 = synth.dense_normal(1, p, seed=3101, device=_dev()).reshape(-1).contiguous()
    A2 = grass.grass_score(G, Gt2, compute_mode=0)
    grad, obj = grass.grass_selective_mask_grad(G, Gt2, A2, S2, lam)
    torch.cuda.synchronize()
    keep = [0, 1, 3, 4, 5]
    Gh, Gth, Sh = G.cpu().numpy(), Gt2.cpu().numpy()[keep], S2.cpu().numpy()
    # mean over 6 rows with one zero contribution = 5/6 of the mean over the 5 proper rows (penalty unchanged)
    pen = lam * (1 / (1 + np.exp(-Sh.astype(np.float64)))).sum()
    want_obj = (orc.selective_mask_objective(Sh, Gh, Gth, 0.0) * 5 / 6) - pen
    assert abs(float(obj.item()) - want_obj) <= 1e-5
    want_grad = orc.selective_mask_gradient(Sh, Gh, Gth, 0.0) * 5 / 6 + orc.selective_mask_gradient(Sh, Gh, Gth, lam) \
        - orc.selective_mask_gradient(Sh, Gh, Gth, 0.0)
    assert np.abs(grad.cpu().numpy() - want_grad).max() <= 2e-3 * np.abs(want_grad).max()
    assert torch.isfinite(grad).all()


def test_selective_mask_ascent_step_improves_the_objective(grass):
    n, m, p, lam = 64, 16, 2048, 1e-4
    G, Gt, S = _problem(n, m, p, seed=3200)
    A = grass.grass_score(G, Gt, compute_mode=0)
    grad, obj0 = grass.grass_selective_mask_grad(G, Gt, A, S, lam)
    step = 0.5 / float(grad.abs().max().item())
    _, obj1 = grass.grass_selective_mask_grad(G, Gt, A, (S + step * grad).contiguous(), lam)
    torch.cuda.synchronize()
    assert float(obj1.item()) > float(obj0.item())


@pytest.mark.parametrize("n,m,d_in,d_out,lam,temp", [(8, 3, 5, 4, 0.05, 1.0), (60, 7, 300, 129, 0.01, 0.7),
                                                      (200, 130, 1024, 4096, 1e-3, 1.0), (150, 129, 2050, 513, 1e-4, 2.0)])
def test_selective_mask_factorized_parity(grass, n, m, d_in, d_out, lam, temp):
    """App. B.4 "Linear Layer": Kronecker gradients, factor masks; the layer gradient (d_in * d_out wide) is never formed."""
    Z_in = synth.dense_normal(n, d_in, seed=3600, device=_dev())
    Z_out = synth.dense_normal(n, d_out, seed=3601, device=_dev())
    Zt_in = synth.dense_normal(m, d_in, seed=3602, device=_dev())
    Zt_out = synth.dense_normal(m, d_out, seed=3603, device=_dev())
    S_in = synth.dense_normal(1, d_in, seed=3604, device=_dev(), std=1.5).reshape(-1).contiguous()
    S_out = synth.dense_normal(1, d_out, seed=3605, device=_dev(), std=1.5).reshape(-1).contiguous()
    A = (grass.grass_score(Z_in, Zt_in) * grass.grass_score(Z_out, Zt_out)).contiguous()
    gi, go, obj = grass.grass_selective_mask_grad_factorized(Z_in, Z_out, Zt_in, Zt_out, A, S_in, S_out, lam, temp)
    torch.cuda.synchronize()
    h = lambda t: t.cpu().numpy()
    want_obj, want_gi, want_go = orc.selective_mask_factorized(h(S_in), h(S_out), h(Z_in), h(Z_out), h(Zt_in), h(Zt_out),
                                                               lam, temp)
    assert abs(float(obj.item()) - want_obj) <= 1e-5 * max(1.0, abs(want_obj))
    assert np.abs(h(gi) - want_gi).max() <= 2e-4 * np.abs(want_gi).max()
    assert np.abs(h(go) - want_go).max() <= 2e-4 * np.abs(want_go).max()
    assert torch.isfinite(gi).all() and torch.isfinite(go).all()


@pytest.mark.parametrize("p,k", [(1, 0), (1, 1), (10, 0), (10, 3), (5000, 0), (5000, 1234), (100003, 0), (100003, 4096),
                                 (100003, 100003)])
def test_selective_mask_indices_bit_exact(grass, p, k):
    S = synth.dense_normal(1, p, seed=3300 + p, device=_dev()).reshape(-1).contiguous()
    S[::7] = 0.25                                   # ties
    S[3::11] = 0.0
    S[5::13] = -0.0
    idx = grass.grass_selective_mask_indices(S, k)
    torch.cuda.synchronize()
    want = orc.selective_mask_indices(S.cpu().numpy(), None if k == 0 else k)
    assert idx.dtype == torch.int32
    assert np.array_equal(idx.cpu().numpy(), want)


def test_selective_mask_indices_feed_the_fused_kernel(grass):
    """The extracted indices are a mask like any other: GraSS with them equals the oracle's."""
    n, p, k = 6, 20000, 256
    G, _, S = _problem(n, 1, p, seed=3400)
    idx = grass.grass_selective_mask_indices(S, 2048)
    out = grass.grass_sjlt(G, k, 1, seed=0, stream_id=1, idx=idx)
    torch.cuda.synchronize()
    ref = orc.grass(G.cpu().numpy(), orc.selective_mask_indices(S.cpu().numpy(), 2048), k, 1, 0)
    assert orc.max_rel_err(out.cpu().numpy(), ref) <= 1e-5


def test_selective_mask_argument_checks(grass):
    G, Gt, S = _problem(8, 2, 16, seed=3500)
    A = grass.grass_score(G, Gt, compute_mode=0)
    with pytest.raises(grass.GrassError):
        grass.grass_selective_mask_grad(G, Gt, A, S, -1.0)
    with pytest.raises(grass.GrassError):
        grass.grass_selective_mask_grad(G, Gt, A, S, 0.1, temperature=0.0)
    with pytest.raises(grass.GrassError):
        grass.grass_selective_mask_grad(G[:1], Gt, A[:, :1], S, 0.1)      # n = 1: no correlation
    with pytest.raises(grass.GrassError):
        grass.grass_selective_mask_indices(S, 17)


# ------------------------------------------------------------------ training (Sec. 3.2 Eq. (1) by gradient ascent)
def _oracle_path(S0, Gh, Gth, lam, lr, temps):
    """The oracle's training run, one step at a time, with the length of the path the logits travelled."""
    S, hist, path = np.asarray(S0, np.float64), [], 0.0
    for T in temps:
        nxt, h = orc.selective_mask_train(S, Gh, Gth, lam, lr, [T])
        path += np.abs(nxt - S).max()
        hist.append(h[0])
        S = nxt
    return S, np.asarray(hist), path


@pytest.mark.parametrize("n,m,p,lam,lr,steps,pad", [(60, 5, 333, 0.01, 3.0, 12, 1), (300, 130, 4096, 1e-3, 40.0, 25, 0),
                                                    (140, 128, 5004, 1e-4, 60.0, 10, 0)])
def test_selective_mask_train_parity(grass, n, m, p, lam, lr, steps, pad):
    """S after `steps` device-side steps against the oracle's loop.  Every step adds lr * grad with the gradient bar
    of 2e-4 of its largest entry, so the logits may drift apart by 2e-4 of the path length (plus fp32 rounding of S)."""
    G, Gt, S0 = _problem(n, m, p, seed=3300 + p, pad=pad)
    S0 = (0.2 * S0).contiguous()
    temps = np.geomspace(1.0, 0.4, steps)
    A = grass.grass_score(G, Gt, compute_mode=0)
    S = S0.clone()
    _, objs = grass.grass_selective_mask_train(G, Gt, A, S, lam, lr, temps)
    torch.cuda.synchronize()
    want, hist, path = _oracle_path(S0.cpu().numpy(), G.cpu().numpy(), Gt.cpu().numpy(), lam, lr, temps)
    got = S.cpu().numpy().astype(np.float64)
    assert path > 0 and np.abs(want - S0.cpu().numpy()).max() > 10 * 2e-4 * path       # the run really moved the logits
    assert np.abs(got - want).max() <= 2e-4 * path + steps * 2.0 ** -23 * np.abs(want).max()
    assert np.abs(objs.cpu().numpy() - hist).max() <= 1e-5 * max(1.0, np.abs(hist).max())
    # the same run as separate calls of the gradient entry point and a host-side update gives the same logits
    S2 = S0.clone()
    for T in temps:
        grad, _ = grass.grass_selective_mask_grad(G, Gt, A, S2, lam, float(T))
        S2 = (S2.double() + lr * grad.double()).float()
    torch.cuda.synchronize()
    assert torch.equal(S2, S)


def test_selective_mask_train_recovers_planted_coordinates_and_beats_random_mask(grass):
    """End to end on gradients with planted informative coordinates: device training, extraction (exact k and plain
    threshold), and the first term of Eq. (1) for the resulting binary mask against a Random Mask of the same size."""
    n, m, p, kept, lam, lr = 512, 32, 4096, 128, 3e-4, 300.0
    G, Gt, planted = synth.planted_gradients(n, m, p, kept, seed=3400, device=_dev())
    S0 = synth.dense_normal(1, p, seed=3401, device=_dev(), std=0.1).reshape(-1).contiguous()
    temps = np.geomspace(1.0, 0.6, 60)       # mild annealing: saturated logits make the run sensitive to rounding
    A = grass.grass_score(G, Gt, compute_mode=0)
    S = S0.clone()
    _, objs = grass.grass_selective_mask_train(G, Gt, A, S, lam, lr, temps)
    idx_k = grass.grass_selective_mask_indices(S, kept)
    idx_thr = grass.grass_selective_mask_indices(S)
    torch.cuda.synchronize()
    Gh, Gth = G.cpu().numpy(), Gt.cpu().numpy()
    want_S, hist = orc.selective_mask_train(S0.cpu().numpy(), Gh, Gth, lam, lr, temps)
    want_idx = orc.selective_mask_indices(want_S, kept)
    planted_h = planted.numpy().astype(np.int32)
    assert np.array_equal(want_idx, planted_h)                       # the oracle's run finds the planted set ...
    gap = want_S[planted_h].min() - np.delete(want_S, planted_h).max()
    assert gap > 100 * np.abs(S.cpu().numpy() - want_S).max()        # ... with a margin far above the GPU's deviation,
    assert np.array_equal(idx_k.cpu().numpy(), want_idx)             # so the extracted indices must agree bit for bit
    assert np.array_equal(idx_thr.cpu().numpy(), orc.selective_mask_indices(want_S))
    assert objs[-1].item() > objs[0].item()

    def masked_correlation(idx):
        Y = grass.grass_score(grass.grass_mask(G, idx), grass.grass_mask(Gt, idx), compute_mode=0)
        return float(grass.grass_score_correlation(A, Y).item())

    c_sel = masked_correlation(idx_k)
    assert abs(c_sel - orc.graddot_correlation(Gh, Gth, want_idx)) <= 1e-5
    c_rand = []
    for seed in range(5):
        ridx = grass.grass_mask_indices(seed, 0, p, kept, device=_dev())
        c = masked_correlation(ridx)
        assert abs(c - orc.graddot_correlation(Gh, Gth, ridx.cpu().numpy())) <= 1e-5
        c_rand.append(c)
    assert c_sel > 0.9 and c_sel > max(c_rand) + 0.2


def test_selective_mask_train_edge_cases(grass):
    G, Gt, S0 = _problem(20, 3, 50, seed=3500)
    A = grass.grass_score(G, Gt, compute_mode=0)
    S = S0.clone()
    grass.grass_selective_mask_train(G, Gt, A, S, 0.01, 1.0, [])     # no steps: nothing happens
    torch.cuda.synchronize()
    assert torch.equal(S, S0)
    grass.grass_selective_mask_train(G, Gt, A, S, 0.01, 0.0, [1.0, 0.5])   # zero step size: logits stay
    torch.cuda.synchronize()
    assert torch.equal(S, S0)
    for bad in ([1.0, 0.0], [-1.0], [float("nan")]):
        with pytest.raises(grass.GrassError):
            grass.grass_selective_mask_train(G, Gt, A, S, 0.01, 1.0, bad)
    with pytest.raises(grass.GrassError):
        grass.grass_selective_mask_train(G, Gt, A, S, -0.01, 1.0, [1.0])
    with pytest.raises(grass.GrassError):
        grass.grass_selective_mask_train(G, Gt, A, S, 0.01, 1.0, [1.0], ws=torch.empty(256, dtype=torch.uint8, device=_dev()))
    torch.cuda.synchronize()
    assert torch.equal(S, S0)                                       # refused calls did nothing


def test_score_correlation_parity(grass):
    from scipy import stats
    m, n = 37, 1000
    X = synth.dense_normal(m, n, seed=3600, device=_dev())
    Y = (0.6 * X + synth.dense_normal(m, n, seed=3601, device=_dev()))[:, :n].contiguous()
    Y[5] = 2.0                                                       # a constant row contributes 0
    got = float(grass.grass_score_correlation(X, Y).item())
    Xh, Yh = X.cpu().numpy().astype(np.float64), Y.cpu().numpy().astype(np.float64)
    want = sum(stats.pearsonr(Xh[t], Yh[t])[0] for t in range(m) if t != 5) / m
    assert abs(got - want) <= 1e-6


# ------------------------------------------------------------------- factorised training (App. B.4 "Linear Layer")
def _factor_problem(n, m, d_in, d_out, seed):
    Z_in = synth.dense_normal(n, d_in, seed=seed, device=_dev())
    Z_out = synth.dense_normal(n, d_out, seed=seed + 1, device=_dev())
    Zt_in = synth.dense_normal(m, d_in, seed=seed + 2, device=_dev())
    Zt_out = synth.dense_normal(m, d_out, seed=seed + 3, device=_dev())
    S_in = synth.dense_normal(1, d_in, seed=seed + 4, device=_dev(), std=0.3).reshape(-1).contiguous()
    S_out = synth.dense_normal(1, d_out, seed=seed + 5, device=_dev(), std=0.3).reshape(-1).contiguous()
    return Z_in, Z_out, Zt_in, Zt_out, S_in, S_out


@pytest.mark.parametrize("n,m,d_in,d_out,lam,lr,steps", [(8, 3, 5, 4, 0.05, 0.5, 6), (60, 7, 300, 129, 0.01, 2.0, 12),
                                                         (200, 130, 1024, 2050, 1e-3, 20.0, 10)])
def test_selective_mask_train_factorized_parity(grass, n, m, d_in, d_out, lam, lr, steps):
    """Both logit vectors after `steps` device-side steps against the oracle's loop, with the drift bound of the plain
    training test (2e-4 of each vector's path length plus fp32 rounding of the logits), and bit for bit against the
    same run made of separate calls of the factorised gradient entry point with a host-side update."""
    Z_in, Z_out, Zt_in, Zt_out, S_in0, S_out0 = _factor_problem(n, m, d_in, d_out, seed=3800 + d_in)
    temps = np.geomspace(1.0, 0.5, steps)
    A = (grass.grass_score(Z_in, Zt_in) * grass.grass_score(Z_out, Zt_out)).contiguous()
    S_in, S_out = S_in0.clone(), S_out0.clone()
    _, _, objs = grass.grass_selective_mask_train_factorized(Z_in, Z_out, Zt_in, Zt_out, A, S_in, S_out, lam, lr, temps)
    torch.cuda.synchronize()
    h = lambda t: t.cpu().numpy().astype(np.float64)
    # the oracle's loop, step by step, to get the path lengths as well
    a, b = h(S_in0), h(S_out0)
    path_in = path_out = 0.0
    hist = []
    for T in temps:
        a2, b2, h1 = orc.selective_mask_train_factorized(a, b, h(Z_in), h(Z_out), h(Zt_in), h(Zt_out), lam, lr, [T])
        path_in += np.abs(a2 - a).max(); path_out += np.abs(b2 - b).max()
        hist.append(h1[0]); a, b = a2, b2
    whole = orc.selective_mask_train_factorized(h(S_in0), h(S_out0), h(Z_in), h(Z_out), h(Zt_in), h(Zt_out), lam, lr, temps)
    assert np.array_equal(whole[0], a) and np.array_equal(whole[1], b)
    assert np.abs(a - h(S_in0)).max() > 10 * 2e-4 * path_in and np.abs(b - h(S_out0)).max() > 10 * 2e-4 * path_out
    assert np.abs(h(S_in) - a).max() <= 2e-4 * path_in + steps * 2.0 ** -23 * np.abs(a).max()
    assert np.abs(h(S_out) - b).max() <= 2e-4 * path_out + steps * 2.0 ** -23 * np.abs(b).max()
    assert np.abs(objs.cpu().numpy() - np.asarray(hist)).max() <= 1e-5 * max(1.0, np.abs(hist).max())
    T_in, T_out = S_in0.clone(), S_out0.clone()
    for T in temps:
        gi, go, _ = grass.grass_selective_mask_grad_factorized(Z_in, Z_out, Zt_in, Zt_out, A, T_in, T_out, lam, float(T))
        T_in = (T_in.double() + lr * gi.double()).float()
        T_out = (T_out.double() + lr * go.double()).float()
    torch.cuda.synchronize()
    assert torch.equal(T_in, S_in) and torch.equal(T_out, S_out)


def test_selective_mask_train_factorized_recovers_the_planted_coordinates_of_both_factors(grass):
    n, m, d_in, d_out, k_in, k_out, lam, lr = 256, 32, 512, 384, 16, 12, 1e-3, 100.0
    Z_in, Zt_in, p_in = synth.planted_gradients(n, m, d_in, k_in, seed=3700, device=_dev())
    Z_out, Zt_out, p_out = synth.planted_gradients(n, m, d_out, k_out, seed=3701, device=_dev())
    S_in0 = synth.dense_normal(1, d_in, seed=3702, device=_dev(), std=0.1).reshape(-1).contiguous()
    S_out0 = synth.dense_normal(1, d_out, seed=3703, device=_dev(), std=0.1).reshape(-1).contiguous()
    temps = np.geomspace(1.0, 0.6, 60)
    A = (grass.grass_score(Z_in, Zt_in) * grass.grass_score(Z_out, Zt_out)).contiguous()
    S_in, S_out = S_in0.clone(), S_out0.clone()
    _, _, objs = grass.grass_selective_mask_train_factorized(Z_in, Z_out, Zt_in, Zt_out, A, S_in, S_out, lam, lr, temps)
    ii = grass.grass_selective_mask_indices(S_in, k_in)
    io = grass.grass_selective_mask_indices(S_out, k_out)
    torch.cuda.synchronize()
    h = lambda t: t.cpu().numpy().astype(np.float64)
    a, b, hist = orc.selective_mask_train_factorized(h(S_in0), h(S_out0), h(Z_in), h(Z_out), h(Zt_in), h(Zt_out), lam, lr, temps)
    pi, po = p_in.numpy().astype(np.int32), p_out.numpy().astype(np.int32)
    assert np.array_equal(orc.selective_mask_indices(a, k_in), pi) and np.array_equal(orc.selective_mask_indices(b, k_out), po)
    gap = min(a[pi].min() - np.delete(a, pi).max(), b[po].min() - np.delete(b, po).max())
    assert gap > 100 * max(np.abs(h(S_in) - a).max(), np.abs(h(S_out) - b).max())
    assert np.array_equal(ii.cpu().numpy(), pi) and np.array_equal(io.cpu().numpy(), po)
    assert objs[-1].item() > objs[0].item()

    # first term of Eq. (1) for the binary Kronecker mask, from factor scores: <a (x) b, c (x) d> = <a, c> <b, d>
    def masked_correlation(ji, jo):
        Y = grass.grass_score(grass.grass_mask(Z_in, ji), grass.grass_mask(Zt_in, ji)) * \
            grass.grass_score(grass.grass_mask(Z_out, jo), grass.grass_mask(Zt_out, jo))
        return float(grass.grass_score_correlation(A, Y.contiguous()).item())
    c_sel = masked_correlation(ii, io)
    c_rand = [masked_correlation(grass.grass_mask_indices(sd, 0, d_in, k_in, device=_dev()),
                                 grass.grass_mask_indices(sd, 1, d_out, k_out, device=_dev())) for sd in range(5)]
    assert c_sel > 0.9 and c_sel > max(c_rand) + 0.2


def test_selective_mask_train_factorized_edge_cases(grass):
    Z_in, Z_out, Zt_in, Zt_out, S_in0, S_out0 = _factor_problem(20, 3, 50, 30, seed=3900)
    A = (grass.grass_score(Z_in, Zt_in) * grass.grass_score(Z_out, Zt_out)).contiguous()
    S_in, S_out = S_in0.clone(), S_out0.clone()
    grass.grass_selective_mask_train_factorized(Z_in, Z_out, Zt_in, Zt_out, A, S_in, S_out, 0.01, 1.0, [])
    grass.grass_selective_mask_train_factorized(Z_in, Z_out, Zt_in, Zt_out, A, S_in, S_out, 0.01, 0.0, [1.0, 0.5])
    for bad in ([1.0, 0.0], [-1.0], [float("nan")]):
        with pytest.raises(grass.GrassError):
            grass.grass_selective_mask_train_factorized(Z_in, Z_out, Zt_in, Zt_out, A, S_in, S_out, 0.01, 1.0, bad)
    with pytest.raises(grass.GrassError):
        grass.grass_selective_mask_train_factorized(Z_in, Z_out, Zt_in, Zt_out, A, S_in, S_out, -0.01, 1.0, [1.0])
    torch.cuda.synchronize()
    assert torch.equal(S_in, S_in0) and torch.equal(S_out, S_out0)


# ------------------------------------------------------------------- factorised form on sequences of tokens
def _seq_tensors(n, T, m, Tt, d_in, d_out, seed):
    def t(rows, tok, d, sd):
        return synth.dense_normal(rows * tok, d, seed=sd, device=_dev()).reshape(rows, tok, d)
    return (t(n, T, d_in, seed), t(n, T, d_out, seed + 1), t(m, Tt, d_in, seed + 2), t(m, Tt, d_out, seed + 3),
            synth.dense_normal(1, d_in, seed=seed + 4, device=_dev(), std=1.0).reshape(-1).contiguous(),
            synth.dense_normal(1, d_out, seed=seed + 5, device=_dev(), std=1.0).reshape(-1).contiguous())


@pytest.mark.parametrize("n,T,m,Tt,d_in,d_out,lam,temp", [(6, 3, 2, 2, 5, 4, 0.05, 1.0), (20, 7, 5, 9, 70, 33, 0.01, 0.7),
                                                          (40, 16, 9, 16, 260, 129, 1e-3, 1.0), (130, 2, 129, 1, 64, 512, 1e-3, 2.0)])
def test_selective_mask_factorized_sequences_parity(grass, n, T, m, Tt, d_in, d_out, lam, temp):
    """Exact scores and the factorised objective / gradients for samples of T (train) and Tt (test) tokens: the token
    sum of Eq. (2) inside the Kronecker inner products of App. B.4; the layer gradients are never formed."""
    Z_in, Z_out, Zt_in, Zt_out, S_in, S_out = _seq_tensors(n, T, m, Tt, d_in, d_out, seed=4000 + d_in)
    h = lambda t: t.cpu().numpy().astype(np.float64)
    A = grass.grass_graddot_factorized(Z_in, Z_out, Zt_in, Zt_out)
    torch.cuda.synchronize()
    want_A = orc.graddot_factorized_seq(h(Z_in), h(Z_out), h(Zt_in), h(Zt_out))
    assert orc.max_rel_err(h(A), want_A) <= 1e-5
    gi, go, obj = grass.grass_selective_mask_grad_factorized_seq(Z_in, Z_out, Zt_in, Zt_out, A, S_in, S_out, lam, temp)
    torch.cuda.synchronize()
    want_obj, want_gi, want_go = orc.selective_mask_factorized_seq(h(S_in), h(S_out), h(Z_in), h(Z_out), h(Zt_in), h(Zt_out),
                                                                   lam, temp)
    assert abs(float(obj.item()) - want_obj) <= 1e-5 * max(1.0, abs(want_obj))
    assert np.abs(h(gi) - want_gi).max() <= 2e-4 * np.abs(want_gi).max()
    assert np.abs(h(go) - want_go).max() <= 2e-4 * np.abs(want_go).max()
    assert torch.isfinite(gi).all() and torch.isfinite(go).all()


def test_selective_mask_factorized_sequences_of_one_token_are_the_single_token_entry_point(grass):
    n, m, d_in, d_out = 60, 7, 300, 129
    Z_in, Z_out, Zt_in, Zt_out, S_in, S_out = _seq_tensors(n, 1, m, 1, d_in, d_out, seed=4100)
    A = grass.grass_graddot_factorized(Z_in, Z_out, Zt_in, Zt_out)
    A1 = (grass.grass_score(Z_in[:, 0], Zt_in[:, 0]) * grass.grass_score(Z_out[:, 0], Zt_out[:, 0])).contiguous()
    a = grass.grass_selective_mask_grad_factorized_seq(Z_in, Z_out, Zt_in, Zt_out, A, S_in, S_out, 0.01, 0.7)
    b = grass.grass_selective_mask_grad_factorized(Z_in[:, 0], Z_out[:, 0], Zt_in[:, 0], Zt_out[:, 0], A, S_in, S_out, 0.01, 0.7)
    torch.cuda.synchronize()
    assert orc.max_rel_err(A.cpu().numpy(), A1.cpu().numpy().astype(np.float64)) <= 1e-5
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1]) and torch.equal(a[2], b[2])


def test_selective_mask_factorized_sequences_argument_checks(grass):
    Z_in, Z_out, Zt_in, Zt_out, S_in, S_out = _seq_tensors(4, 3, 2, 2, 8, 6, seed=4200)
    A = grass.grass_graddot_factorized(Z_in, Z_out, Zt_in, Zt_out)
    with pytest.raises(grass.GrassError):
        grass.grass_selective_mask_grad_factorized_seq(Z_in, Z_out, Zt_in, Zt_out, A, S_in, S_out, -1.0, 1.0)
    with pytest.raises(grass.GrassError):
        grass.grass_selective_mask_grad_factorized_seq(Z_in, Z_out, Zt_in, Zt_out, A, S_in, S_out, 0.1, 0.0)
    with pytest.raises(grass.GrassError):       # one train sample: no correlation over the train rows
        grass.grass_graddot_factorized(Z_in[:1], Z_out[:1], Zt_in, Zt_out)
    # the scores land in the first n columns of the caller's rows and nowhere else
    wide = torch.full((2, 9), -7.0, dtype=torch.float32, device=_dev())
    grass.grass_graddot_factorized(Z_in, Z_out, Zt_in, Zt_out, out=wide[:, :4])
    torch.cuda.synchronize()
    assert torch.equal(wide[:, :4], A) and bool((wide[:, 4:] == -7.0).all())


@pytest.mark.parametrize("n,T,m,Tt,d_in,d_out,lam,lr,steps", [(6, 3, 2, 2, 5, 4, 0.05, 0.05, 5), (20, 7, 5, 9, 70, 33, 0.01, 0.02, 8),
                                                              (40, 16, 9, 16, 260, 129, 1e-3, 0.01, 6)])
def test_selective_mask_train_factorized_sequences_parity(grass, n, T, m, Tt, d_in, d_out, lam, lr, steps):
    """The device-side training loop on sequences against the oracle's loop (drift bound of the other training tests),
    and bit for bit against separate calls of the sequence gradient entry point with a host-side update."""
    Z_in, Z_out, Zt_in, Zt_out, S_in0, S_out0 = _seq_tensors(n, T, m, Tt, d_in, d_out, seed=4300 + d_in)
    S_in0, S_out0 = (0.3 * S_in0).contiguous(), (0.3 * S_out0).contiguous()
    temps = np.geomspace(1.0, 0.5, steps)
    A = grass.grass_graddot_factorized(Z_in, Z_out, Zt_in, Zt_out)
    S_in, S_out = S_in0.clone(), S_out0.clone()
    _, _, objs = grass.grass_selective_mask_train_factorized_seq(Z_in, Z_out, Zt_in, Zt_out, A, S_in, S_out, lam, lr, temps)
    torch.cuda.synchronize()
    h = lambda t: t.cpu().numpy().astype(np.float64)
    a, b = h(S_in0), h(S_out0)
    path_in = path_out = 0.0
    hist = []
    for Tm in temps:
        a2, b2, h1 = orc.selective_mask_train_factorized_seq(a, b, h(Z_in), h(Z_out), h(Zt_in), h(Zt_out), lam, lr, [Tm])
        path_in += np.abs(a2 - a).max(); path_out += np.abs(b2 - b).max()
        hist.append(h1[0]); a, b = a2, b2
    assert np.abs(a - h(S_in0)).max() > 10 * 2e-4 * path_in and np.abs(b - h(S_out0)).max() > 10 * 2e-4 * path_out
    assert np.abs(h(S_in) - a).max() <= 2e-4 * path_in + steps * 2.0 ** -23 * np.abs(a).max()
    assert np.abs(h(S_out) - b).max() <= 2e-4 * path_out + steps * 2.0 ** -23 * np.abs(b).max()
    assert np.abs(objs.cpu().numpy() - np.asarray(hist)).max() <= 1e-5 * max(1.0, np.abs(hist).max())
    T_in, T_out = S_in0.clone(), S_out0.clone()
    for Tm in temps:
        gi, go, _ = grass.grass_selective_mask_grad_factorized_seq(Z_in, Z_out, Zt_in, Zt_out, A, T_in, T_out, lam, float(Tm))
        T_in = (T_in.double() + lr * gi.double()).float()
        T_out = (T_out.double() + lr * go.double()).float()
    torch.cuda.synchronize()
    assert torch.equal(T_in, S_in) and torch.equal(T_out, S_out)


def test_selective_mask_train_factorized_sequences_of_one_token_and_edge_cases(grass):
    n, m, d_in, d_out = 60, 7, 300, 129
    Z_in, Z_out, Zt_in, Zt_out, S_in0, S_out0 = _seq_tensors(n, 1, m, 1, d_in, d_out, seed=4400)
    A = grass.grass_graddot_factorized(Z_in, Z_out, Zt_in, Zt_out)
    temps = [1.0, 0.8, 0.6]
    a_in, a_out = S_in0.clone(), S_out0.clone()
    _, _, oa = grass.grass_selective_mask_train_factorized_seq(Z_in, Z_out, Zt_in, Zt_out, A, a_in, a_out, 0.01, 0.5, temps)
    b_in, b_out = S_in0.clone(), S_out0.clone()
    _, _, ob = grass.grass_selective_mask_train_factorized(Z_in[:, 0], Z_out[:, 0], Zt_in[:, 0], Zt_out[:, 0], A, b_in, b_out,
                                                           0.01, 0.5, temps)
    torch.cuda.synchronize()
    assert torch.equal(a_in, b_in) and torch.equal(a_out, b_out) and torch.equal(oa, ob)
    assert not torch.equal(a_in, S_in0) and not torch.equal(a_out, S_out0)
    # no steps: nothing moves; a non-positive temperature anywhere in the schedule is refused before any launch
    c_in, c_out = S_in0.clone(), S_out0.clone()
    grass.grass_selective_mask_train_factorized_seq(Z_in, Z_out, Zt_in, Zt_out, A, c_in, c_out, 0.01, 0.5, [])
    with pytest.raises(grass.GrassError):
        grass.grass_selective_mask_train_factorized_seq(Z_in, Z_out, Zt_in, Zt_out, A, c_in, c_out, 0.01, 0.5, [1.0, 0.0])
    with pytest.raises(grass.GrassError):
        grass.grass_selective_mask_train_factorized_seq(Z_in, Z_out, Zt_in, Zt_out, A, c_in, c_out, -0.01, 0.5, [1.0])
    torch.cuda.synchronize()
    assert torch.equal(c_in, S_in0) and torch.equal(c_out, S_out0)
