"""Seeded random-shape sweeps of the GEMM-backed entry points against the CPU oracle, through the C ABI.

The fixed cases of the other GPU tests sit on the boundaries their authors thought of; host-side planning (tile shape,
number of K ranges, chunking, alignment classes) has more of them.  Every case here draws its sizes, row distances and
alignments from lists that straddle those decisions - in particular row counts on both sides of the multiples of 512
at which the FIM of rows that are not 16-byte aligned changes its number of K ranges - and is compared with the oracle
at the bars of the fixed tests."""
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


def _h(t):
    return t.float().cpu().numpy().astype(np.float64)


def _view(rows, cols, pad, seed, std=1.0):
    """rows x cols view of a (cols + pad)-wide matrix: pad decides the alignment class of the rows."""
    return synth.dense_normal(rows, cols + pad, seed=seed, device=_dev(), std=std)[:, :cols]


@pytest.mark.parametrize("seed", range(4))
def test_score_random_shapes(grass, seed):
    rng = np.random.default_rng(9000 + seed)
    pick = lambda o: int(o[rng.integers(len(o))])
    for case in range(12):
        M = pick([1, 3, 64, 100, 127, 128, 129, 200, 256, 257, 300, 384, 385, 513])
        N = pick([1, 5, 100, 128, 383, 384, 385, 700, 768, 1000, 2048, 4099])
        K = pick([1, 7, 16, 32, 48, 64, 96, 100, 512, 1040, 4096, 4112, 8200, 16384])
        tr, te = _view(N, K, pick([0, 0, 4, 8, 1, 16]), 9100 + 50 * seed + case), _view(M, K, pick([0, 0, 4, 8, 3]), 9500 + 50 * seed + case)
        ref0 = orc.score(_h(tr), _h(te))
        ref1 = orc.score(_h(tr.bfloat16()), _h(te.bfloat16()))
        for mode, ref in ((0, ref0), (1, ref1)):
            for ws in (True, None):
                out = grass.grass_score(tr, te, compute_mode=mode, ws=ws)
                torch.cuda.synchronize()
                assert np.abs(_h(out) - ref).max() <= 2e-5 * max(np.abs(ref).max(), 1e-30), (seed, case, M, N, K, mode, ws)
        if K % 8 == 0:
            trb, teb = grass.grass_to_bf16(tr.contiguous()), grass.grass_to_bf16(te.contiguous())
            out = grass.grass_score_bf16(trb, teb)
            torch.cuda.synchronize()
            assert torch.equal(trb.float(), tr.bfloat16().float()) and np.abs(_h(out) - ref1).max() <= 2e-5 * max(np.abs(ref1).max(), 1e-30)


@pytest.mark.parametrize("seed", range(4))
def test_fim_inverse_ifvp_random_shapes(grass, seed):
    rng = np.random.default_rng(9200 + seed)
    pick = lambda o: int(o[rng.integers(len(o))])
    for case in range(10):
        k = pick([1, 5, 63, 64, 65, 128, 200, 256, 300, 511, 512, 513, 576, 640, 1000, 1024, 1100])
        N = pick([1, 7, 100, 500, 511, 513, 1000, 1010, 1024, 1030, 1500, 1515, 1536, 2040, 4099, 10000])
        G = _view(N, k, pick([0, 0, 4, 1, 2]), 9300 + 50 * seed + case)
        F = grass.grass_fim(G)
        torch.cuda.synchronize()
        assert bool(torch.isfinite(F).all()) and torch.equal(F, F.T), (seed, case, N, k)
        assert orc.max_rel_err(F.cpu().numpy(), orc.fim(G.cpu().numpy())) <= 1e-5, (seed, case, N, k)
        Fh = _h(F)
        lam = 0.05 * float(np.diag(Fh).mean()) + 1e-3
        info = torch.full((1,), -1, dtype=torch.int32, device=_dev())
        W = grass.grass_fim_inverse(F, lam, info=info)
        torch.cuda.synchronize()
        A = Fh + lam * np.eye(k)
        refW = np.linalg.inv(A)
        assert int(info.item()) == 0 and torch.equal(W, W.T)
        assert orc.max_rel_err(_h(W), refW) <= 2.0 ** -23 + np.linalg.cond(A) * 1e-13, (seed, case, N, k)
        X = grass.grass_ifvp(G, W)
        torch.cuda.synchronize()
        Gh, Wh = _h(G), _h(W)
        assert np.all(np.abs(_h(X) - Gh @ Wh) <= 1e-5 * (np.abs(Gh) @ np.abs(Wh)) + 1e-30), (seed, case, N, k)


@pytest.mark.parametrize("seed", range(3))
def test_selective_mask_step_random_shapes(grass, seed):
    rng = np.random.default_rng(9400 + seed)
    pick = lambda o: int(o[rng.integers(len(o))])
    for case in range(6):
        n = pick([2, 9, 64, 130, 131, 160, 200, 300])
        m = pick([1, 3, 100, 127, 128, 129, 256, 260, 300])
        p = pick([7, 333, 4096, 4098, 4100, 5004, 8200])
        G = _view(n, p, pick([0, 0, 1, 2, 4]), 9600 + 50 * seed + case)
        Gt = synth.dense_normal(m, p, seed=9700 + 50 * seed + case, device=_dev())
        S = synth.dense_normal(1, p, seed=9800 + 50 * seed + case, device=_dev(), std=0.5).reshape(-1).contiguous()
        lam, temp = 1e-3, float(pick([1, 2])) / 2 + 0.5
        A = grass.grass_score(G, Gt)
        grad, obj = grass.grass_selective_mask_grad(G, Gt, A, S, lam, temp)
        torch.cuda.synchronize()
        want_obj = orc.selective_mask_objective(_h(S), _h(G), _h(Gt), lam, temp)
        want_grad = orc.selective_mask_gradient(_h(S), _h(G), _h(Gt), lam, temp)
        assert abs(float(obj.item()) - want_obj) <= 1e-5 * max(1.0, abs(want_obj)), (seed, case, n, m, p)
        assert np.abs(_h(grad) - want_grad).max() <= 2e-4 * np.abs(want_grad).max(), (seed, case, n, m, p)
